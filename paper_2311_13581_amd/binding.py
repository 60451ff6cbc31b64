"""Thin ctypes binding of libpass_hip.so (include/pass.h).  Argument marshalling only.

PyTorch supplies device memory (the arena) and the HIP stream; every step of the decode path runs
in the library's kernels.  There is no CPU fallback: a missing library or GPU raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpass_hip.so")

PASS_F32, PASS_BF16 = 0, 1
MAX_K, MAX_ROWS = 15, 64

SYMBOLS = ["pass_arena_bytes", "pass_create", "pass_load_weights", "pass_prefill", "pass_prefill_batch", "pass_release",
           "pass_draft", "pass_draft_static", "pass_verify", "pass_generate", "pass_sps_iteration", "pass_run_iterations", "pass_kernel_time", "pass_plain_read", "pass_rng_uniforms", "pass_get_logits", "pass_seq_len",
           "pass_train_bytes", "pass_train_begin", "pass_train_step", "pass_train_read", "pass_train_resume", "pass_set_option", "pass_attention_plan", "pass_prefill_plan", "pass_get_tokens", "pass_time_step", "pass_last_error", "pass_destroy"]


class PassConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32),
                ("k", C.c_int32), ("max_slots", C.c_int32), ("max_seq_len", C.c_int32),
                ("page_size", C.c_int32), ("n_pages", C.c_int32)]


class PassSampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_k", C.c_int32), ("seed", C.c_uint64)]


class PassStats(C.Structure):
    _fields_ = [("iterations", C.c_int64), ("drafts_proposed", C.c_int64), ("drafts_accepted", C.c_int64),
                ("tokens_out", C.c_int64), ("draft_ms", C.c_double), ("verify_ms", C.c_double)]


_PP = C.POINTER(C.c_void_p)


class PassWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("lookahead", C.c_void_p),
                ("attn_norm", _PP), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP),
                ("ffn_norm", _PP), ("w_gate", _PP), ("w_up", _PP), ("w_down", _PP)]


class PassAdamW(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


class PassError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"pass error {code}: {msg}")
        self.code = code


_lib = None


def load_library():
    """Load libpass_hip.so (built by paper_2311_13581_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built: run `python -m paper_2311_13581_amd.build` "
                                "(there is no fallback path)")
    # PyTorch ships its own HIP runtime under the same soname as the system one; whichever is
    # loaded first serves the whole process.  Import torch first so that the arena it allocates
    # and the kernels launched here share one runtime.
    import torch  # noqa: F401
    L = C.CDLL(path)
    ip = C.POINTER(C.c_int32)
    L.pass_arena_bytes.restype = C.c_size_t
    L.pass_arena_bytes.argtypes = [C.POINTER(PassConfig)]
    L.pass_create.argtypes = [C.POINTER(PassConfig), C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]
    L.pass_load_weights.argtypes = [C.c_void_p, C.POINTER(PassWeights), C.c_int]
    L.pass_prefill.argtypes = [C.c_void_p, C.c_int, C.c_uint32, ip, C.c_int]
    L.pass_prefill_batch.argtypes = [C.c_void_p, ip, C.POINTER(C.c_uint32), ip, ip, C.c_int]
    L.pass_release.argtypes = [C.c_void_p, C.c_int]
    L.pass_draft.argtypes = [C.c_void_p, ip, C.c_int, C.POINTER(PassSampling), ip, ip]
    L.pass_draft_static.argtypes = [C.c_void_p, ip, C.c_int, C.POINTER(PassSampling), ip, ip]
    L.pass_verify.argtypes = [C.c_void_p, ip, C.c_int, C.POINTER(PassSampling), ip, ip]
    L.pass_generate.argtypes = [C.c_void_p, ip, C.c_int, C.c_int, C.POINTER(PassSampling), ip, C.POINTER(PassStats)]
    L.pass_sps_iteration.argtypes = [C.c_void_p, C.c_void_p, ip, ip, C.c_int, C.POINTER(PassSampling), ip, ip, ip]
    L.pass_run_iterations.argtypes = [C.c_void_p, ip, C.c_int, C.c_int, C.POINTER(PassSampling), C.POINTER(PassStats)]
    L.pass_kernel_time.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.pass_plain_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_double)]
    L.pass_rng_uniforms.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                    C.c_size_t, C.POINTER(C.c_float)]
    L.pass_get_logits.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_float)]
    L.pass_seq_len.argtypes = [C.c_void_p, C.c_int, ip, ip]
    L.pass_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int]
    L.pass_train_bytes.restype = C.c_size_t
    L.pass_train_bytes.argtypes = [C.c_void_p]
    L.pass_train_begin.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32]
    L.pass_train_step.argtypes = [C.c_void_p, ip, C.c_int, ip, C.POINTER(PassAdamW), C.POINTER(C.c_float)]
    L.pass_train_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_float)]
    L.pass_train_resume.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_int64]
    L.pass_get_tokens.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, ip]
    L.pass_attention_plan.argtypes = [C.c_int, C.c_int, ip, ip, ip]
    L.pass_prefill_plan.argtypes = [C.c_int, ip, C.c_int, C.c_int, ip, ip]
    L.pass_time_step.argtypes = [C.c_void_p, ip, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double)]
    L.pass_last_error.restype = C.c_char_p
    L.pass_last_error.argtypes = [C.c_void_p]
    L.pass_destroy.argtypes = [C.c_void_p]
    _lib = L
    return L


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def make_config(shape, k, max_slots, max_seq_len, page_size=64, n_pages=0) -> PassConfig:
    return PassConfig(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                      shape.rms_eps, shape.rope_base, shape.dtype, k, max_slots, max_seq_len, page_size, n_pages)


class Pass:
    """One model instance on the current CUDA(HIP) device.  Methods mirror the C entry points."""

    def __init__(self, cfg: PassConfig, options: dict | None = None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the PaSS decode path has no CPU fallback")
        self._torch = torch
        self.lib = load_library()
        self.cfg = cfg
        self.k = cfg.k
        self.vocab = cfg.vocab
        nbytes = self.lib.pass_arena_bytes(C.byref(cfg))
        if nbytes == 0:
            raise PassError(-1, "configuration not supported")
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        base = (self.arena.data_ptr() + 255) & ~255
        # a stream of the library's own (default priority): the null stream cannot be captured into
        # HIP graphs.  Everything torch produced for us is complete before the library touches it.
        self.stream = torch.cuda.Stream()
        torch.cuda.synchronize()
        h = C.c_void_p()
        rc = self.lib.pass_create(C.byref(cfg), C.c_void_p(self.stream.cuda_stream), C.c_void_p(base), nbytes,
                                  C.byref(h))
        if rc != 0:
            raise PassError(rc, self.lib.pass_last_error(None).decode())
        self.h = h
        for name, val in (options or {}).items():
            self.set_option(name, val)

    def _check(self, rc):
        if rc != 0:
            raise PassError(rc, self.lib.pass_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            self.lib.pass_destroy(self.h)
            self.h = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, name: str, value: int):
        self._check(self.lib.pass_set_option(self.h, name.encode(), int(value)))
        if name == "lookahead_rows":
            self.k_act = int(value)  # rows 1 .. k_act of drafts / logits are live, the rest padding

    def load_weights(self, weights: dict):
        """weights: dict of numpy arrays (host) or torch CUDA tensors (device), plain layout."""
        torch = self._torch
        sample = weights["tok_emb"]
        on_device = isinstance(sample, torch.Tensor)

        def ptr(a):
            if a is None:
                return None
            if on_device:
                assert a.is_cuda and a.is_contiguous()
                return a.data_ptr()
            assert a.flags["C_CONTIGUOUS"] or a.size == 0
            return a.ctypes.data

        if on_device:
            torch.cuda.synchronize()  # tensors were produced on torch's streams
        w = PassWeights()
        keep = []
        for name in ("tok_emb", "lm_head", "final_norm"):
            setattr(w, name, ptr(weights[name]))
        w.lookahead = ptr(weights["lookahead"]) if self.k > 0 else None
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            lst = weights[name]
            arr = (C.c_void_p * len(lst))(*[ptr(a) for a in lst])
            keep.append(arr)
            setattr(w, name, C.cast(arr, _PP))
        self._check(self.lib.pass_load_weights(self.h, C.byref(w), int(on_device)))

    def prefill(self, slot: int, prompt, seq_id: int = 0):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        self._check(self.lib.pass_prefill(self.h, slot, seq_id, _ip(p), p.size))

    def prefill_batch(self, slots, prompts, seq_ids=None):
        s = np.ascontiguousarray(slots, dtype=np.int32)
        ps = [np.ascontiguousarray(p, dtype=np.int32) for p in prompts]
        lens = np.array([p.size for p in ps], dtype=np.int32)
        cat = np.ascontiguousarray(np.concatenate(ps), dtype=np.int32)
        ids = np.ascontiguousarray(s if seq_ids is None else seq_ids, dtype=np.uint32)
        self._check(self.lib.pass_prefill_batch(self.h, _ip(s), ids.ctypes.data_as(C.POINTER(C.c_uint32)), _ip(cat), _ip(lens), s.size))

    def release(self, slot: int):
        self._check(self.lib.pass_release(self.h, slot))

    def draft(self, slots, temperature: float, seed: int, top_k: int = 0, static: bool = False):
        s = np.ascontiguousarray(slots, dtype=np.int32)
        sp = PassSampling(temperature, top_k, seed)
        first = np.zeros(s.size, dtype=np.int32)
        drafts = np.zeros(max(1, s.size * self.k), dtype=np.int32)
        fn = self.lib.pass_draft_static if static else self.lib.pass_draft
        self._check(fn(self.h, _ip(s), s.size, C.byref(sp), _ip(first), _ip(drafts)))
        return first, drafts[:s.size * self.k].reshape(s.size, self.k)

    def verify(self, slots, temperature: float, seed: int, top_k: int = 0):
        s = np.ascontiguousarray(slots, dtype=np.int32)
        sp = PassSampling(temperature, top_k, seed)
        n_acc = np.zeros(s.size, dtype=np.int32)
        toks = np.zeros(s.size * (self.k + 1), dtype=np.int32)
        self._check(self.lib.pass_verify(self.h, _ip(s), s.size, C.byref(sp), _ip(n_acc), _ip(toks)))
        return n_acc, toks.reshape(s.size, self.k + 1)

    def generate(self, slots, max_new: int, temperature: float, seed: int, top_k: int = 0):
        s = np.ascontiguousarray(slots, dtype=np.int32)
        sp = PassSampling(temperature, top_k, seed)
        out = np.zeros(max(1, s.size * max_new), dtype=np.int32)
        st = PassStats()
        self._check(self.lib.pass_generate(self.h, _ip(s), s.size, max_new, C.byref(sp), _ip(out), C.byref(st)))
        stats = {f: getattr(st, f) for f, _ in PassStats._fields_}
        return out[:s.size * max_new].reshape(s.size, max_new), stats

    def sps_iteration(self, drafter: "Pass", slots, drafter_slots, temperature: float, seed: int, top_k: int = 0):
        """One iteration of two-model speculative sampling; self is the target.  Returns (drafts
        [n, k], accepted counts [n], tokens [n, k + 1])."""
        s = np.ascontiguousarray(slots, dtype=np.int32)
        ds = np.ascontiguousarray(drafter_slots, dtype=np.int32)
        assert s.size == ds.size
        sp = PassSampling(temperature, top_k, seed)
        drafts = np.zeros(max(1, s.size * self.k), dtype=np.int32)
        n_acc = np.zeros(s.size, dtype=np.int32)
        toks = np.zeros(s.size * (self.k + 1), dtype=np.int32)
        self._check(self.lib.pass_sps_iteration(self.h, drafter.h, _ip(s), _ip(ds), s.size, C.byref(sp), _ip(drafts),
                                                _ip(n_acc), _ip(toks)))
        return drafts[:s.size * self.k].reshape(s.size, self.k), n_acc, toks.reshape(s.size, self.k + 1)

    def run_iterations(self, slots, n_iters: int, temperature: float, seed: int, top_k: int = 0) -> dict:
        s = np.ascontiguousarray(slots, dtype=np.int32)
        sp = PassSampling(temperature, top_k, seed)
        st = PassStats()
        self._check(self.lib.pass_run_iterations(self.h, _ip(s), s.size, n_iters, C.byref(sp), C.byref(st)))
        return {f: getattr(st, f) for f, _ in PassStats._fields_}

    def kernel_time(self):
        ms, n = C.c_double(0), C.c_int64(0)
        self._check(self.lib.pass_kernel_time(self.h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def plain_read(self, nbytes: int, iters: int) -> float:
        us = C.c_double(0)
        self._check(self.lib.pass_plain_read(self.h, nbytes, iters, C.byref(us)))
        return us.value

    def rng_uniforms(self, seed: int, seq_id: int, iteration: int, row: int, purpose: int, first: int, n: int) -> np.ndarray:
        out = np.empty(n, dtype=np.float32)
        self._check(self.lib.pass_rng_uniforms(self.h, seed, seq_id, iteration, row, purpose, first, n,
                                               out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def get_logits(self, slot: int, which: int) -> np.ndarray:
        out = np.empty((self.k + 1, self.vocab), dtype=np.float32)
        self._check(self.lib.pass_get_logits(self.h, slot, which, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def train_begin(self, init_token: int = -1):
        """Set up look-ahead embedding training (the workspace is a torch tensor this object keeps)."""
        nbytes = self.lib.pass_train_bytes(self.h)
        if nbytes == 0:
            raise PassError(-1, "no look-ahead embeddings to train")
        self.train_ws = self._torch.empty(nbytes + 256, dtype=self._torch.uint8, device="cuda")
        self._torch.cuda.synchronize()
        base = (self.train_ws.data_ptr() + 255) & ~255
        self._check(self.lib.pass_train_begin(self.h, C.c_void_p(base), nbytes, init_token))

    def train_step(self, slots, targets, lr: float, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01) -> float:
        s = np.ascontiguousarray(slots, dtype=np.int32)
        t = np.ascontiguousarray(targets, dtype=np.int32)
        assert t.size == s.size * self.k
        opt = PassAdamW(lr, beta1, beta2, eps, weight_decay)
        loss = C.c_float(0)
        self._check(self.lib.pass_train_step(self.h, _ip(s), s.size, _ip(t), C.byref(opt), C.byref(loss)))
        return loss.value

    def train_read(self, what: int) -> np.ndarray:
        out = np.empty((self.k, self.cfg.d_model), dtype=np.float32)
        self._check(self.lib.pass_train_read(self.h, what, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def train_resume(self, master=None, m1=None, m2=None, steps: int = 0):
        keep = [None if a is None else np.ascontiguousarray(a, dtype=np.float32).reshape(self.k, self.cfg.d_model) for a in (master, m1, m2)]
        ptr = [None if a is None else a.ctypes.data_as(C.POINTER(C.c_float)) for a in keep]
        self._check(self.lib.pass_train_resume(self.h, ptr[0], ptr[1], ptr[2], steps))

    def get_tokens(self, slot: int, first: int, n: int) -> np.ndarray:
        out = np.empty(max(1, n), dtype=np.int32)
        self._check(self.lib.pass_get_tokens(self.h, slot, first, n, _ip(out)))
        return out[:n]

    def seq_len(self, slot: int):
        a, b = C.c_int32(0), C.c_int32(0)
        self._check(self.lib.pass_seq_len(self.h, slot, C.byref(a), C.byref(b)))
        return a.value, b.value

    def time_step(self, slots, warmup: int, iters: int) -> float:
        s = np.ascontiguousarray(slots, dtype=np.int32)
        ms = C.c_double(0)
        self._check(self.lib.pass_time_step(self.h, _ip(s), s.size, warmup, iters, C.byref(ms)))
        return ms.value
