"""ctypes wrapper of the CPU oracle (oracle/pass_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  It never imports the HIP package and the HIP package never imports it.
Argument marshalling only; every computation is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import sys

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, _HERE)
import build as _build  # noqa: E402  (oracle/build.py)

sys.path.pop(0)

F32, BF16 = 0, 1
DRAFT, ACCEPT, RESIDUAL, BONUS = 0, 1, 2, 3
MAX_K = 15


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32),
                ("k", C.c_int32), ("act_bf16", C.c_int32), ("la_token", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("lookahead", C.c_void_p),
                ("attn_norm", _PP), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP),
                ("ffn_norm", _PP), ("w_gate", _PP), ("w_up", _PP), ("w_down", _PP)]


class Sampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_k", C.c_int32), ("seed", C.c_uint64)]


class Ctr(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("seq_id", C.c_uint32), ("iteration", C.c_uint32),
                ("row", C.c_uint32), ("purpose", C.c_uint32)]


_lib = None
_PROGRESS = C.CFUNCTYPE(None, C.c_int, C.c_int)
_progress_keep = None


def set_progress(fn):
    """fn(rows_done, rows_total) is called after every chunk of a prompt pass; None switches it off."""
    global _progress_keep
    _progress_keep = _PROGRESS(fn) if fn else _PROGRESS(0)
    lib().orc_set_progress(_progress_keep)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        L = _lib
        L.orc_bf16_round.restype = C.c_double
        L.orc_bf16_round.argtypes = [C.c_double]
        L.orc_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
        L.orc_uniform.restype = C.c_double
        L.orc_uniform.argtypes = [C.c_uint64] + [C.c_uint32] * 5
        L.orc_uniforms.restype = None
        L.orc_uniforms.argtypes = [C.c_uint64] + [C.c_uint32] * 5 + [C.c_size_t, C.POINTER(C.c_double)]
        fp = C.POINTER(C.c_float)
        ip = C.POINTER(C.c_int32)
        L.orc_sample_softmax.argtypes = [fp, C.c_int, C.c_double, C.c_int, C.POINTER(Ctr), C.c_double, ip]
        L.orc_accept.argtypes = [fp, fp, C.c_int, C.c_int, C.c_double, C.c_int, C.POINTER(Ctr), C.c_double, ip]
        L.orc_sample_residual.argtypes = [fp, fp, C.c_int, C.c_double, C.c_int, C.POINTER(Ctr), C.c_double, ip, ip]
        L.orc_model_create.restype = C.c_void_p
        L.orc_model_create.argtypes = [C.POINTER(Config), C.POINTER(Weights)]
        L.orc_model_free.argtypes = [C.c_void_p]
        L.orc_seq_create.restype = C.c_void_p
        L.orc_seq_create.argtypes = [C.c_void_p, C.c_int, C.c_uint32]
        L.orc_seq_free.argtypes = [C.c_void_p]
        L.orc_forward.argtypes = [C.c_void_p, C.c_int, ip, ip, C.c_int, fp]
        L.orc_prefill.argtypes = [C.c_void_p, ip, C.c_int]
        L.orc_draft.argtypes = [C.c_void_p, C.POINTER(Sampling), C.c_double, ip, ip]
        L.orc_verify.argtypes = [C.c_void_p, C.POINTER(Sampling), C.c_double, ip, ip]
        L.orc_generate.argtypes = [C.c_void_p, C.c_int, C.POINTER(Sampling), C.c_double, ip, ip, ip,
                                   C.c_int, ip]
        L.orc_generate_ar.argtypes = [C.c_void_p, C.c_int, C.POINTER(Sampling), ip]
        L.orc_seq_kv_len.argtypes = [C.c_void_p]
        L.orc_seq_pending.argtypes = [C.c_void_p]
        L.orc_seq_n_generated.argtypes = [C.c_void_p]
        L.orc_seq_n_generated.restype = C.c_int64
        L.orc_seq_fallbacks.argtypes = [C.c_void_p]
        L.orc_seq_logits.argtypes = [C.c_void_p, C.c_int]
        L.orc_seq_logits.restype = fp
        L.orc_seq_decision_flags.argtypes = [C.c_void_p, ip, ip, ip]
        L.orc_seq_read_kv.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double)]
        L.orc_seq_set_pending.argtypes = [C.c_void_p, C.c_int32]
        L.orc_seq_set_draft.argtypes = [C.c_void_p, ip, fp]
        L.orc_seq_copy_state.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_sps_iteration.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(Sampling), C.c_double, ip, ip, fp]
        L.orc_generate_sps.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(Sampling), C.c_double, ip, ip, ip,
                                       C.c_int, ip]
        L.orc_set_progress.restype = None
        L.orc_set_progress.argtypes = [_PROGRESS]
    return _lib


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


# ------------------------------------------------------------------------------------------
# primitives
# ------------------------------------------------------------------------------------------
def bf16_round(x: float) -> float:
    return lib().orc_bf16_round(float(x))


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return tuple(int(v) for v in o)


def uniform(seed, seq_id, iteration, row, purpose, j) -> float:
    return lib().orc_uniform(seed, seq_id, iteration, row, purpose, j)


def uniforms(seed, seq_id, iteration, row, purpose, first, n) -> np.ndarray:
    """uniform(.., j) for j = first .. first + n - 1."""
    out = np.empty(n, dtype=np.float64)
    lib().orc_uniforms(seed, seq_id, iteration, row, purpose, first, n, out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def _ctr(seed, seq_id, iteration, row, purpose):
    return Ctr(seed, seq_id, iteration, row, purpose)


def sample_softmax(logits, temperature, seed=0, seq_id=0, iteration=0, row=0, purpose=DRAFT, tau=0.0, top_k=0):
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    st = C.c_int32(0)
    c = _ctr(seed, seq_id, iteration, row, purpose)
    tok = lib().orc_sample_softmax(_fp(logits), logits.size, temperature, top_k, C.byref(c), tau, C.byref(st))
    return tok, bool(st.value)


def accept(p_logits, d_logits, x, temperature, seed=0, seq_id=0, iteration=0, row=1, tau=0.0, top_k=0):
    p = np.ascontiguousarray(p_logits, dtype=np.float32)
    d = np.ascontiguousarray(d_logits, dtype=np.float32)
    st = C.c_int32(0)
    c = _ctr(seed, seq_id, iteration, row, ACCEPT)
    a = lib().orc_accept(_fp(p), _fp(d), p.size, int(x), temperature, top_k, C.byref(c), tau, C.byref(st))
    return bool(a), bool(st.value)


def sample_residual(p_logits, d_logits, temperature, seed=0, seq_id=0, iteration=0, row=1, tau=0.0, top_k=0):
    p = np.ascontiguousarray(p_logits, dtype=np.float32)
    d = np.ascontiguousarray(d_logits, dtype=np.float32)
    st, fb = C.c_int32(0), C.c_int32(0)
    c = _ctr(seed, seq_id, iteration, row, RESIDUAL)
    tok = lib().orc_sample_residual(_fp(p), _fp(d), p.size, temperature, top_k, C.byref(c), tau,
                                    C.byref(st), C.byref(fb))
    return tok, bool(st.value), bool(fb.value)


# ------------------------------------------------------------------------------------------
# model and sequences
# ------------------------------------------------------------------------------------------
class Model:
    """Borrowed-weights transformer.  `weights` is the dict made by the synthetic generator."""

    def __init__(self, shape, weights: dict, k: int, act_bf16: bool | None = None, la_token: int = -1):
        self.shape = shape
        self.k = k
        if act_bf16 is None:
            act_bf16 = False
        self.cfg = Config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn,
                          shape.vocab, shape.rms_eps, shape.rope_base, shape.dtype, k, int(act_bf16), int(la_token))
        self._keep = weights  # keep the numpy buffers alive
        w = Weights()
        for name in ("tok_emb", "lm_head", "final_norm", "lookahead"):
            arr = weights[name]
            assert arr.flags["C_CONTIGUOUS"] or arr.size == 0
            setattr(w, name, arr.ctypes.data)
        self._arrays = []
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            lst = weights[name]
            arr = (C.c_void_p * max(1, len(lst)))(*[a.ctypes.data for a in lst])
            self._arrays.append(arr)
            setattr(w, name, C.cast(arr, _PP))
        self._w = w
        self.handle = lib().orc_model_create(C.byref(self.cfg), C.byref(w))
        if not self.handle:
            raise RuntimeError("orc_model_create failed")

    def __del__(self):
        if getattr(self, "handle", None):
            lib().orc_model_free(self.handle)
            self.handle = None

    def sequence(self, max_len: int, seq_id: int = 0) -> "Sequence":
        return Sequence(self, max_len, seq_id)


class Sequence:
    def __init__(self, model: Model, max_len: int, seq_id: int):
        self.model = model
        self.k = model.k
        self.vocab = model.shape.vocab
        self.handle = lib().orc_seq_create(model.handle, max_len, seq_id)
        if not self.handle:
            raise RuntimeError("orc_seq_create failed")

    def __del__(self):
        if getattr(self, "handle", None):
            lib().orc_seq_free(self.handle)
            self.handle = None

    # raw model call ------------------------------------------------------------------
    def forward(self, ids, la, pos0, want_logits=True):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        la = np.ascontiguousarray(la, dtype=np.int32)
        out = np.empty((ids.size, self.vocab), dtype=np.float32) if want_logits else None
        rc = lib().orc_forward(self.handle, ids.size, _ip(ids), _ip(la), pos0,
                               _fp(out) if want_logits else None)
        _check(rc, "forward")
        return out

    # Algorithm 1 ------------------------------------------------------------------------
    def prefill(self, prompt):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        _check(lib().orc_prefill(self.handle, _ip(p), p.size), "prefill")

    def draft(self, temperature, seed, tau=0.0, top_k=0):
        sp = Sampling(temperature, top_k, seed)
        first = C.c_int32(0)
        drafts = np.zeros(max(1, self.k), dtype=np.int32)
        _check(lib().orc_draft(self.handle, C.byref(sp), tau, C.byref(first), _ip(drafts)), "draft")
        return int(first.value), drafts[:self.k].copy()

    def verify(self, temperature, seed, tau=0.0, top_k=0):
        sp = Sampling(temperature, top_k, seed)
        a = C.c_int32(0)
        toks = np.zeros(self.k + 1, dtype=np.int32)
        _check(lib().orc_verify(self.handle, C.byref(sp), tau, C.byref(a), _ip(toks)), "verify")
        return int(a.value), toks[:a.value + 1].copy()

    def generate(self, max_new, temperature, seed, tau=0.0, top_k=0):
        sp = Sampling(temperature, top_k, seed)
        out = np.zeros(max(1, max_new), dtype=np.int32)
        cap = max_new // 2 + 2
        acc = np.zeros(cap, dtype=np.int32)
        stab = np.zeros(cap, dtype=np.int32)
        iters = C.c_int32(0)
        _check(lib().orc_generate(self.handle, max_new, C.byref(sp), tau, _ip(out), _ip(acc), _ip(stab),
                                  cap, C.byref(iters)), "generate")
        n = iters.value
        return out[:max_new].copy(), acc[:n].copy(), stab[:n].astype(bool)

    # Algorithm 2 (two-model speculative sampling): self is the target ----------------------
    def sps_iteration(self, drafter: "Sequence", temperature, seed, tau=0.0, top_k=0):
        """One iteration with `drafter` (a sequence of a model with the same vocabulary holding the
        same tokens).  Returns (accepted count, tokens added, drafter logits [k, vocab])."""
        sp = Sampling(temperature, top_k, seed)
        a = C.c_int32(0)
        toks = np.zeros(self.k + 1, dtype=np.int32)
        dl = np.zeros((max(1, self.k), self.vocab), dtype=np.float32)
        _check(lib().orc_sps_iteration(self.handle, drafter.handle, C.byref(sp), tau, C.byref(a), _ip(toks), _fp(dl)),
               "sps_iteration")
        return int(a.value), toks[:a.value + 1].copy(), dl[:self.k]

    def generate_sps(self, drafter: "Sequence", max_new, temperature, seed, tau=0.0, top_k=0):
        sp = Sampling(temperature, top_k, seed)
        out = np.zeros(max(1, max_new), dtype=np.int32)
        cap = max_new + 2
        acc = np.zeros(cap, dtype=np.int32)
        stab = np.zeros(cap, dtype=np.int32)
        iters = C.c_int32(0)
        _check(lib().orc_generate_sps(self.handle, drafter.handle, max_new, C.byref(sp), tau, _ip(out), _ip(acc),
                                      _ip(stab), cap, C.byref(iters)), "generate_sps")
        n = iters.value
        return out[:max_new].copy(), acc[:n].copy(), stab[:n].astype(bool)

    def generate_ar(self, max_new, temperature, seed, top_k=0):
        sp = Sampling(temperature, top_k, seed)
        out = np.zeros(max(1, max_new), dtype=np.int32)
        _check(lib().orc_generate_ar(self.handle, max_new, C.byref(sp), _ip(out)), "generate_ar")
        return out[:max_new].copy()

    # state ------------------------------------------------------------------------------
    @property
    def kv_len(self):
        return lib().orc_seq_kv_len(self.handle)

    @property
    def pending(self):
        return lib().orc_seq_pending(self.handle)

    @property
    def n_generated(self):
        return lib().orc_seq_n_generated(self.handle)

    @property
    def fallbacks(self):
        return lib().orc_seq_fallbacks(self.handle)

    def logits(self, which):
        """Copy of the [(1+k), vocab] logits of the last draft (0) or verify (1) call."""
        p = lib().orc_seq_logits(self.handle, which)
        return np.ctypeslib.as_array(p, shape=(self.k + 1, self.vocab)).copy()

    def decision_flags(self):
        d = np.zeros(MAX_K + 1, dtype=np.int32)
        a = np.zeros(MAX_K + 1, dtype=np.int32)
        f = C.c_int32(0)
        lib().orc_seq_decision_flags(self.handle, _ip(d), _ip(a), C.byref(f))
        return d[:self.k + 1].astype(bool), a[:self.k + 1].astype(bool), bool(f.value)

    def read_kv(self, which, layer, pos):
        s = self.model.shape
        out = np.zeros(s.n_heads * s.head_dim, dtype=np.float64)
        lib().orc_seq_read_kv(self.handle, which, layer, pos, out.ctypes.data_as(C.POINTER(C.c_double)))
        return out

    def copy_state_from(self, other: "Sequence"):
        """Take over the cache, length, pending token and counters of `other` (between iterations)."""
        _check(lib().orc_seq_copy_state(self.handle, other.handle), "copy_state")

    def set_pending(self, tok):
        lib().orc_seq_set_pending(self.handle, int(tok))

    def set_draft(self, drafts, draft_logits=None):
        d = np.ascontiguousarray(drafts, dtype=np.int32)
        if draft_logits is not None:
            dl = np.ascontiguousarray(draft_logits, dtype=np.float32)
            assert dl.shape == (self.k + 1, self.vocab)
            lib().orc_seq_set_draft(self.handle, _ip(d), _fp(dl))
        else:
            lib().orc_seq_set_draft(self.handle, _ip(d), None)
