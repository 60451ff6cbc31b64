"""Seeded synthetic inputs: model shapes, random-init weights, look-ahead embeddings, prompts.

This module is the only thing the CPU oracle's tests and the HIP path share.  It holds no
arithmetic of the method (no transformer math, no sampling): it draws normal / uniform values
from NumPy's counter-based Philox bit generator, scales them, and converts storage formats.
Both sides receive the same byte buffers.

The paper evaluates a re-implemented LLaMA-7B loaded in bfloat16 on text corpora that are not
available here (Experiments section; Training details).  The shapes below stand in for those
workloads: same tensor shapes, dtype, context lengths and batch raggedness; random values.
"""
from __future__ import annotations

import concurrent.futures as _cf
import os as _os
from dataclasses import dataclass, field, replace

import numpy as np

F32 = 0
BF16 = 1

# sub-streams of one config seed
_STREAM_WEIGHTS = 0
_STREAM_LOOKAHEAD = 1
_STREAM_PROMPTS = 2
_STREAM_SAMPLING = 3


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: int = BF16  # storage type of every tensor of the model

    @property
    def n_params_streamed(self) -> int:
        """Parameters one decode step reads: all layer matrices and gains, final gain, LM head."""
        d, f = self.d_model, self.d_ffn
        per_layer = 4 * d * d + 3 * d * f + 2 * d
        return self.n_layers * per_layer + d + d * self.vocab


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    seed: int
    k: int                      # number of look-ahead embeddings (L in Algorithm 1)
    batch: int
    prompt_len: tuple           # (lo, hi) inclusive; lo == hi for a fixed length
    max_new: int
    temperature: float          # 0 = greedy
    lm_head_scale: float = 1.0
    k_sweep: tuple = field(default_factory=tuple)


_TINY = ModelShape(2, 256, 4, 64, 688, 512, dtype=F32)
_7B = ModelShape(32, 4096, 32, 128, 11008, 32000, dtype=BF16)
_13B = ModelShape(40, 5120, 40, 128, 13824, 32000, dtype=BF16)

WORKLOADS = {
    # the five configurations of the build's baseline file, in its order
    "tiny_fp32_greedy": Workload("tiny_fp32_greedy", _TINY, 0, 2, 1, (16, 16), 64, 0.0, 8.0),
    "tiny_fp32_t1": Workload("tiny_fp32_t1", _TINY, 0, 2, 1, (16, 16), 64, 1.0, 8.0),
    "7b_k4_greedy": Workload("7b_k4_greedy", _7B, 1, 4, 1, (512, 512), 256, 0.0, 4.0),
    "7b_ksweep_t0.8": Workload("7b_ksweep_t0.8", _7B, 2, 4, 1, (2048, 2048), 256, 0.8, 4.0,
                               k_sweep=(0, 1, 2, 3, 4, 6)),
    "7b_b8_ragged_t1": Workload("7b_b8_ragged_t1", _7B, 3, 4, 8, (128, 2048), 128, 1.0, 4.0),
    "13b_k4_t0.8": Workload("13b_k4_t0.8", _13B, 4, 4, 1, (4096, 4096), 256, 0.8, 1.0),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (fewer layers, shorter prompt...)."""
    shape_keys = {f for f in ModelShape.__dataclass_fields__}
    skw = {k: v for k, v in kw.items() if k in shape_keys}
    wkw = {k: v for k, v in kw.items() if k not in shape_keys}
    shape = replace(w.shape, **skw) if skw else w.shape
    return replace(w, shape=shape, **wkw)


# ----------------------------------------------------------------------------------------------
# storage-format helpers
# ----------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of float32 to bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | stream, tensor]))


_CHUNK = 1 << 22


def _normal_tensor(seed, stream, tensor_id, shape, std, dtype):
    """N(0, std) tensor from its own Philox stream; float32 or bfloat16 bit patterns."""
    n = int(np.prod(shape))
    g = _rng(seed, stream, tensor_id)
    out = np.empty(n, dtype=np.float32 if dtype == F32 else np.uint16)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        x = g.standard_normal(hi - lo, dtype=np.float32)
        x *= np.float32(std)
        out[lo:hi] = x if dtype == F32 else f32_to_bf16_bits(x)
    return out.reshape(shape)


def _ones(shape, dtype):
    if dtype == F32:
        return np.ones(shape, dtype=np.float32)
    return np.full(shape, 0x3F80, dtype=np.uint16)


def make_weights(shape: ModelShape, seed: int, k: int, lm_head_scale: float = 1.0,
                 std: float = 0.02, threads: int | None = None) -> dict:
    """Random-init model.  Matrices and embeddings N(0, std); norm gains 1; LM head scaled.

    Matrices are [out_features, in_features] row-major.  Returns a dict:
      tok_emb [V,d], lm_head [V,d], final_norm [d], lookahead [k,d],
      and per-layer lists attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down.
    """
    s = shape
    d, f, v, hd = s.d_model, s.d_ffn, s.vocab, s.n_heads * s.head_dim
    jobs = {}  # name -> (tensor_id, shape, std)
    tid = 0

    def add(name, shp, sd):
        nonlocal tid
        jobs[name] = (tid, shp, sd)
        tid += 1

    add("tok_emb", (v, d), std)
    add("lm_head", (v, d), std * lm_head_scale)
    for l in range(s.n_layers):
        add(f"wq.{l}", (hd, d), std)
        add(f"wk.{l}", (hd, d), std)
        add(f"wv.{l}", (hd, d), std)
        add(f"wo.{l}", (d, hd), std)
        add(f"w_gate.{l}", (f, d), std)
        add(f"w_up.{l}", (f, d), std)
        add(f"w_down.{l}", (d, f), std)

    threads = threads or min(16, _os.cpu_count() or 1)
    res = {}
    with _cf.ThreadPoolExecutor(max_workers=threads) as ex:
        futs = {name: ex.submit(_normal_tensor, seed, _STREAM_WEIGHTS, t, shp, sd, s.dtype)
                for name, (t, shp, sd) in jobs.items()}
        for name, fu in futs.items():
            res[name] = fu.result()

    out = {
        "tok_emb": res["tok_emb"],
        "lm_head": res["lm_head"],
        "final_norm": _ones((d,), s.dtype),
        "lookahead": _normal_tensor(seed, _STREAM_LOOKAHEAD, 0, (max(k, 1), d), std, s.dtype)[:k],
    }
    for key in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        out[key] = [res[f"{key}.{l}"] for l in range(s.n_layers)]
    out["attn_norm"] = [_ones((d,), s.dtype) for _ in range(s.n_layers)]
    out["ffn_norm"] = [_ones((d,), s.dtype) for _ in range(s.n_layers)]
    return out


def make_prompts(w: Workload) -> list:
    """Uniform-random token ids; ragged lengths uniform in [lo, hi] when lo < hi."""
    g = _rng(w.seed, _STREAM_PROMPTS, 0)
    lo, hi = w.prompt_len
    lens = [lo] * w.batch if lo == hi else [int(x) for x in g.integers(lo, hi + 1, size=w.batch)]
    return [g.integers(0, w.shape.vocab, size=n).astype(np.int32) for n in lens]


def sampling_seed(w: Workload) -> int:
    """64-bit seed of the sampling RNG for this workload."""
    g = _rng(w.seed, _STREAM_SAMPLING, 0)
    return int(g.integers(0, 2 ** 63 - 1))


def random_logits(seed: int, rows: int, vocab: int, scale: float = 3.0) -> np.ndarray:
    """Synthetic fp32 logits for sampler tests: N(0, scale)."""
    g = _rng(seed, 7, 0)
    return (g.standard_normal((rows, vocab), dtype=np.float32) * np.float32(scale)).astype(np.float32)
