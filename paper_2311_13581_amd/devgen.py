"""Random-init model generated directly in device memory (torch generator), for runs that need no
CPU-side copy of the weights: the benchmark and the full-size property tests.  Same recipe as
`synth.make_weights` (matrices and embeddings N(0, 0.02), LM head scaled, gains 1), different stream."""
from __future__ import annotations


def device_weights(shape, k: int, lm_head_scale: float, seed: int) -> dict:
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    dt = torch.bfloat16 if shape.dtype == 1 else torch.float32

    def normal(rows, cols, scale=1.0):
        return (torch.randn(rows, cols, generator=g, device="cuda", dtype=torch.float32) * (0.02 * scale)).to(dt)

    d, f, v, hd = shape.d_model, shape.d_ffn, shape.vocab, shape.n_heads * shape.head_dim
    ones = torch.ones(d, device="cuda", dtype=dt)
    W = {"tok_emb": normal(v, d), "lm_head": normal(v, d, lm_head_scale), "final_norm": ones,
         "lookahead": normal(max(k, 1), d)[:k].contiguous()}
    for name, (r, c) in {"wq": (hd, d), "wk": (hd, d), "wv": (hd, d), "wo": (d, hd), "w_gate": (f, d),
                         "w_up": (f, d), "w_down": (d, f)}.items():
        W[name] = [normal(r, c) for _ in range(shape.n_layers)]
    W["attn_norm"] = [ones] * shape.n_layers
    W["ffn_norm"] = [ones] * shape.n_layers
    return W
