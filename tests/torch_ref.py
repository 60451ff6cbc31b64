"""Independent fp64 reference of a LLaMA-style forward built from PyTorch library routines.

Used only to pin the CPU oracle: no KV cache (the whole sequence is recomputed), attention through
torch.nn.functional.scaled_dot_product_attention, rotary embedding through complex multiplication.
"""
import numpy as np
import torch
import torch.nn.functional as F

from paper_2311_13581_amd import synth


def to_t(a, dtype):
    if dtype == synth.BF16:
        a = synth.bf16_bits_to_f32(a)
    return torch.from_numpy(np.ascontiguousarray(a)).double()


def forward_full(shape, W, ids, n_la):
    """Logits [len(ids)+n_la, V] (fp64) of the sequence ids followed by look-ahead rows 0..n_la-1."""
    dt = shape.dtype
    x = to_t(W["tok_emb"], dt)[torch.as_tensor(np.asarray(ids), dtype=torch.long)]
    if n_la:
        x = torch.cat([x, to_t(W["lookahead"], dt)[:n_la]], 0)
    T, H, hd = x.shape[0], shape.n_heads, shape.head_dim
    inv = 1.0 / (shape.rope_base ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    ang = torch.outer(torch.arange(T, dtype=torch.float64), inv)
    rot = torch.polar(torch.ones_like(ang), ang)  # [T, hd/2] complex

    def rope(t):  # t [T, H, hd]
        c = torch.view_as_complex(t.reshape(T, H, hd // 2, 2).contiguous())
        return torch.view_as_real(c * rot[:, None, :]).reshape(T, H, hd)

    def norm(t, g):
        return F.rms_norm(t, (t.shape[-1],), to_t(g, dt), eps=shape.rms_eps)

    for l in range(shape.n_layers):
        n1 = norm(x, W["attn_norm"][l])
        q = rope(F.linear(n1, to_t(W["wq"][l], dt)).view(T, H, hd))
        k = rope(F.linear(n1, to_t(W["wk"][l], dt)).view(T, H, hd))
        v = F.linear(n1, to_t(W["wv"][l], dt)).view(T, H, hd)
        if dt == synth.BF16:  # the K/V cache of a bf16 model stores bf16 values (rounded once, from fp64)
            k = k.to(torch.bfloat16).double()
            v = v.to(torch.bfloat16).double()
        a = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0]
        x = x + F.linear(a.transpose(0, 1).reshape(T, H * hd), to_t(W["wo"][l], dt))
        n2 = norm(x, W["ffn_norm"][l])
        x = x + F.linear(F.silu(F.linear(n2, to_t(W["w_gate"][l], dt))) * F.linear(n2, to_t(W["w_up"][l], dt)),
                         to_t(W["w_down"][l], dt))
    return F.linear(norm(x, W["final_norm"]), to_t(W["lm_head"], dt))
