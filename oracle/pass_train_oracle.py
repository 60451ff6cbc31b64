"""CPU oracle of the look-ahead embedding training step (plain PyTorch CPU ops, fp64).

TEST INFRASTRUCTURE ONLY, like the rest of this directory: imported by tests/ (and by nothing of the
HIP package); it shares no code with the accelerated path.

What it implements, and from where (the paper's Training details and Section 2.2.1):
  - the sequence (w_1 .. w_T, [LA]_1 .. [LA]_L) goes through the frozen model in one pass; the loss is
    taken on the outputs of the look-ahead rows only: row [LA]_i predicts token w_{T+1+i} (the row of
    w_T predicts w_{T+1}, so the i-th look-ahead row looks i + 1 tokens ahead);
  - every parameter of the model is frozen; only the L x d_model look-ahead embeddings are trained;
  - AdamW (decoupled weight decay), learning rate 0.01, batches of 8 sequences, linear warm-up then
    a cosine schedule; the embeddings start from the embedding of one token ([UNK] in the paper).
The forward pass is written out with torch library ops (linear, softmax, rms norm by its formula,
rotary embedding on interleaved pairs); the gradient is torch's reverse-mode differentiation of
exactly that graph; AdamW is written out from its definition.

Readings where the paper is silent:
  - the loss is the mean cross-entropy over the look-ahead rows of the batch;
  - the trained embeddings are kept in fp32 ("master" values, fp64 here) and enter the forward pass
    unrounded; the model's own tensors keep their storage type (bfloat16 weights; K/V rows of a
    bfloat16 model are rounded when cached, and the gradient passes through that rounding unchanged);
  - AdamW's betas, epsilon and weight decay are not given: they are arguments (defaults 0.9, 0.999,
    1e-8, 0.01, the values of the optimiser's publication and of common libraries).
"""
from __future__ import annotations

import math

import numpy as np
import torch

BF16 = 1


def _t(a, dtype):
    """Model tensor (numpy; bf16 models hold uint16 bit patterns) as an fp64 torch tensor."""
    a = np.ascontiguousarray(a)
    if dtype == BF16:
        a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return torch.from_numpy(a.astype(np.float64))


def forward_logits(shape, W, prefix, la, rounding=None):
    """Logits [L, V] of the look-ahead rows for the sequence prefix + L look-ahead embeddings.
    la: [L, d] fp64 tensor (may require grad).  rounding (tests of this file's gradient only): a list
    that receives, per layer, what the cache's rounding added to K and V; handed in again, those
    amounts are added as constants instead of rounding, which makes the pass a smooth function with
    the same value and the same gradient at the point where the list was filled."""
    dt = shape.dtype
    H, hd, eps = shape.n_heads, shape.head_dim, shape.rms_eps
    x = torch.cat([_t(W["tok_emb"], dt)[torch.as_tensor(np.asarray(prefix), dtype=torch.long)], la], 0)
    T = x.shape[0]
    half = hd // 2
    theta = shape.rope_base ** (-2.0 * torch.arange(half, dtype=torch.float64) / hd)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * theta[None, :]
    cs, sn = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

    def rope(t):  # [T, H, hd], pairs (2i, 2i+1)
        a, b = t[..., 0::2], t[..., 1::2]
        return torch.stack([a * cs - b * sn, a * sn + b * cs], -1).reshape(T, H, hd)

    def norm(t, g):
        return t * torch.rsqrt((t * t).mean(-1, keepdim=True) + eps) * _t(g, dt)

    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    for l in range(shape.n_layers):
        n1 = norm(x, W["attn_norm"][l])
        q = rope((n1 @ _t(W["wq"][l], dt).T).view(T, H, hd))
        k = rope((n1 @ _t(W["wk"][l], dt).T).view(T, H, hd))
        v = (n1 @ _t(W["wv"][l], dt).T).view(T, H, hd)
        if dt == BF16:  # the cache stores bfloat16 values; gradients pass the rounding unchanged (a cast
            # node would round the gradient to bfloat16 on its way back as well)
            if rounding is not None and len(rounding) > l:
                dk, dv = rounding[l]
            else:
                dk, dv = (k.to(torch.bfloat16).double() - k).detach(), (v.to(torch.bfloat16).double() - v).detach()
                if rounding is not None:
                    rounding.append((dk, dv))
            k, v = k + dk, v + dv
        s = torch.einsum("qhd,khd->hqk", q, k) / math.sqrt(hd)
        p = torch.softmax(s.masked_fill(~mask[None], -math.inf), -1)
        a = torch.einsum("hqk,khd->qhd", p, v).reshape(T, H * hd)
        x = x + a @ _t(W["wo"][l], dt).T
        n2 = norm(x, W["ffn_norm"][l])
        g = n2 @ _t(W["w_gate"][l], dt).T
        x = x + (g * torch.sigmoid(g) * (n2 @ _t(W["w_up"][l], dt).T)) @ _t(W["w_down"][l], dt).T
    return norm(x, W["final_norm"])[len(prefix):] @ _t(W["lm_head"], dt).T


def loss_and_grad(shape, W, la, prefixes, targets, rounding=None):
    """Mean cross-entropy over the look-ahead rows of a batch, and its gradient w.r.t. the look-ahead
    embeddings.  prefixes: list of token lists (w_1 .. w_T); targets: [B, L] tokens w_{T+2} .. w_{T+1+L}.
    rounding: None, or one list per sequence (see forward_logits).
    Returns (loss float, grad [L, d] float64 numpy)."""
    p = torch.tensor(np.asarray(la, dtype=np.float64), requires_grad=True)
    total = 0.0
    L = p.shape[0]
    for b, (prefix, tg) in enumerate(zip(prefixes, targets)):
        lg = forward_logits(shape, W, prefix, p, None if rounding is None else rounding[b])
        logp = torch.log_softmax(lg, -1)
        total = total - logp[torch.arange(L), torch.as_tensor(np.asarray(tg), dtype=torch.long)].sum()
    loss = total / (len(prefixes) * L)
    loss.backward()
    return float(loss.detach()), p.grad.numpy().copy()


class AdamW:
    """Decoupled weight decay regularisation (AdamW): theta <- theta - lr * (m_hat / (sqrt(v_hat) + eps) + wd * theta)."""

    def __init__(self, n, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
        self.m = np.zeros(n)
        self.v = np.zeros(n)
        self.t = 0
        self.b1, self.b2, self.eps, self.wd = beta1, beta2, eps, weight_decay

    def step(self, theta, grad, lr):
        self.t += 1
        g = np.asarray(grad, dtype=np.float64).ravel()
        self.m = self.b1 * self.m + (1 - self.b1) * g
        self.v = self.b2 * self.v + (1 - self.b2) * g * g
        m_hat = self.m / (1 - self.b1 ** self.t)
        v_hat = self.v / (1 - self.b2 ** self.t)
        th = np.asarray(theta, dtype=np.float64).ravel()
        return (th - lr * (m_hat / (np.sqrt(v_hat) + self.eps) + self.wd * th)).reshape(np.shape(theta))


def learning_rate(step, peak=0.01, warmup=2000, total=10000):
    """Linear warm-up to `peak` over `warmup` steps, then a cosine down to zero at `total` (step counts from 0)."""
    if step < warmup:
        return peak * (step + 1) / warmup
    return 0.5 * peak * (1 + math.cos(math.pi * (step - warmup) / max(1, total - warmup)))
