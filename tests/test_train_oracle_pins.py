"""Pins of the training oracle (oracle/pass_train_oracle.py) against what the mathematics fixes and
against the independent C oracle's forward pass."""
import math

import numpy as np
import pytest

import pass_oracle as O
import pass_train_oracle as TO
from paper_2311_13581_amd import synth

SHAPE = synth.ModelShape(2, 32, 2, 16, 48, 24, dtype=synth.F32)
SHAPE_BF16 = synth.ModelShape(2, 64, 4, 16, 96, 40, dtype=synth.BF16)


def _setup(shape, k=3, seed=5, scale=3.0):
    W = synth.make_weights(shape, seed, k, scale, std=0.1)
    rng = np.random.default_rng(seed)
    prefixes = [rng.integers(0, shape.vocab, n).tolist() for n in (7, 4)]
    targets = rng.integers(0, shape.vocab, (2, k))
    la = rng.standard_normal((k, shape.d_model)) * 0.1
    return W, prefixes, targets, la


@pytest.mark.parametrize("shape", [SHAPE, SHAPE_BF16], ids=["fp32", "bf16"])
def test_training_forward_equals_the_c_oracles_drafting_call(shape):
    """The logits of the look-ahead rows equal those of the C oracle's drafting call on the same
    sequence (two independent implementations of the forward pass) when the look-ahead embeddings
    hold storage-format values."""
    k = 3
    W, prefixes, _, _ = _setup(shape, k)
    la = TO._t(W["lookahead"], shape.dtype)
    m = O.Model(shape, W, k)
    for prefix in prefixes:
        s = m.sequence(32)
        s.prefill(np.array(prefix, np.int32))
        s.draft(1.0, 1)
        ref = s.logits(0)[1:]
        got = TO.forward_logits(shape, W, prefix, la).detach().numpy()
        assert np.allclose(got, ref, rtol=0, atol=2e-6 * np.abs(ref).max())


@pytest.mark.parametrize("shape", [SHAPE, SHAPE_BF16], ids=["fp32", "bf16"])
def test_gradient_equals_central_differences(shape):
    """Reverse-mode gradient of the batch loss w.r.t. the look-ahead embeddings against central
    differences of the loss itself, on coordinates of every look-ahead row."""
    k = 3
    W, prefixes, targets, la = _setup(shape, k)
    # a bfloat16 model rounds the cached K/V: the loss is piecewise constant in them and finite
    # differences would see the steps, so the amounts the rounding adds at `la` are recorded and
    # held fixed for the shifted points (same value and gradient at `la`, smooth around it)
    frozen = [[] for _ in prefixes] if shape.dtype == synth.BF16 else None
    loss, grad = TO.loss_and_grad(shape, W, la, prefixes, targets, frozen)
    assert (loss, grad.tolist()) == (lambda r: (r[0], r[1].tolist()))(TO.loss_and_grad(shape, W, la, prefixes, targets))
    assert loss > 0 and np.abs(grad).max() > 1e-4
    h = 1e-5
    for (i, j) in [(0, 0), (0, 17), (1, 5), (2, 31), (2, 8)]:
        e = np.zeros_like(la)
        e[i, j] = h
        lp, _ = TO.loss_and_grad(shape, W, la + e, prefixes, targets, frozen)
        lm, _ = TO.loss_and_grad(shape, W, la - e, prefixes, targets, frozen)
        fd = (lp - lm) / (2 * h)
        assert abs(fd - grad[i, j]) <= 1e-6 * max(1.0, np.abs(grad).max()) + 1e-5 * abs(grad[i, j]), (i, j, fd, grad[i, j])


def test_loss_closed_form_with_a_zero_lm_head():
    """A zero LM head gives uniform predictions: the loss is ln V and the gradient vanishes."""
    k = 2
    W, prefixes, targets, la = _setup(SHAPE, k)
    W = dict(W)
    W["lm_head"] = np.zeros_like(W["lm_head"])
    loss, grad = TO.loss_and_grad(SHAPE, W, la[:k], prefixes, targets[:, :k])
    assert abs(loss - math.log(SHAPE.vocab)) < 1e-12 and np.abs(grad).max() == 0


def test_only_later_rows_feel_an_earlier_lookahead_embedding():
    """Causality: look-ahead row i attends to rows 1 .. i only, so the loss of row 1 alone has no
    gradient w.r.t. embeddings 2 .. L, while the loss of the last row reaches all of them."""
    import torch
    k = 3
    W, prefixes, targets, la = _setup(SHAPE, k)
    p = torch.tensor(la, requires_grad=True)
    lg = TO.forward_logits(SHAPE, W, prefixes[0], p)
    torch.log_softmax(lg[0], -1)[targets[0, 0]].backward(retain_graph=True)
    g = p.grad.clone()
    assert g[0].abs().max() > 0 and g[1:].abs().max() == 0
    p.grad.zero_()
    torch.log_softmax(lg[2], -1)[targets[0, 2]].backward()
    assert all(p.grad[i].abs().max() > 0 for i in range(3))


def test_adamw_first_steps_closed_form():
    """First step: m_hat = g, v_hat = g^2, so the step is lr * (g / (|g| + eps) + wd * theta); with zero
    gradient only the decay acts; the moments follow their recurrences."""
    opt = TO.AdamW(4, 0.9, 0.999, 1e-8, 0.1)
    th = np.array([1.0, -2.0, 0.5, 0.0])
    g = np.array([0.3, -0.7, 0.0, 2.0])
    t1 = opt.step(th, g, 0.01)
    want = th - 0.01 * (g / (np.abs(g) + 1e-8) + 0.1 * th)
    assert np.allclose(t1, want, rtol=0, atol=1e-15)
    t2 = opt.step(t1, np.zeros(4), 0.01)
    m_hat = (0.9 * 0.1 * g) / (1 - 0.9 ** 2)
    v_hat = (0.999 * 0.001 * g * g) / (1 - 0.999 ** 2)
    assert np.allclose(t2, t1 - 0.01 * (m_hat / (np.sqrt(v_hat) + 1e-8) + 0.1 * t1), rtol=0, atol=1e-15)


def test_adamw_equals_the_library_optimiser():
    """Twelve steps with random gradients and a changing learning rate against torch.optim.AdamW in fp64
    (decoupled weight decay, bias-corrected moments, epsilon added to the root of the second moment)."""
    import torch
    rng = np.random.default_rng(8)
    th0 = rng.standard_normal(40)
    ref = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    lib = torch.optim.AdamW([ref], lr=0.01, betas=(0.85, 0.97), eps=1e-7, weight_decay=0.05)
    opt = TO.AdamW(40, 0.85, 0.97, 1e-7, 0.05)
    th = th0.copy()
    for step in range(12):
        g = rng.standard_normal(40) * (10.0 ** rng.integers(-3, 2))
        lr = 0.01 * (step + 1) / 12
        for grp in lib.param_groups:
            grp["lr"] = lr
        ref.grad = torch.tensor(g, dtype=torch.float64)
        lib.step()
        th = opt.step(th, g, lr)
        assert np.allclose(th, ref.detach().numpy(), rtol=1e-12, atol=1e-14), step


def test_learning_rate_schedule():
    """Linear warm-up over 2000 steps to 0.01, cosine to zero at step 10000."""
    assert TO.learning_rate(0) == pytest.approx(0.01 / 2000)
    assert TO.learning_rate(1999) == pytest.approx(0.01)
    assert TO.learning_rate(2000) == pytest.approx(0.01)
    assert TO.learning_rate(6000) == pytest.approx(0.005)
    assert TO.learning_rate(10000) == pytest.approx(0.0, abs=1e-12)


def test_training_reduces_the_loss():
    """Twenty AdamW steps on a fixed batch lower the loss (the optimiser and the gradient agree in sign)."""
    k = 3
    W, prefixes, targets, la = _setup(SHAPE, k)
    opt = TO.AdamW(la.size)
    first = None
    for step in range(20):
        loss, grad = TO.loss_and_grad(SHAPE, W, la, prefixes, targets)
        first = loss if first is None else first
        la = opt.step(la, grad, 0.01)
    assert loss < first - 0.05
