"""Look-ahead embedding training (pass_train_*) against the training oracle: loss, gradient and the
AdamW trajectory of several steps on a batch of ragged prefixes, and the drafting call afterwards."""
import copy

import numpy as np
import pytest

import parity
import pass_oracle as O
import pass_train_oracle as TO
from paper_2311_13581_amd import synth

pytestmark = pytest.mark.gpu

TINY = synth.WORKLOADS["tiny_fp32_greedy"].shape
SMALL_BF16 = synth.ModelShape(2, 256, 4, 64, 704, 512, dtype=synth.BF16)
HD128_BF16 = synth.ModelShape(2, 256, 2, 128, 512, 384, dtype=synth.BF16)


def _gpu(shape, W, k, max_slots, max_seq_len, page, options=None):
    from paper_2311_13581_amd import binding
    g = binding.Pass(binding.make_config(shape, k, max_slots, max_seq_len, page), options)
    g.load_weights(W)
    return g


def _update_bound(opt, la, grad, lr, delta):
    """How far one AdamW step may move apart when every gradient component is off by at most delta: the
    oracle's own step taken at grad - delta, grad and grad + delta (the first steps divide a component
    by its own magnitude, so a component within delta of zero may go either way by lr)."""
    lo, mid, hi = (copy.deepcopy(opt).step(la, grad + s * delta, lr) for s in (-1.0, 0.0, 1.0))
    return np.maximum(np.abs(lo - mid), np.abs(hi - mid))


# bf16 models: the cache holds K and V in bf16 on both sides; a value that fp32 and fp64 arithmetic put on
# different sides of a rounding boundary differs by 2^-9 of itself between them (measured: up to 8e-5 of
# the largest gradient component, 1.5e-5 of the loss; fp32 models 5e-7 and 7e-8)
@pytest.mark.parametrize("shape,page,path,lockstep,tol_loss,tol_grad",
                         [(TINY, 16, 1, False, 1e-6, 5e-6), (TINY, 16, 1, True, 1e-6, 5e-6), (SMALL_BF16, 16, 1, True, 6e-5, 4e-4),
                          (HD128_BF16, 64, 1, True, 6e-5, 4e-4), (SMALL_BF16, 16, 0, True, 6e-5, 4e-4),
                          (HD128_BF16, 64, 0, True, 6e-5, 4e-4)],
                         ids=["fp32-free", "fp32", "bf16-generic", "bf16-hd128-generic", "bf16", "bf16-hd128"])
def test_training_steps_match_the_oracle(shape, page, path, lockstep, tol_loss, tol_grad):
    """Five AdamW steps on changing batches of three ragged prefixes (one of them ends where the
    attention backward's chunks of 256 keys meet, so that the block's own rows straddle two workgroups): the loss and the gradient of every step and the trained
    values after it, against the fp64 oracle fed with the same weights; the embeddings start from the
    embedding of one token, as in the paper.  "free": both sides run their own trajectory from the
    common start; otherwise the oracle's state (values, moments, step count, rounded to fp32) is
    written into the library before every step, so that every step is compared at the same point."""
    k, init_token = 3, 7
    W = synth.make_weights(shape, 13, k, 6.0)
    g = _gpu(shape, W, k, 3, 320, page, {"path": path})
    g.train_begin(init_token)
    la = TO._t(W["tok_emb"], shape.dtype)[init_token].numpy()[None, :].repeat(k, 0)
    assert np.array_equal(g.train_read(0), la.astype(np.float32))
    opt = TO.AdamW(la.size, 0.9, 0.999, 1e-8, 0.01)
    rng = np.random.default_rng(3)
    slack = np.zeros_like(la)
    for step in range(5):
        prefixes = [rng.integers(0, shape.vocab, n).astype(np.int32) for n in (5 + step, 255 + step, 97 + 7 * step)]
        targets = rng.integers(0, shape.vocab, (3, k)).astype(np.int32)
        for i, p in enumerate(prefixes):
            g.prefill(i, p, seq_id=i)
        lr = 0.01 * (step + 1) / 5
        if lockstep:
            la = la.astype(np.float32).astype(np.float64)
            opt.m = opt.m.astype(np.float32).astype(np.float64)
            opt.v = opt.v.astype(np.float32).astype(np.float64)
            g.train_resume(la, opt.m, opt.v, opt.t)
            slack[:] = 0
        loss = g.train_step([0, 1, 2], targets, lr)
        o_loss, o_grad = TO.loss_and_grad(shape, W, la, [p.tolist() for p in prefixes], targets)
        grad = g.train_read(1)
        e_loss, e_grad, g_max = abs(loss - o_loss) / abs(o_loss), float(np.abs(grad - o_grad).max()), float(np.abs(o_grad).max())
        print(f"step {step}: loss {loss:.6f} (oracle {o_loss:.6f}, rel {e_loss:.1e}) grad err {e_grad / g_max:.1e} of max {g_max:.3f}")
        assert e_loss <= tol_loss, (step, loss, o_loss)
        assert e_grad <= tol_grad * g_max, (step, e_grad, g_max)
        slack = slack + 1.5 * _update_bound(opt, la, o_grad, lr, tol_grad * g_max) + 1e-6
        la = opt.step(la, o_grad, lr)
        over = float((np.abs(g.train_read(0) - la) - slack).max())
        assert over <= 0, (step, over)
        if lockstep:  # the moments, too
            assert float(np.abs(g.train_read(2).ravel() - opt.m).max()) <= 0.11 * tol_grad * g_max + 1e-7
            assert float(np.abs(g.train_read(3).ravel() - opt.v).max()) <= 0.003 * tol_grad * g_max * g_max + 1e-7
        assert g.seq_len(0)[0] == len(prefixes[0]) - 1  # the slots are left as they were
    g.close()


@pytest.mark.parametrize("k", [1, 5, 7, 8, 15])
@pytest.mark.parametrize("shape,page,path", [(TINY, 16, 1), (SMALL_BF16, 16, 0), (HD128_BF16, 64, 0)], ids=["fp32", "bf16", "bf16-hd128"])
def test_one_training_step_for_every_row_bound(shape, page, path, k):
    """One step for look-ahead counts that select each compile-time row bound of the attention backward
    (2, 6, 8 and 16 rows per slot; 3, 4 and 5 are the other tests'), two slots, the second prefix
    longer than one chunk of keys."""
    W = synth.make_weights(shape, 31 + k, k, 6.0)
    g = _gpu(shape, W, k, 2, 320, page, {"path": path})
    g.train_begin(-1)
    la = TO._t(W["lookahead"], shape.dtype).numpy()
    rng = np.random.default_rng(k)
    prefixes = [rng.integers(0, shape.vocab, n).astype(np.int32) for n in (1, 270 + k)]
    targets = rng.integers(0, shape.vocab, (2, k)).astype(np.int32)
    for i, p in enumerate(prefixes):
        g.prefill(i, p, seq_id=i)
    loss = g.train_step([0, 1], targets, 0.01)
    o_loss, o_grad = TO.loss_and_grad(shape, W, la, [p.tolist() for p in prefixes], targets)
    grad = g.train_read(1)
    e_loss, e_grad, g_max = abs(loss - o_loss) / abs(o_loss), float(np.abs(grad - o_grad).max()), float(np.abs(o_grad).max())
    print(f"k={k}: loss rel {e_loss:.1e} grad err {e_grad / g_max:.1e} of max {g_max:.3f}")
    fp32 = shape.dtype == synth.F32
    assert e_loss <= (1e-6 if fp32 else 6e-5) and e_grad <= (5e-6 if fp32 else 4e-4) * g_max
    g.close()


def test_training_step_at_13b_width_vs_oracle():
    """One step at the 13B model's width (one layer, full vocabulary, bf16: d_model 5120, 40 heads of
    128, d_ffn 13824 -- 320 and 864 strips, 160 and 432 k-tiles, none a power of two), k = 4, four ragged
    prefixes, matrix-core path."""
    import time
    w = synth.scaled(synth.WORKLOADS["13b_k4_t0.8"], n_layers=1)
    k = 4
    W = synth.make_weights(w.shape, w.seed, k, w.lm_head_scale)
    g = _gpu(w.shape, W, k, 4, 448, 64)
    g.train_begin(-1)
    la = TO._t(W["lookahead"], w.shape.dtype).numpy()
    rng = np.random.default_rng(12)
    prefixes = [rng.integers(0, w.shape.vocab, n).astype(np.int32) for n in (19, 258, 77, 385)]
    targets = rng.integers(0, w.shape.vocab, (4, k)).astype(np.int32)
    g.prefill_batch([0, 1, 2, 3], prefixes)
    loss = g.train_step([0, 1, 2, 3], targets, 0.01)
    grad = g.train_read(1)
    t0 = time.time()
    o_loss, o_grad = TO.loss_and_grad(w.shape, W, la, [p.tolist() for p in prefixes], targets)
    e_loss, e_grad, g_max = abs(loss - o_loss) / abs(o_loss), float(np.abs(grad - o_grad).max()), float(np.abs(o_grad).max())
    print(f"13B width: oracle {time.time() - t0:.0f} s; loss {loss:.6f} (oracle {o_loss:.6f}, rel {e_loss:.1e}) grad err {e_grad / g_max:.1e} of max {g_max:.3f}", flush=True)
    assert e_loss <= 1e-4 and e_grad <= 1.5e-3 * g_max
    g.close()


@pytest.mark.parametrize("shape,page,path", [(SMALL_BF16, 16, 0), (HD128_BF16, 64, 0), (TINY, 16, 1)], ids=["bf16", "bf16-hd128", "fp32"])
def test_training_step_with_the_most_rows_and_a_long_prefix(shape, page, path):
    """Four slots of sixteen rows (the 64 rows a call can carry: eight row groups in every GEMM, two
    column groups in the forward attention, the vector-ALU attention backward), one prefix of 2100
    tokens (nine chunks of keys, the forward attention's split plan beyond eight splits)."""
    k = 15
    W = synth.make_weights(shape, 77, k, 6.0)
    g = _gpu(shape, W, k, 4, 2176, page, {"path": path})
    g.train_begin(-1)
    la = TO._t(W["lookahead"], shape.dtype).numpy()
    rng = np.random.default_rng(5)
    prefixes = [rng.integers(0, shape.vocab, n).astype(np.int32) for n in (2100, 1, 300, 64)]
    targets = rng.integers(0, shape.vocab, (4, k)).astype(np.int32)
    g.prefill_batch([0, 1, 2, 3], prefixes)
    loss = g.train_step([0, 1, 2, 3], targets, 0.01)
    o_loss, o_grad = TO.loss_and_grad(shape, W, la, [p.tolist() for p in prefixes], targets)
    grad = g.train_read(1)
    e_loss, e_grad, g_max = abs(loss - o_loss) / abs(o_loss), float(np.abs(grad - o_grad).max()), float(np.abs(o_grad).max())
    print(f"64 rows: loss rel {e_loss:.1e} grad err {e_grad / g_max:.1e} of max {g_max:.3f}")
    fp32 = shape.dtype == synth.F32
    assert e_loss <= (1e-6 if fp32 else 6e-5) and e_grad <= (5e-6 if fp32 else 4e-4) * g_max
    g.close()


_ORACLE_7B = {}


@pytest.mark.parametrize("path", [0, 1], ids=["matrix-core", "generic"])
def test_training_step_at_7b_width_vs_oracle(path):
    """One step at the 7B model's width (two layers, full vocabulary, bf16), k = 4 as in the paper's
    best setting, a batch of eight ragged prefixes as in the paper's training: the column tiling of the transposed GEMMs at d_model 4096, d_ff 11008 and
    the 32000-row LM head, 32 heads of 128.  Measured: loss within 3.4e-5,
    gradient within 5.5e-4 of its largest component (bf16 rounding of the cached K/V falling on different
    sides between fp32 and fp64 arithmetic, as in the forward parity at this width)."""
    import time
    w = synth.scaled(synth.WORKLOADS["7b_b8_ragged_t1"], n_layers=2)
    k = 4
    W = synth.make_weights(w.shape, w.seed, k, w.lm_head_scale)
    g = _gpu(w.shape, W, k, 8, 576, 64, {"path": path})
    g.train_begin(-1)
    la = TO._t(W["lookahead"], w.shape.dtype).numpy()
    rng = np.random.default_rng(11)
    prefixes = [rng.integers(0, w.shape.vocab, n).astype(np.int32) for n in (37, 150, 301, 64, 512, 5, 257, 129)]
    targets = rng.integers(0, w.shape.vocab, (8, k)).astype(np.int32)
    for i, p in enumerate(prefixes):
        g.prefill(i, p, seq_id=i)
    loss = g.train_step(list(range(8)), targets, 0.01)
    grad = g.train_read(1)
    t0 = time.time()
    if not _ORACLE_7B:  # the same inputs on both paths: the oracle runs once
        _ORACLE_7B["r"] = TO.loss_and_grad(w.shape, W, la, [p.tolist() for p in prefixes], targets)
    o_loss, o_grad = _ORACLE_7B["r"]
    e_loss, e_grad, g_max = abs(loss - o_loss) / abs(o_loss), float(np.abs(grad - o_grad).max()), float(np.abs(o_grad).max())
    print(f"7B width: oracle {time.time() - t0:.0f} s; loss {loss:.6f} (oracle {o_loss:.6f}, rel {e_loss:.1e}) grad err {e_grad / g_max:.1e} of max {g_max:.3f}", flush=True)
    assert e_loss <= 1e-4 and e_grad <= 1.5e-3 * g_max
    opt = TO.AdamW(la.size, 0.9, 0.999, 1e-8, 0.01)
    slack = 1.5 * _update_bound(opt, la, o_grad, 0.01, 1.5e-3 * g_max) + 1e-6
    assert float((np.abs(g.train_read(0) - opt.step(la, o_grad, 0.01)) - slack).max()) <= 0
    g.close()


def test_training_state_resumes():
    """Two steps, state saved, two more steps; a fresh context resumed from the saved state takes the
    same two steps to the same values bit for bit."""
    shape, k = SMALL_BF16, 2
    W = synth.make_weights(shape, 17, k, 6.0)
    rng = np.random.default_rng(1)
    batches = [([rng.integers(0, shape.vocab, n).astype(np.int32) for n in (9, 30)], rng.integers(0, shape.vocab, (2, k))) for _ in range(4)]

    def run(g, which):
        for prefixes, targets in which:
            for i, p in enumerate(prefixes):
                g.prefill(i, p, seq_id=i)
            g.train_step([0, 1], targets, 0.01)

    a = _gpu(shape, W, k, 2, 64, 16)
    a.train_begin(11)
    run(a, batches[:2])
    saved = [a.train_read(w) for w in (0, 2, 3)]
    run(a, batches[2:])
    b = _gpu(shape, W, k, 2, 64, 16)
    b.train_begin(-1)
    b.train_resume(saved[0], saved[1], saved[2], 2)
    run(b, batches[2:])
    for w in (0, 2, 3):
        assert np.array_equal(a.train_read(w), b.train_read(w)), w
    a.close()
    b.close()


def test_drafting_call_uses_the_trained_embeddings_and_training_lowers_the_loss():
    """Thirty steps on one fixed batch lower its loss; the drafting call then runs on the trained
    embeddings: its logits equal the C oracle's with the trained values as look-ahead embeddings."""
    shape, k = TINY, 2
    W = synth.make_weights(shape, 21, k, 6.0)
    g = _gpu(shape, W, k, 2, 96, 16, {"path": 1})
    g.train_begin(-1)  # from the model's own look-ahead tensor
    assert np.array_equal(g.train_read(0), W["lookahead"])
    rng = np.random.default_rng(9)
    prefixes = [rng.integers(0, shape.vocab, n).astype(np.int32) for n in (12, 40)]
    targets = rng.integers(0, shape.vocab, (2, k)).astype(np.int32)
    for i, p in enumerate(prefixes):
        g.prefill(i, p, seq_id=i)
    losses = [g.train_step([0, 1], targets, 0.01) for _ in range(30)]
    assert losses[-1] < losses[0] - 0.3, losses
    trained = g.train_read(0)
    W2 = dict(W)
    W2["lookahead"] = trained.copy()
    s = O.Model(shape, W2, k).sequence(96, seq_id=0)
    s.prefill(prefixes[0])
    s.draft(0.0, 1)
    g.draft([0], 0.0, 1)
    parity.logits_error(g.get_logits(0, 0), s.logits(0), 1e-4, "drafting call after training")
    g.verify([0], 0.0, 1)
    g.close()


def test_training_error_paths():
    from paper_2311_13581_amd import binding
    shape, k = SMALL_BF16, 2
    W = synth.make_weights(shape, 5, k, 4.0)
    odd = synth.ModelShape(1, 256, 4, 64, 96, 512, dtype=synth.BF16)  # d_ffn not a multiple of 64
    g = _gpu(odd, synth.make_weights(odd, 5, k, 4.0), k, 1, 64, 16)
    with pytest.raises(binding.PassError) as e:
        g.train_begin(3)  # the matrix-core path cannot train this shape ...
    assert e.value.code == -2
    g.close()
    g = _gpu(odd, synth.make_weights(odd, 5, k, 4.0), k, 1, 64, 16, {"path": 1})
    g.train_begin(3)  # ... the generic kernels can
    g.close()
    g = _gpu(shape, W, k, 1, 64, 16)
    g.prefill(0, [1, 2, 3])
    with pytest.raises(binding.PassError) as e:
        g.train_step([0], [[1, 2]], 0.01)  # before pass_train_begin
    assert e.value.code == -2
    g.train_begin(3)
    with pytest.raises(binding.PassError) as e:
        g.train_step([0], [[1, shape.vocab]], 0.01)
    assert e.value.code == -1
    g.set_option("lookahead_rows", 1)
    with pytest.raises(binding.PassError) as e:
        g.train_step([0], [[1, 2]], 0.01)
    assert e.value.code == -2
    g.set_option("lookahead_rows", 2)
    assert g.train_step([0], [[1, 2]], 0.01) > 0
    g.close()


def test_training_loop_on_text_the_model_wrote_itself():
    """The training recipe end to end on data the model makes itself: sequences decoded greedily from
    random prompts are the corpus, the look-ahead embeddings are trained on them as in the paper (one
    random cut per sequence and step, batches of 8, fresh batches, linear warm-up then cosine, start
    from one token's embedding), and the loss on held-out sequences of the same kind falls.  Greedy
    generation is unchanged by what the embeddings have become (it is the target model's own decoding
    whatever the drafts).  No claim about accepted drafts: a random model has nothing that could look
    ahead, the embeddings can only learn the corpus' token statistics (the counts are printed)."""
    shape, k = SMALL_BF16, 3
    W = synth.make_weights(shape, 3, k, 6.0)
    g = _gpu(shape, W, k, 8, 192, 16)
    rng = np.random.default_rng(0)
    slots = list(range(8))

    def decode(prompts, n_new):
        for i, p in enumerate(prompts):
            g.prefill(i, p, seq_id=100 + i)
        return g.generate(slots, n_new, 0.0, 1)

    def batch_of(seqs, lr):
        targets = np.zeros((8, k), dtype=np.int32)
        for i, seq in enumerate(seqs):
            T = int(rng.integers(4, len(seq) - k - 1))  # prefix w_1 .. w_T; the rows predict w_{T+2} .. w_{T+1+k}
            g.prefill(i, seq[:T], seq_id=i)
            targets[i] = seq[T + 1:T + 1 + k]
        return g.train_step(slots, targets, lr)

    texts = []
    for _ in range(7):  # 56 sequences of 8 prompt tokens + 96 generated ones; the last 8 are held out
        prompts = [rng.integers(0, shape.vocab, 8).astype(np.int32) for _ in slots]
        toks, _ = decode(prompts, 96)
        texts += [np.concatenate([p, t]).astype(np.int32) for p, t in zip(prompts, toks)]
    corpus, held_out = texts[:48], texts[48:]
    eval_prompts = [rng.integers(0, shape.vocab, 8).astype(np.int32) for _ in slots]
    ref, before = decode(eval_prompts, 64)

    def held_out_loss():  # steps with learning rate 0 change no value
        return float(np.mean([batch_of(held_out, 0.0) for _ in range(6)]))

    g.train_begin(1)
    loss0 = held_out_loss()
    start = g.train_read(0)
    g.train_begin(1)  # moments and step count back to zero
    n_steps = 150
    for step in range(n_steps):
        batch_of([corpus[i] for i in rng.choice(len(corpus), 8, replace=False)], TO.learning_rate(step, 0.01, 20, n_steps))
    trained = g.train_read(0)
    loss1 = held_out_loss()
    assert np.array_equal(g.train_read(0), trained) and not np.array_equal(trained, start)
    out, after = decode(eval_prompts, 64)
    rate = lambda st: st["drafts_accepted"] / max(1, st["drafts_proposed"])
    print(f"held-out loss {loss0:.2f} -> {loss1:.2f}; accepted drafts {rate(before):.2f} -> {rate(after):.2f}; "
          f"tokens per iteration {before['tokens_out'] / before['iterations']:.2f} -> {after['tokens_out'] / after['iterations']:.2f}")
    assert np.array_equal(out, ref)
    assert loss1 < loss0 - 0.3, (loss0, loss1)
    g.close()
