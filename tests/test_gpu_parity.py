"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

import parity
import pass_oracle as O
from paper_2311_13581_amd import synth

pytestmark = pytest.mark.gpu

TINY = synth.WORKLOADS["tiny_fp32_greedy"]
TINY_BF16 = synth.scaled(TINY, dtype=synth.BF16)


def _gpu(shape, W, k, max_slots=1, max_seq_len=256, page_size=16, options=None):
    from paper_2311_13581_amd import binding
    g = binding.Pass(binding.make_config(shape, k, max_slots, max_seq_len, page_size), options)
    g.load_weights(W)
    return g


def _both(w, k, seed=None, scale=None, **kw):
    seed = w.seed if seed is None else seed
    W = synth.make_weights(w.shape, seed, max(k, 1), w.lm_head_scale if scale is None else scale)
    return _gpu(w.shape, W, k, **kw), O.Model(w.shape, W, k), W


@pytest.mark.parametrize("w,temp", [(TINY, 0.0), (TINY, 1.0), (TINY_BF16, 0.0), (TINY_BF16, 1.0)],
                         ids=["fp32-greedy", "fp32-t1", "bf16-greedy", "bf16-t1"])
def test_tiny_stepwise(w, temp):
    """Configuration 1 (and its bf16 twin): logits of every call and every decision, 24 iterations."""
    g, m, _ = _both(w, w.k)
    prompt = synth.make_prompts(w)[0]
    seed = synth.sampling_seed(w)
    st = parity.stepwise_parity(g, m, 0, 7, prompt, 24, temp, seed, parity.LOGIT_TOL[w.shape.dtype])
    print(st)
    parity.check_stats(st, 24, parity.ERR_F32 if w.shape.dtype == synth.F32 else parity.ERR_BF16_SMALL, max_unstable=1)
    g.close()


@pytest.mark.parametrize("w,temp", [(TINY, 0.0), (TINY, 1.0)], ids=["greedy", "t1"])
def test_tiny_generate(w, temp):
    """Configuration 1 end to end: 64 tokens, free running."""
    g, m, _ = _both(w, w.k)
    prompt = synth.make_prompts(w)[0]
    seed = synth.sampling_seed(w)
    g.prefill(0, prompt, seq_id=0)
    toks, stats = g.generate([0], 64, temp, seed)
    s = m.sequence(256, seq_id=0)
    s.prefill(prompt)
    tau = 1e-4 * 40.0 / max(temp, 1.0) + parity.F32_ARITH
    ref, acc, stable = s.generate(64, temp, seed, tau=tau)
    n_same = parity.generate_parity(toks[0], ref, acc, stable)
    print("identical prefix", n_same, stats)
    assert n_same == 64  # measured: all 64 tokens identical in both modes (fp32 model, margins far above 1e-4)
    assert stats["tokens_out"] == 64 and 2 * stats["iterations"] <= 64 + w.k + 1
    assert stats["drafts_proposed"] == w.k * stats["iterations"]
    kv, ng = g.seq_len(0)
    assert kv == len(prompt) - 1 + ng and ng >= 64
    g.close()


@pytest.mark.parametrize("k", [0, 1, 4, 6])
def test_lookahead_counts_and_paging(k):
    """k sweep on the tiny model with 16-position pages and a prompt that is not a multiple of the
    page, the attention row group or the prefill chunk."""
    w = synth.scaled(TINY, k=k)
    g, m, _ = _both(w, k, seed=11)
    prompt = np.random.default_rng(k).integers(0, w.shape.vocab, 75).astype(np.int32)
    st = parity.stepwise_parity(g, m, 0, 3, prompt, 10, 0.7, 99, 1e-4)
    print(st)
    parity.check_stats(st, 10, parity.ERR_F32, max_unstable=1)
    g.close()


def test_high_temperature_accepts_drafts():
    """Flat distributions (high temperature) make drafts get accepted: the accept, partial-accept
    and all-accepted (extra token) branches all run under bit-exact comparison."""
    w = synth.scaled(TINY, k=3)
    g, m, _ = _both(w, 3, seed=5, scale=1.0)
    total = parity.StepStats()
    for sid in range(4):
        prompt = np.random.default_rng(sid).integers(0, w.shape.vocab, 9 + sid).astype(np.int32)
        parity.stepwise_parity(g, m, 0, sid, prompt, 12, 3.0, 1234, 1e-4, stats=total)
    print(total)
    assert total.accepted >= 10 and total.iterations == 48 and total.resyncs <= 1


def test_batch_of_ragged_slots_matches_single_runs():
    """Results of a slot do not depend on which other slots share the batch (per-sequence
    counters), with ragged prompt lengths; and they match the oracle."""
    w = synth.scaled(TINY, k=2)
    W = synth.make_weights(w.shape, 21, 2, 6.0)
    lens = [5, 37, 18]
    prompts = [np.random.default_rng(i).integers(0, w.shape.vocab, n).astype(np.int32) for i, n in enumerate(lens)]
    g = _gpu(w.shape, W, 2, max_slots=3)
    for i, p in enumerate(prompts):
        g.prefill(i, p, seq_id=100 + i)
    toks, stats = g.generate([0, 1, 2], 30, 1.0, 555)
    for i, p in enumerate(prompts):
        g.prefill(i, p, seq_id=100 + i)
        single, _ = g.generate([i], 30, 1.0, 555)
        assert np.array_equal(single[0], toks[i]), f"slot {i} depends on its batch"
    m = O.Model(w.shape, W, 2)
    for i, p in enumerate(prompts):
        s = m.sequence(256, seq_id=100 + i)
        s.prefill(p)
        ref, acc, stable = s.generate(30, 1.0, 555, tau=1e-4 * 40 + parity.F32_ARITH)
        parity.generate_parity(toks[i], ref, acc, stable)
    g.close()


def test_gpu_greedy_pass_equals_gpu_autoregressive():
    """Property that holds at any size: greedy PaSS (k=4) and greedy k=0 decoding give the same
    tokens on the GPU path."""
    w = synth.scaled(TINY_BF16, k=4)
    W = synth.make_weights(w.shape, 8, 4, 8.0)
    prompt = np.random.default_rng(3).integers(0, w.shape.vocab, 40).astype(np.int32)
    outs = []
    for k in (4, 0):
        g = _gpu(w.shape, W, k)
        g.prefill(0, prompt)
        outs.append(g.generate([0], 48, 0.0, 0)[0][0])
        g.close()
    assert np.array_equal(outs[0], outs[1])


def test_error_paths():
    from paper_2311_13581_amd import binding
    w = synth.scaled(TINY, k=2)
    W = synth.make_weights(w.shape, 1, 2, 1.0)
    g = _gpu(w.shape, W, 2, max_slots=2, max_seq_len=32)
    with pytest.raises(binding.PassError) as e:
        g.draft([0], 1.0, 1)  # not prefilled
    assert e.value.code == -2
    with pytest.raises(binding.PassError) as e:
        g.prefill(5, [1, 2, 3])
    assert e.value.code == -1
    with pytest.raises(binding.PassError) as e:
        g.prefill(0, [1, 2, 9999])
    assert e.value.code == -1
    with pytest.raises(binding.PassError) as e:
        g.prefill(0, np.arange(40) % 100)  # longer than max_seq_len
    assert e.value.code == -3
    g.prefill(0, [1, 2, 3])
    with pytest.raises(binding.PassError) as e:
        g.verify([0], 1.0, 1)  # verify before draft
    assert e.value.code == -2
    with pytest.raises(binding.PassError) as e:
        g.draft([0, 0], 1.0, 1)
    assert e.value.code == -1
    with pytest.raises(binding.PassError) as e:
        g.draft([0], 1.0, 1, -3)  # negative top-k
    assert e.value.code == -1
    with pytest.raises(binding.PassError) as e:
        g.generate([0], 64, 1.0, 1)  # runs out of positions
    assert e.value.code == -3
    g.prefill(0, [1, 2, 3])  # the slot is usable again after the failure
    g.draft([0], 0.0, 1)
    g.verify([0], 0.0, 1)
    g.close()


def test_device_uniforms_equal_the_oracles_on_a_million_counters():
    """The epilogues' generator (Philox4x32-10 and the bits-to-float step) against the oracle's, bit for
    bit: 2^20 + 3 consecutive vocabulary indices of one stream (more than the staging buffer holds, so
    several pieces and a ragged tail), then every purpose, rows at both ends, keys and counters with high
    bits set, and a start far into the index range."""
    from paper_2311_13581_amd import binding
    w = TINY
    g = binding.Pass(binding.make_config(w.shape, w.k, 1, 64, 16))
    n = (1 << 20) + 3
    got = g.rng_uniforms(0x0123456789ABCDEF, 7, 5, 2, 0, 0, n)
    want = O.uniforms(0x0123456789ABCDEF, 7, 5, 2, 0, 0, n)
    assert got.dtype == np.float32 and np.array_equal(got.astype(np.float64), want)
    assert 0.0 < got.min() and got.max() < 1.0
    for seed, sid, it, row, purpose, first in [(0, 0, 0, 0, 0, 0), (1, 2, 3, 4, 1, 0), (2 ** 64 - 1, 2 ** 32 - 1, 2 ** 32 - 1, 255, 3, 8),
                                              (5 << 32, 1 << 31, 1 << 31, 15, 2, 2 ** 32 - 4096), (9, 3, 1, 1, 2, 31996)]:
        m = 4093 if first < 2 ** 32 - 4096 else 4096
        got = g.rng_uniforms(seed, sid, it, row, purpose, first, m)
        assert np.array_equal(got.astype(np.float64), O.uniforms(seed, sid, it, row, purpose, first, m)), (seed, row, purpose)
    for bad in [dict(row=256), dict(purpose=4), dict(first=2), dict(first=2 ** 32 - 4, n=5)]:
        a = dict(seed=1, seq_id=0, iteration=0, row=0, purpose=0, first=0, n=4)
        a.update(bad)
        with pytest.raises(binding.PassError) as e:
            g.rng_uniforms(**a)
        assert e.value.code == -1
    g.close()


def test_plain_read_yardstick():
    """pass_plain_read: argument checks, and a plausible duration for reading the tiny model."""
    from paper_2311_13581_amd import binding
    w = TINY
    g = binding.Pass(binding.make_config(w.shape, w.k, 1, 64, 16))
    with pytest.raises(binding.PassError) as e:
        g.plain_read(4096, 2)  # no weights yet
    assert e.value.code == -2
    g.load_weights(synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale))
    for bad in (0, 24, 1 << 40):
        with pytest.raises(binding.PassError) as e:
            g.plain_read(bad, 2)
        assert e.value.code == -1
    with pytest.raises(binding.PassError):
        g.plain_read(4096, 0)
    us = g.plain_read(1 << 20, 16)
    assert 0.5 < us < 1000.0, us
    g.close()


# ---------------------------------------------------------------------------------------------
# matrix-core (bf16 MFMA) path: shapes whose dimensions are multiples of the 16x32 weight tile
# ---------------------------------------------------------------------------------------------
MFMA_SMALL = synth.Workload("mfma_small", synth.ModelShape(2, 256, 4, 64, 704, 512, dtype=synth.BF16),
                            40, 2, 1, (21, 21), 32, 1.0, 8.0)
MFMA_HD128 = synth.Workload("mfma_hd128", synth.ModelShape(3, 512, 4, 128, 1184, 1008, dtype=synth.BF16),
                            41, 4, 1, (70, 70), 32, 1.0, 6.0)


@pytest.mark.parametrize("w", [MFMA_SMALL, MFMA_HD128], ids=["hd64", "hd128"])
@pytest.mark.parametrize("temp", [0.0, 1.0])
@pytest.mark.parametrize("path", [0, 1], ids=["mfma", "generic"])
def test_mfma_path_stepwise(w, temp, path):
    """Packed-tile MFMA GEMMs with fused epilogues against the oracle; the generic kernels on the
    same model as a cross-check of the tolerance."""
    g, m, _ = _both(w, w.k, options={"path": path})
    prompt = synth.make_prompts(w)[0]
    st = parity.stepwise_parity(g, m, 0, 5, prompt, 16, temp, 4242, parity.LOGIT_TOL[synth.BF16])
    print(st)
    parity.check_stats(st, 16, parity.ERR_BF16_SMALL)
    g.close()


def test_mfma_path_batches_span_several_row_tiles():
    """M = 4 slots x (1+4) rows = 20 rows (three 8-row MFMA groups, ragged), ragged prompts: every
    slot's tokens equal its single-slot run (same random streams; logits differ by the GEMMs'
    reduction order only, below the decision margins of this seeded run), and prefill chunks (up
    to 64 rows) agree with the oracle through the stepwise check of one of the slots."""
    w = MFMA_HD128
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    lens = [9, 75, 33, 50]
    prompts = [np.random.default_rng(10 + i).integers(0, w.shape.vocab, n).astype(np.int32) for i, n in enumerate(lens)]
    g = _gpu(w.shape, W, w.k, max_slots=4)
    for i, p in enumerate(prompts):
        g.prefill(i, p, seq_id=i)
    toks, stats = g.generate([0, 1, 2, 3], 24, 0.9, 77)
    for i, p in enumerate(prompts):
        g.prefill(i, p, seq_id=i)
        single, _ = g.generate([i], 24, 0.9, 77)
        assert np.array_equal(single[0], toks[i]), f"slot {i} depends on its batch"
    m = O.Model(w.shape, W, w.k)
    st = parity.stepwise_parity(g, m, 2, 2, prompts[1], 6, 0.9, 77, parity.LOGIT_TOL[synth.BF16])
    print(st, stats)
    parity.check_stats(st, 6, parity.ERR_BF16_SMALL)
    g.close()


def test_7b_layer_shapes_two_layers():
    """The 7B workload's layer shapes (d 4096, 32 heads x 128, FFN 11008, vocab 32000) with two
    layers, k = 4: logits and decisions against the oracle at the real tile counts."""
    w = synth.scaled(synth.WORKLOADS["7b_k4_greedy"], n_layers=2)
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    g = _gpu(w.shape, W, w.k, max_seq_len=128, page_size=64)
    m = O.Model(w.shape, W, w.k)
    prompt = synth.make_prompts(w)[0][:37]
    for temp, top_k in ((0.0, 0), (0.8, 0), (0.8, 10)):
        st = parity.stepwise_parity(g, m, 0, 1, prompt, 2, temp, 99, parity.LOGIT_TOL[synth.BF16], max_len=128,
                                    top_k=top_k)
        print(temp, top_k, st)
        # greedy on a random model with a scaled LM head meets near-ties: unstable decisions are counted, and one resync was seen
        parity.check_stats(st, 2, parity.ERR_BF16_7B_2L, max_unstable=12, max_resyncs=2)
    # The paper's own implementation runs all in bfloat16.  The oracle's variant that also rounds the
    # activations between matrix products (normalised rows, q, attention output, gated FFN rows) is
    # not the reference here, but the HIP path must stay within the bf16 tolerance of it too.
    mb = O.Model(w.shape, W, w.k, act_bf16=True)
    sb = mb.sequence(128, seq_id=1)
    sb.prefill(prompt)
    sb.draft(0.0, 99)
    g.prefill(0, prompt, seq_id=1)
    g.draft([0], 0.0, 99)
    err = parity.logits_error(g.get_logits(0, 0), sb.logits(0), parity.LOGIT_TOL[synth.BF16], "all-bf16-activation oracle")
    print("against the oracle with bf16 activations: max |diff| %.3e of max |logit| %.3e" % (err, np.abs(sb.logits(0)).max()))
    g.verify([0], 0.0, 99)
    g.close()


def test_graph_replay_equals_eager_launches():
    """The captured (model call + epilogue) graph is replayed many times with eager work (prefill,
    report copies, synchronisations) in between; every replay must give what eager launches give:
    stepwise against the oracle with graphs on, and token-identical generations graph on / off."""
    w = MFMA_HD128
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    m = O.Model(w.shape, W, w.k)
    prompt = synth.make_prompts(w)[0]
    outs = {}
    for graph in (1, 0):
        g = _gpu(w.shape, W, w.k, max_slots=2, options={"graph": graph})
        st = parity.stepwise_parity(g, m, 0, 9, prompt, 8, 1.0, 4242, parity.LOGIT_TOL[synth.BF16])
        parity.check_stats(st, 8, parity.ERR_BF16_SMALL)
        toks = []
        for rep in range(3):  # same sequence three times: replays after replays
            g.prefill(1, prompt[:33], seq_id=rep)
            toks.append(g.generate([1], 40, 0.7, 5)[0][0])
        g.prefill(0, prompt, seq_id=3)
        g.prefill(1, prompt[:50], seq_id=4)
        toks.append(g.generate([0, 1], 30, 1.0, 6)[0])
        outs[graph] = toks
        g.close()
    for a, b in zip(outs[1], outs[0]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("temp", [0.0, 0.9])
@pytest.mark.parametrize("plen", [5, 70, 200])
def test_matrix_core_attention(temp, plen):
    """bf16, head_dim 128, 64-position pages: the MFMA attention kernel over transposed V pages
    (prompt lengths below one 32-key block, inside one step, and over several splits), against the
    oracle, and against the lane-per-key kernel on the same model ("attention" option)."""
    w = MFMA_HD128
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    m = O.Model(w.shape, W, w.k)
    prompt = np.random.default_rng(plen).integers(0, w.shape.vocab, plen).astype(np.int32)
    for attn in (0, 1):
        g = _gpu(w.shape, W, w.k, max_seq_len=384, page_size=64, options={"attention": attn})
        st = parity.stepwise_parity(g, m, 0, 2, prompt, 6, temp, 777, parity.LOGIT_TOL[synth.BF16], max_len=384)
        print(attn, st)
        parity.check_stats(st, 6, parity.ERR_BF16_SMALL)
        g.close()



@pytest.mark.parametrize("plen,attn_rows,rows,strips,block", [
    (66, 0, 128, 0, 0), (130, 16, 128, 2, 203), (200, 32, 128, 4, 101), (300, 128, 128, 1, 1602),
    (300, 16, 256, 2, 364), (37, 32, 128, 4, 0), (300, 128, 384, 0, 6401), (150, 128, 128, 0, 0)])
def test_tiled_prompt_pass(plen, attn_rows, rows, strips, block):
    """The compute-bound prompt pass (tiled GEMMs, unsplit causal attention): ragged row tiles (65,
    129, 199, 299 rows against 64-row tiles; 36 rows forced through it), ragged feature tiles (148
    gate/up strips against 16 per workgroup), an odd number of k-steps (37), several passes over the
    weights (299 rows at 128 per pass: later passes attend to the earlier ones through the cache),
    every attention block height (128: the kernel with K/V tiles shared through LDS, with ragged
    last blocks and wavefronts without rows), every width of the GEMM tiles, and blocks of tiles per
    die from 1 x 1 to 64 x 1 (mostly empty blocks: every tile must still be computed exactly once).
    The first drafting and validation calls after it are compared with the oracle, which prefills row
    by row."""
    w = MFMA_HD128
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    m = O.Model(w.shape, W, w.k)
    prompt = np.random.default_rng(plen).integers(0, w.shape.vocab, plen).astype(np.int32)
    g = _gpu(w.shape, W, w.k, max_seq_len=384, page_size=64,
             options={"prefill_tiled": 1, "tune.prefill_tile": attn_rows, "tune.prefill_rows": rows, "tune.prefill_strips": strips,
                      "tune.prefill_block": block})
    st = parity.stepwise_parity(g, m, 0, 2, prompt, 3, 0.9, 777, parity.LOGIT_TOL[synth.BF16], max_len=384)
    print(st)
    parity.check_stats(st, 3, parity.ERR_BF16_SMALL)
    g.close()


@pytest.mark.parametrize("rows,lens", [(384, (37, 300, 129, 2, 1, 260)), (128, (200, 5, 131)), (256, (129, 128, 127, 1, 64, 65))])
def test_prompt_pass_over_several_slots(rows, lens):
    """pass_prefill_batch: ragged prompts of several sequences share tiled passes over the weights (every
    sequence starts on a block of 128 rows; prompts that spill into the next pass, that end exactly on a
    block, one-token prompts with nothing to cache, more blocks than one pass holds).  Every slot is then
    followed by the oracle through three iterations of calls that carry the whole batch, and its
    state equals what pass_prefill leaves."""
    w = MFMA_HD128
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    m = O.Model(w.shape, W, w.k)
    rng = np.random.default_rng(rows)
    prompts = [rng.integers(0, w.shape.vocab, n).astype(np.int32) for n in lens]
    slots = list(range(len(lens)))[::-1]  # slots in another order than the prompts
    seq_ids = [20 + i for i in range(len(lens))]
    g = _gpu(w.shape, W, w.k, max_slots=len(lens), max_seq_len=384, page_size=64,
             options={"prefill_tiled": 1, "tune.prefill_rows": rows})
    stats = parity.batch_parity(g, m, slots, seq_ids, prompts, slots, 3, 0.9, 777, parity.LOGIT_TOL[synth.BF16], max_len=384,
                                one_call=True)
    for sl in slots:
        print(sl, stats[sl])
        parity.check_stats(stats[sl], 3, parity.ERR_BF16_SMALL)
    # against one pass_prefill per slot: same lengths, and the next call's logits agree to rounding
    g.prefill_batch(slots, prompts, seq_ids)
    assert [g.seq_len(sl) for sl in slots] == [(n - 1, 0) for n in lens]
    g.draft(slots, 0.0, 1)
    a = [g.get_logits(sl, 0).copy() for sl in slots]
    for sl, sid, p in zip(slots, seq_ids, prompts):
        g.prefill(sl, p, seq_id=sid)
    g.draft(slots, 0.0, 1)
    for i, sl in enumerate(slots):
        b = g.get_logits(sl, 0)
        assert np.abs(a[i] - b).max() <= 1e-3 * np.abs(b).max(), (sl, np.abs(a[i] - b).max() / np.abs(b).max())
    with pytest.raises(Exception):
        g.prefill_batch([0, 0], prompts[:2], [1, 2])
    g.close()


def test_prompt_pass_over_several_slots_on_the_generic_path():
    """pass_prefill_batch where the tiled kernels do not apply: the prompts go one by one, same results."""
    w = TINY
    g, m, _ = _both(w, w.k, max_slots=3, max_seq_len=128)
    rng = np.random.default_rng(4)
    prompts = [rng.integers(0, w.shape.vocab, n).astype(np.int32) for n in (9, 1, 70)]
    stats = parity.batch_parity(g, m, [2, 0, 1], [5, 6, 7], prompts, [2, 0, 1], 3, 0.9, 11, parity.LOGIT_TOL[synth.F32], max_len=128,
                                one_call=True)
    for sl in stats:
        parity.check_stats(stats[sl], 3, parity.ERR_F32)
    g.close()


def test_tiled_and_chunked_prompt_passes_fill_the_same_cache():
    """Same prompt through the tiled pass and through the decode kernels in 64-row chunks: the logits
    of the next call agree to rounding (different summation orders, same bf16 cache up to the last
    bit of a few entries), and greedy generation continues with the same tokens."""
    w = MFMA_HD128
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    prompt = np.random.default_rng(5).integers(0, w.shape.vocab, 333).astype(np.int32)
    out = {}
    for tiled in (1, 0):
        g = _gpu(w.shape, W, w.k, max_seq_len=512, page_size=64, options={"prefill_tiled": tiled})
        g.prefill(0, prompt, seq_id=3)
        g.draft([0], 0.0, 1)
        lg = g.get_logits(0, 0).copy()
        g.verify([0], 0.0, 1)
        toks, _ = g.generate([0], 24, 0.0, 1)
        out[tiled] = (lg, toks[0])
        g.close()
    err = np.abs(out[1][0] - out[0][0]).max() / np.abs(out[0][0]).max()
    print("tiled vs chunked logits", err)
    assert err < 1e-3
    assert np.array_equal(out[1][1], out[0][1])


@pytest.mark.parametrize("w", [TINY, TINY_BF16, MFMA_HD128], ids=["fp32", "bf16", "mfma"])
@pytest.mark.parametrize("top_k", [1, 10, 25, 100000])
def test_top_k_sampling_stepwise(w, top_k):
    """Top-k sampling (the paper's sampler: k = 10, 25) in both epilogues: every decision of 16
    iterations against the oracle; K = 1 is greedy in effect, K above the vocabulary no filter."""
    g, m, _ = _both(w, w.k, max_seq_len=256, page_size=64 if w is MFMA_HD128 else 16)
    prompt = synth.make_prompts(w)[0]
    st = parity.stepwise_parity(g, m, 0, 5, prompt, 16, 0.8, 4242, parity.LOGIT_TOL[w.shape.dtype], top_k=top_k)
    print(top_k, st)
    # a top-k boundary adds decisions that sit near a tie by construction (measured: up to 5 unstable on the bf16 models)
    parity.check_stats(st, 16, (parity.ERR_F32 if w.shape.dtype == synth.F32 else parity.ERR_BF16_SMALL), max_unstable=2 if w.shape.dtype == synth.F32 else 10)
    g.close()


def test_top_k_boundary_ties_keep_the_lower_indices():
    """Exactly equal logits across the top-k boundary (LM-head rows repeated in blocks of 8): the
    kept set is the K largest with ties to the lower index.  Checked on the GPU's own logits with
    a stable sort: over many draws at a high temperature every sampled token lies in that set, and
    every member of the set shows up."""
    w = TINY
    W = synth.make_weights(w.shape, 77, w.k, 8.0)
    V = w.shape.vocab
    lm = W["lm_head"].reshape(V, -1).copy()
    lm[:] = lm[(np.arange(V) // 8) * 8]      # rows 8b..8b+7 all equal row 8b
    W["lm_head"] = lm.reshape(W["lm_head"].shape)
    g = _gpu(w.shape, W, w.k, max_seq_len=256)
    K = 11                                    # one whole block of 8 and 3 of the next
    prompt = synth.make_prompts(w)[0]
    g.prefill(0, prompt, seq_id=0)
    seen = [set() for _ in range(w.k + 1)]
    kept = None
    for seed in range(300):
        first, drafts = g.draft([0], 50.0, seed, K)   # commits x_{n+1}; restart below keeps the rows the same
        lg = g.get_logits(0, 0)
        order = [np.argsort(-lg[r], kind="stable")[:K] for r in range(w.k + 1)]
        if kept is None:
            kept = [set(int(j) for j in o) for o in order]
            for r in range(w.k + 1):          # the boundary really cuts a block of equal logits
                srt = np.sort(lg[r])[::-1]
                assert srt[K - 1] == srt[K]
        toks = [int(first[0])] + [int(t) for t in drafts[0]]
        for r, t in enumerate(toks):
            assert t in kept[r], (seed, r, t)
            seen[r].add(t)
        g.prefill(0, prompt, seq_id=0)        # same context again: same logits, new seed
    for r in range(w.k + 1):
        assert seen[r] == kept[r]
    g.close()


def test_lookahead_rows_change_at_run_time():
    """One loaded model (k = 6), the number of look-ahead rows per call switched by option: every
    setting must equal an oracle model built with that many look-ahead embeddings (the paper's sweep
    over the number of look-ahead tokens, without reloading)."""
    from paper_2311_13581_amd import binding
    w = synth.scaled(TINY, k=6)
    W = synth.make_weights(w.shape, 31, 6, 6.0)
    g = _gpu(w.shape, W, 6)
    prompt = np.random.default_rng(9).integers(0, w.shape.vocab, 29).astype(np.int32)
    for k_act in (0, 2, 6, 3):
        g.set_option("lookahead_rows", k_act)
        m = O.Model(w.shape, W, k_act)
        st = parity.stepwise_parity(g, m, 0, 2, prompt, 8, 0.9, 321, 1e-4)
        print(k_act, st)
        parity.check_stats(st, 8, parity.ERR_F32, max_unstable=1)
    g.prefill(0, prompt)
    g.draft([0], 0.0, 1)
    with pytest.raises(binding.PassError) as e:   # not between a drafting and a validation call
        g.set_option("lookahead_rows", 1)
    assert e.value.code == -2
    g.verify([0], 0.0, 1)
    with pytest.raises(binding.PassError) as e:
        g.set_option("lookahead_rows", 7)
    assert e.value.code == -1
    g.close()


@pytest.mark.parametrize("w", [TINY, MFMA_HD128], ids=["fp32", "mfma"])
def test_fixed_token_as_lookahead(w):
    """The paper's second baseline: a fixed token's embedding appended instead of the trained
    look-ahead embeddings ("lookahead_token" option), against the oracle in the same mode."""
    unk = 3
    g, _, W = _both(w, w.k, max_seq_len=256, page_size=64 if w is MFMA_HD128 else 16)
    g.set_option("lookahead_token", unk)
    m = O.Model(w.shape, W, w.k, la_token=unk)
    prompt = synth.make_prompts(w)[0]
    for temp in (0.0, 1.0):
        st = parity.stepwise_parity(g, m, 0, 4, prompt, 10, temp, 77, parity.LOGIT_TOL[w.shape.dtype])
        print(temp, st)
        parity.check_stats(st, 10, (parity.ERR_F32 if w.shape.dtype == synth.F32 else parity.ERR_BF16_SMALL))
    g.close()


@pytest.mark.parametrize("attn", [0, 1], ids=["matrix-core", "lane-per-key"])
def test_attention_over_many_splits(attn):
    """A context of 1100+ keys: more than 8 splits (the merge kernel's four-quarter form) and, for
    the lane-per-key kernel, chunks longer than one step; logits and decisions against the oracle."""
    w = MFMA_HD128
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    m = O.Model(w.shape, W, w.k)
    prompt = np.random.default_rng(12).integers(0, w.shape.vocab, 1100).astype(np.int32)
    g = _gpu(w.shape, W, w.k, max_seq_len=1280, page_size=64, options={"attention": attn})
    st = parity.stepwise_parity(g, m, 0, 3, prompt, 3, 0.9, 31, parity.LOGIT_TOL[synth.BF16], max_len=1280)
    print(attn, st)
    parity.check_stats(st, 3, parity.ERR_BF16_SMALL)
    g.close()


def test_attention_splits_of_several_steps():
    """32 heads and 3150 keys: 25 steps of 128 keys x 32 heads are more workgroups than the chip holds at
    once, so the split plan gives every workgroup two steps (the second step's K/V is requested at the
    end of the first) and 13 splits go through the merge kernel's four-quarter form; a narrow model
    (d_model 256 against an attention width of 4096) keeps the oracle's row-by-row prompt pass short."""
    shape = synth.ModelShape(1, 256, 32, 128, 704, 512, dtype=synth.BF16)
    W = synth.make_weights(shape, 77, 2, 8.0)
    m = O.Model(shape, W, 2)
    prompt = np.random.default_rng(5).integers(0, shape.vocab, 3150).astype(np.int32)
    g = _gpu(shape, W, 2, max_seq_len=3328, page_size=64)
    st = parity.stepwise_parity(g, m, 0, 1, prompt, 3, 0.9, 4711, parity.LOGIT_TOL[synth.BF16], max_len=3328)
    print(st)
    parity.check_stats(st, 3, parity.ERR_BF16_SMALL)
    g.close()


MANY_HEADS = synth.ModelShape(1, 256, 64, 128, 512, 512, dtype=synth.BF16)  # 64 heads: 12 steps x 64 = 768 workgroups


def test_split_plan_breakpoint_inside_the_pipelined_loop():
    """With 64 heads the split plan drops from 12 splits (1536 keys) to 7 (1537 keys).  A sequence
    that crosses that length inside pass_run_iterations, where the host sizes the grid for an upper
    bound of the length (up to k + 2 keys too many), must still get every split its own plan asks
    for: greedy tokens against the oracle's, then the logits of one more synchronised iteration."""
    shape, k = MANY_HEADS, 4
    W = synth.make_weights(shape, 61, k, 10.0)
    m = O.Model(shape, W, k)
    prompt = np.random.default_rng(3).integers(0, shape.vocab, 1528).astype(np.int32)
    g = _gpu(shape, W, k, max_seq_len=1664, page_size=64)
    g.prefill(0, prompt, seq_id=8)
    st = g.run_iterations([0], 8, 0.0, 17)
    kv, ng = g.seq_len(0)
    assert kv > 1536 + k + 2 and ng == st["tokens_out"]  # the sequence is past the breakpoint
    toks = g.get_tokens(0, 0, ng)
    s = m.sequence(1664, seq_id=8)
    s.prefill(prompt)
    ref, acc, stable = s.generate(ng, 0.0, 17, tau=1e-3 * 40)
    n_same = parity.generate_parity(toks, ref, acc, stable)
    print("identical prefix", n_same, "of", ng, "stable", stable)
    assert n_same == ng
    hist = list(prompt) + [int(t) for t in toks]
    st2 = parity.stepwise_parity(g, m, 0, 8, np.array(hist[:1540], np.int32), 2, 0.0, 17, parity.LOGIT_TOL[synth.BF16],
                                 max_len=1664)
    print(st2)
    parity.check_stats(st2, 2, parity.ERR_BF16_SMALL)
    g.close()


def test_split_plan_breakpoint_inside_one_batch():
    """Two slots either side of the breakpoint in one call (1530 and 1545 cached keys with 64 heads:
    12 and 7 splits): the grid must be as wide as the shorter sequence's plan.  Both slots against
    the oracle, every call."""
    shape, k = MANY_HEADS, 4
    W = synth.make_weights(shape, 61, k, 10.0)
    m = O.Model(shape, W, k)
    prompts = [np.random.default_rng(30 + i).integers(0, shape.vocab, n).astype(np.int32) for i, n in enumerate((1531, 1546))]
    g = _gpu(shape, W, k, max_slots=2, max_seq_len=1664, page_size=64)
    stats = parity.batch_parity(g, m, [0, 1], [3, 4], prompts, [0, 1], 2, 0.9, 23, parity.LOGIT_TOL[synth.BF16], max_len=1664)
    for sl in (0, 1):
        print(sl, stats[sl])
        parity.check_stats(stats[sl], 2, parity.ERR_BF16_SMALL)
    g.close()


@pytest.mark.parametrize("which,seed,len0", [("fp32", 2, 40), ("mfma", 5, 228)], ids=["fp32", "mfma"])
def test_finished_slot_at_its_capacity_does_not_touch_its_neighbours(which, seed, len0):
    """pass_generate keeps a slot that has reached its token target stepping with the batch.  In
    these seeded runs (found with the oracle) slot 0 reaches 24 tokens two iterations before slot 1
    and ends within k positions of max_seq_len: its rows then lie beyond its capacity and must
    neither write K/V (its block-table row ends there; the next entries are slot 1's pages) nor
    read any.  Both slots' tokens equal their single-slot runs and the oracle's."""
    k, n_new, temp = 4, 24, 1.5
    w = synth.scaled(TINY if which == "fp32" else MFMA_HD128, k=k)
    page = 64 if w.shape.head_dim == 128 else 16
    cap = 4 * page
    W = synth.make_weights(w.shape, 29, k, 3.0)
    rng = np.random.default_rng(2)
    p0 = rng.integers(0, w.shape.vocab, cap).astype(np.int32)[:len0]
    p1 = rng.integers(0, w.shape.vocab, 20).astype(np.int32)
    g = _gpu(w.shape, W, k, max_slots=2, max_seq_len=cap, page_size=page)
    single, iters, kv_end = {}, {}, {}
    for slot, p, sid in ((0, p0, 1), (1, p1, 2)):
        g.prefill(slot, p, seq_id=sid)
        toks, st = g.generate([slot], n_new, temp, seed)
        single[slot], iters[slot], kv_end[slot] = toks[0], st["iterations"], g.seq_len(slot)[0]
    # the scenario: slot 0 is finished, beyond its capacity, while slot 1 still runs
    assert iters[0] < iters[1] and kv_end[0] + 1 + k > cap, (iters, kv_end)
    g.prefill(0, p0, seq_id=1)
    g.prefill(1, p1, seq_id=2)
    both, st = g.generate([0, 1], n_new, temp, seed)
    assert st["iterations"] == iters[0] + iters[1]
    assert np.array_equal(both[0], single[0]) and np.array_equal(both[1], single[1])
    assert g.seq_len(0)[0] == kv_end[0] and g.seq_len(1)[0] == kv_end[1]
    m = O.Model(w.shape, W, k)
    tau = (2e-2 * 40 if w.shape.dtype == synth.BF16 else 1e-4 * 40) / temp + parity.F32_ARITH
    for slot, p, sid in ((0, p0, 1), (1, p1, 2)):
        s = m.sequence(cap + 8, seq_id=sid)
        s.prefill(p)
        ref, acc, stable = s.generate(n_new, temp, seed, tau=tau)
        n_same = parity.generate_parity(both[slot], ref, acc, stable)
        print(which, "slot", slot, "identical prefix", n_same, "stable", stable.all())
    g.close()


@pytest.mark.parametrize("w", [TINY, MFMA_HD128], ids=["fp32", "mfma"])
def test_maximum_lookahead_count(w):
    """k = 15 (the most the interface takes): 16 rows per call, so the attention kernels see two
    row groups per sequence and the second group's causal bound starts 8 positions later."""
    w = synth.scaled(w, k=15)
    g, m, _ = _both(w, 15, seed=19, max_seq_len=384, page_size=64 if w.shape.head_dim == 128 else 16)
    prompt = np.random.default_rng(4).integers(0, w.shape.vocab, 83).astype(np.int32)
    for temp in (0.0, 1.2):
        st = parity.stepwise_parity(g, m, 0, 6, prompt, 6, temp, 2024, parity.LOGIT_TOL[w.shape.dtype], max_len=384)
        print(temp, st)
        parity.check_stats(st, 6, (parity.ERR_F32 if w.shape.dtype == synth.F32 else parity.ERR_BF16_SMALL))
    g.close()


def test_maximum_rows_per_call():
    """8 slots x (1+7) rows = 64 rows, the most one call carries (eight 8-row MFMA groups): every
    slot against the oracle, free running, with ragged prompts."""
    w = synth.scaled(MFMA_SMALL, k=7)
    W = synth.make_weights(w.shape, 23, 7, 8.0)
    lens = [5, 64, 33, 90, 17, 129, 48, 71]
    prompts = [np.random.default_rng(40 + i).integers(0, w.shape.vocab, n).astype(np.int32) for i, n in enumerate(lens)]
    g = _gpu(w.shape, W, 7, max_slots=8, max_seq_len=256, page_size=16)
    for i, p in enumerate(prompts):
        g.prefill(i, p, seq_id=200 + i)
    toks, stats = g.generate(list(range(8)), 20, 1.0, 808)
    m = O.Model(w.shape, W, 7)
    for i, p in enumerate(prompts):
        s = m.sequence(256, seq_id=200 + i)
        s.prefill(p)
        ref, acc, stable = s.generate(20, 1.0, 808, tau=2e-2 * 40 + parity.F32_ARITH)
        parity.generate_parity(toks[i], ref, acc, stable)
    st = parity.stepwise_parity(g, m, 3, 203, prompts[3], 4, 1.0, 808, parity.LOGIT_TOL[synth.BF16])
    print(stats, st)
    parity.check_stats(st, 4, parity.ERR_BF16_SMALL)
    with pytest.raises(Exception):  # a ninth slot does not exist
        g.prefill(8, prompts[0])
    g.close()


@pytest.mark.parametrize("w", [TINY, MFMA_SMALL], ids=["fp32", "mfma"])
def test_degenerate_inputs(w):
    """The smallest inputs the interface takes: a prompt of one token (nothing cached before the
    first call), a generation of zero tokens, an empty slot list (an error, not a crash)."""
    from paper_2311_13581_amd import binding
    g, m, _ = _both(w, w.k, max_seq_len=128)
    st = parity.stepwise_parity(g, m, 0, 9, np.array([5], np.int32), 6, 0.0, 3, parity.LOGIT_TOL[w.shape.dtype],
                                max_len=128)
    parity.check_stats(st, 6, (parity.ERR_F32 if w.shape.dtype == synth.F32 else parity.ERR_BF16_SMALL))
    g.prefill(0, [7], seq_id=1)
    toks, stats = g.generate([0], 0, 1.0, 1)
    assert toks.shape == (1, 0) and stats["iterations"] == 0 and g.seq_len(0) == (0, 0)
    with pytest.raises(binding.PassError) as e:
        g.draft([], 1.0, 1)
    assert e.value.code == -1
    with pytest.raises(binding.PassError) as e:
        g.prefill(0, [])
    assert e.value.code == -1
    g.close()


def test_page_pool_limits_and_reuse():
    """A K/V page pool smaller than max_slots x pages per sequence: a prompt that does not fit the
    free pages is refused (capacity error, nothing half-done), releasing a slot returns its pages,
    and a sequence living on recycled, out-of-order pages still matches the oracle."""
    from paper_2311_13581_amd import binding
    w = TINY
    W = synth.make_weights(w.shape, w.seed, w.k, w.lm_head_scale)
    g = binding.Pass(binding.make_config(w.shape, w.k, 2, 128, 16, n_pages=9))
    g.load_weights(W)
    m = O.Model(w.shape, W, w.k)
    rng = np.random.default_rng(8)
    long_p, short_p = rng.integers(0, w.shape.vocab, 100).astype(np.int32), rng.integers(0, w.shape.vocab, 40).astype(np.int32)
    g.prefill(0, long_p, seq_id=1)                      # 7 of 9 pages
    with pytest.raises(binding.PassError) as e:
        g.prefill(1, short_p, seq_id=2)                 # needs 3 more
    assert e.value.code == -3
    g.draft([0], 0.0, 1)                                # slot 0 is untouched by the failure
    g.verify([0], 0.0, 1)
    g.release(0)
    st = parity.stepwise_parity(g, m, 1, 2, short_p, 5, 0.8, 17, 1e-4, max_len=128)   # recycled pages, reversed order
    parity.check_stats(st, 5, parity.ERR_F32, max_unstable=1)
    st = parity.stepwise_parity(g, m, 0, 3, long_p[:60], 3, 0.8, 17, 1e-4, max_len=128)
    parity.check_stats(st, 3, parity.ERR_F32, max_unstable=1)
    g.close()


@pytest.mark.parametrize("w", [TINY, MFMA_HD128], ids=["fp32", "mfma"])
def test_run_iterations_equals_stepwise_calls(w):
    """pass_run_iterations issues iteration i+1 before it has read the report of iteration i (it
    works with an upper bound of the sequence lengths meanwhile); the sequences must end up exactly
    where the same number of draft / verify calls, each synchronised, leaves them: same lengths,
    same token counts, same logits of the last two calls.  High temperature, so accepted drafts
    make the lengths grow unevenly; two ragged slots; enough iterations to cross page boundaries."""
    w = synth.scaled(w, k=3)
    W = synth.make_weights(w.shape, 5, 3, 1.0)
    page = 64 if w.shape.head_dim == 128 else 16
    prompts = [np.random.default_rng(i).integers(0, w.shape.vocab, n).astype(np.int32) for i, n in enumerate((9, 58))]
    res = []
    for mode in ("iterations", "stepwise"):
        g = _gpu(w.shape, W, 3, max_slots=2, max_seq_len=256, page_size=page)
        for i, p in enumerate(prompts):
            g.prefill(i, p, seq_id=50 + i)
        if mode == "iterations":
            st = g.run_iterations([0, 1], 17, 3.0, 1234)
            assert st["iterations"] == 34 and st["drafts_proposed"] == 3 * 34
        else:
            acc = 0
            for _ in range(17):
                g.draft([0, 1], 3.0, 1234)
                a, _t = g.verify([0, 1], 3.0, 1234)
                acc += int(a.sum())
        res.append((g.seq_len(0), g.seq_len(1), g.get_logits(0, 0), g.get_logits(1, 1),
                    st["drafts_accepted"] if mode == "iterations" else acc))
        g.close()
    assert res[0][0] == res[1][0] and res[0][1] == res[1][1]
    assert np.array_equal(res[0][2], res[1][2]) and np.array_equal(res[0][3], res[1][3])
    assert res[0][4] == res[1][4] and res[0][4] > 0


@pytest.mark.parametrize("w", [TINY, MFMA_HD128], ids=["fp32", "mfma"])
def test_generate_equals_stepwise_calls(w):
    """pass_generate runs Algorithm 1's loop with the report of an iteration read one iteration late
    (it issues the next one blind only while some slot needs it whatever the one in flight yields):
    tokens, lengths and the number of iterations must be those of synchronised draft / verify
    calls that stop each slot at its target.  High temperature (accepted drafts: uneven progress,
    so one slot finishes first and is frozen while the other goes on); two calls in a row, the
    second continuing after the tokens the first one made beyond its target."""
    w = synth.scaled(w, k=3)
    W = synth.make_weights(w.shape, 5, 3, 1.0)
    page = 64 if w.shape.head_dim == 128 else 16
    prompts = [np.random.default_rng(i).integers(0, w.shape.vocab, n).astype(np.int32) for i, n in enumerate((9, 58))]
    g = _gpu(w.shape, W, 3, max_slots=2, max_seq_len=256, page_size=page)
    for i, p in enumerate(prompts):
        g.prefill(i, p, seq_id=50 + i)
    out_a, st_a = g.generate([0, 1], 37, 3.0, 1234)
    len_a = [g.seq_len(i) for i in (0, 1)]
    out_b, st_b = g.generate([0, 1], 11, 3.0, 1234)
    len_b = [g.seq_len(i) for i in (0, 1)]
    all_toks = [g.get_tokens(i, 0, len_b[i][1]) for i in (0, 1)]
    g.close()
    # the same with synchronised calls: a slot steps while it is short of its target
    g = _gpu(w.shape, W, 3, max_slots=2, max_seq_len=256, page_size=page)
    for i, p in enumerate(prompts):
        g.prefill(i, p, seq_id=50 + i)
    toks = {0: [], 1: []}
    iters = []
    for target in (37, 11):
        start = {i: len(toks[i]) for i in (0, 1)}
        n_it = 0
        while True:
            live = [i for i in (0, 1) if len(toks[i]) - start[i] < target]
            if not live:
                break
            first, _d = g.draft(live, 3.0, 1234)
            a, out = g.verify(live, 3.0, 1234)
            for j, i in enumerate(live):
                toks[i] += [int(first[j])] + [int(t) for t in out[j, :a[j] + 1]]
            n_it += len(live)
        iters.append(n_it)
        if target == 37:
            assert [g.seq_len(i) for i in (0, 1)] == len_a
            for i in (0, 1):
                assert np.array_equal(out_a[i], toks[i][:37])
    assert [g.seq_len(i) for i in (0, 1)] == len_b
    for i in (0, 1):
        assert np.array_equal(all_toks[i], toks[i])                      # every token, those beyond a target included
        assert np.array_equal(out_b[i], toks[i][len_a[i][1]:len_a[i][1] + 11])  # the second call continues after them
    assert [st_a["iterations"], st_b["iterations"]] == iters
    assert st_a["tokens_out"] == 74 and st_a["drafts_accepted"] > 0
    g.close()


def test_run_iterations_stops_exactly_where_stepwise_calls_stop():
    """Near the end of a sequence's room the look-ahead bound of pass_run_iterations no longer fits
    and it falls back to exact lengths: it must run as many iterations as synchronised calls can,
    report the capacity error, and leave the same state."""
    from paper_2311_13581_amd import binding
    w = synth.scaled(TINY, k=3)
    W = synth.make_weights(w.shape, 5, 3, 1.0)
    prompt = np.random.default_rng(1).integers(0, w.shape.vocab, 9).astype(np.int32)
    state = []
    for mode in ("iterations", "stepwise"):
        g = _gpu(w.shape, W, 3, max_seq_len=64)
        g.prefill(0, prompt, seq_id=3)
        with pytest.raises(binding.PassError) as e:
            if mode == "iterations":
                g.run_iterations([0], 1000, 3.0, 99)
            else:
                for _ in range(1000):
                    g.draft([0], 3.0, 99)
                    g.verify([0], 3.0, 99)
        assert e.value.code == -3
        state.append(g.seq_len(0))
        g.close()
    assert state[0] == state[1] and state[0][0] + 2 + 3 > 64


# ---------------------------------------------------------------------------------------------
# Algorithm 2 (appendix): two-model speculative sampling through pass_sps_iteration
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("which", ["fp32", "mfma"])
@pytest.mark.parametrize("temp", [0.0, 0.9])
def test_two_model_speculative_sampling_stepwise(which, temp):
    """A target context and a drafter context (a smaller model of the same vocabulary) against the
    oracle's Algorithm 2: the drafter's k sequential rows and tokens, the target's validation logits,
    accept bits, residual / extra token and both sequences' lengths, every iteration."""
    k = 3
    if which == "fp32":
        shape_t, page = TINY.shape, 16
        shape_d = synth.ModelShape(1, 128, 2, 64, 256, shape_t.vocab, dtype=synth.F32)
    else:
        shape_t, page = MFMA_HD128.shape, 64
        shape_d = synth.ModelShape(1, 256, 2, 128, 512, shape_t.vocab, dtype=synth.BF16)
    Wt = synth.make_weights(shape_t, 71, k, 5.0)
    Wd = synth.make_weights(shape_d, 72, 1, 5.0)
    gt = _gpu(shape_t, Wt, k, max_seq_len=256, page_size=page)
    gd = _gpu(shape_d, Wd, 0, max_seq_len=256, page_size=page)
    mt, md = O.Model(shape_t, Wt, k), O.Model(shape_d, Wd, 0)
    prompt = np.random.default_rng(17).integers(0, shape_t.vocab, 41).astype(np.int32)
    st = parity.sps_parity(gt, gd, mt, md, 0, 6, prompt, 12, temp, 2027, parity.LOGIT_TOL[shape_t.dtype])
    print(which, temp, st)
    parity.check_stats(st, 12, parity.ERR_F32 if which == "fp32" else parity.ERR_BF16_SMALL)
    gt.close()
    gd.close()


def test_two_model_speculative_sampling_with_the_target_as_drafter_accepts_everything():
    """The same model in both contexts: draft t is drawn from the distribution validation row t-1
    scores it with, so every draft is accepted and each iteration adds k + 1 tokens (which also
    exercises the extra drafter call that makes the last draft's cache row); a batch of two slot
    pairs; greedy, where the tokens are the target's greedy decoding."""
    w, k = TINY, 4
    W = synth.make_weights(w.shape, 9, k, 4.0)
    gt = _gpu(w.shape, W, k, max_slots=2, max_seq_len=256)
    gd = _gpu(w.shape, W, 0, max_slots=2, max_seq_len=256)
    prompts = [np.random.default_rng(i).integers(0, w.shape.vocab, n).astype(np.int32) for i, n in enumerate((12, 30))]
    for i, p in enumerate(prompts):
        gt.prefill(i, p, seq_id=i)
        gd.prefill(i, p, seq_id=i)
    toks = {0: [], 1: []}
    for _ in range(5):
        drafts, a, out = gt.sps_iteration(gd, [0, 1], [0, 1], 0.8, 11)
        assert list(a) == [k, k]
        for i in (0, 1):
            assert np.array_equal(out[i, :k], drafts[i])
            toks[i] += [int(x) for x in out[i]]
    for i in (0, 1):
        assert gt.seq_len(i)[0] == gd.seq_len(i)[0] == len(prompts[i]) - 1 + 5 * (k + 1)
        assert np.array_equal(gt.get_tokens(i, 0, 5 * (k + 1)), toks[i])
    # greedy: Algorithm 2's output is the target's own greedy decoding
    m = O.Model(w.shape, W, k)
    gt.prefill(0, prompts[0], seq_id=0)
    gd.prefill(0, prompts[0], seq_id=0)
    got = []
    for _ in range(4):
        _d, a, out = gt.sps_iteration(gd, [0], [0], 0.0, 11)
        got += [int(x) for x in out[0, :a[0] + 1]]
    s = m.sequence(256, seq_id=0)
    s.prefill(prompts[0])
    assert np.array_equal(got, s.generate_ar(len(got), 0.0, 11))
    gt.close()
    gd.close()
