"""pass_draft_static (the entry point that allocates nothing: its attention partials live in a
static device array of the library) against pass_draft, through the C ABI: same tokens and the
same logits, bit for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from paper_2311_13581_amd import synth

pytestmark = pytest.mark.gpu

MFMA = synth.ModelShape(3, 512, 4, 128, 1184, 1008, dtype=synth.BF16)
TINY = synth.WORKLOADS["tiny_fp32_greedy"].shape


@pytest.mark.parametrize("shape,page", [(MFMA, 64), (TINY, 16)], ids=["mfma", "fp32"])
def test_static_scratch_draft_equals_draft(shape, page):
    from paper_2311_13581_amd import binding
    k = 4
    W = synth.make_weights(shape, 41, k, 6.0)
    rng = np.random.default_rng(9)
    # first call: two slots, 10 rows, 300 and 70 cached keys (three splits); second: one slot, 5 rows, 20 keys
    prompts = [rng.integers(0, shape.vocab, n).astype(np.int32) for n in (301, 71, 21)]
    res = {}
    for static in (False, True):
        g = binding.Pass(binding.make_config(shape, k, 3, 512, page), {"graph": 1})
        g.load_weights(W)
        for i, p in enumerate(prompts):
            g.prefill(i, p, seq_id=i)
        out = []
        for slots in ([0, 1], [2]):
            first, drafts = g.draft(slots, 0.9, 77, static=static)
            out.append((first.copy(), drafts.copy(), [g.get_logits(s, 0) for s in slots], [g.seq_len(s) for s in slots]))
            g.verify(slots, 0.9, 77)
        # and once more on the grown sequences, static and ordinary calls interleaved on one context
        first, drafts = g.draft([0, 1, 2], 0.9, 77, static=static)
        out.append((first.copy(), drafts.copy(), [g.get_logits(s, 0) for s in (0, 1, 2)], None))
        res[static] = out
        g.close()
    for a, b in zip(res[False], res[True]):
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        for la, lb in zip(a[2], b[2]):
            assert np.array_equal(la, lb)
        assert a[3] == b[3]
    assert np.abs(res[True][0][2][0]).max() > 0.1


def test_static_scratch_rejects_calls_beyond_its_size():
    """8 MiB hold the partials of 15 rows of a 32-head model: a 20-row call is refused with a
    capacity error before anything runs, and the slots stay usable."""
    from paper_2311_13581_amd import binding
    shape = synth.ModelShape(1, 256, 32, 128, 512, 512, dtype=synth.BF16)
    W = synth.make_weights(shape, 3, 4, 4.0)
    g = binding.Pass(binding.make_config(shape, 4, 4, 128, 64))
    g.load_weights(W)
    for i in range(4):
        g.prefill(i, [1 + i, 2, 3], seq_id=i)
    with pytest.raises(binding.PassError) as e:
        g.draft([0, 1, 2, 3], 0.0, 1, static=True)
    assert e.value.code == -3 and "static scratch" in str(e.value)
    a, _ = g.draft([0, 1, 2], 0.0, 1, static=True)   # 15 rows fit
    g.verify([0, 1, 2], 0.0, 1)
    b, _ = g.draft([3], 0.0, 1)
    assert a.shape == (3,) and b.shape == (1,)
    g.close()
