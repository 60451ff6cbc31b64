"""Host-side checks that need no GPU: the library loads, exports every declared symbol, and sizes arenas."""
import ctypes as C
import os
import re

from paper_2311_13581_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "pass.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pass_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = _declared()
    assert {"pass_load_weights", "pass_prefill", "pass_draft", "pass_verify", "pass_generate"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.SYMBOLS) == names


def test_arena_size_and_config_validation():
    lib = binding.load_library()
    w = synth.WORKLOADS["7b_k4_greedy"]
    cfg = binding.make_config(w.shape, 4, 1, 1024)
    n = lib.pass_arena_bytes(C.byref(cfg))
    weights = w.shape.n_params_streamed * 2
    assert weights < n < weights + 3 * 2 ** 30  # weights + embedding table + K/V + workspaces
    for field, bad in [("head_dim", 96), ("k", 16), ("page_size", 24), ("max_slots", 99), ("dtype", 3),
                       ("d_model", 4100), ("max_seq_len", 3)]:
        c2 = binding.make_config(w.shape, 4, 1, 1024)
        setattr(c2, field, bad)
        assert lib.pass_arena_bytes(C.byref(c2)) == 0, field


def test_struct_layouts_match_header_sizes():
    assert C.sizeof(binding.PassConfig) == 14 * 4
    assert C.sizeof(binding.PassSampling) == 16
    assert C.sizeof(binding.PassStats) == 48
    assert C.sizeof(binding.PassWeights) == 13 * 8
    assert C.sizeof(binding.PassAdamW) == 5 * 4


def test_calls_without_a_context_are_rejected():
    """The entry points added for training and the batched prompt pass return PASS_EINVAL for a null context
    (or 0 bytes) before they touch the device."""
    lib = binding.load_library()
    assert lib.pass_train_bytes(None) == 0
    assert lib.pass_train_begin(None, None, 0, 0) == -1
    assert lib.pass_train_step(None, None, 0, None, None, None) == -1
    assert lib.pass_train_read(None, 0, None) == -1
    assert lib.pass_train_resume(None, None, None, None, 0) == -1
    assert lib.pass_prefill_batch(None, None, None, None, None, 0) == -1


def test_attention_grid_covers_every_shorter_group():
    """The split plan of the matrix-core attention is not monotone in the key count (32 heads: 3072 keys
    give 24 splits, 3073 give 13).  A launch serves groups of several lengths and, in the pipelined
    loop, only knows an upper bound of them: its grid must be at least as wide as the plan of every
    length up to that bound, and the plan itself must cover all keys with at most 32 splits."""
    lib = binding.load_library()
    ns, ch, grid = C.c_int32(), C.c_int32(), C.c_int32()
    for heads in (1, 4, 8, 32, 40, 64):
        widest = 0
        plans = []
        for n in range(1, 16500):
            assert lib.pass_attention_plan(heads, n, C.byref(ns), C.byref(ch), C.byref(grid)) == 0
            assert 1 <= ns.value <= 32 and ch.value % 128 == 0
            assert (ns.value - 1) * ch.value < n <= ns.value * ch.value  # every key in exactly one split, none empty
            widest = max(widest, ns.value)
            assert grid.value == widest, (heads, n)  # the running maximum: no shorter group has more splits
            plans.append(ns.value)
        if heads == 32:
            assert plans[3072 - 1] == 24 and plans[3073 - 1] == 13  # the drop the grid width must survive
        if heads == 40:
            assert plans[2432 - 1] == 19 and plans[2433 - 1] == 10
    assert lib.pass_attention_plan(0, 5, None, None, None) == -1
    assert lib.pass_attention_plan(4, 0, None, None, None) == -1


def test_prompt_packing_plan_covers_every_row_once():
    """How pass_prefill_batch packs prompts into tiled passes: every row of every prompt lies in exactly one
    segment, a prompt's segments follow each other in position order (a later pass reads what an earlier
    one cached), segments start on blocks of 128 rows, never overlap inside a pass, never exceed it, and
    passes are filled in order (a new pass only when the block cursor has reached the pass's end)."""
    import numpy as np
    lib = binding.load_library()
    rng = np.random.default_rng(0)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    cases = [(2048, [170, 1075, 1235, 968, 773, 1159, 474, 1774]), (128, [1, 2, 129, 130, 500]), (256, [257, 257, 1, 128, 129])]
    cases += [(int(cap), rng.integers(1, 3000, int(n)).tolist()) for cap, n in zip(rng.choice([128, 384, 1024, 2048], 40), rng.integers(1, 12, 40))]
    for cap, lens in cases:
        lens_a = np.array(lens, dtype=np.int32)
        n_segs = C.c_int32()
        assert lib.pass_prefill_plan(cap, ip(lens_a), len(lens), 0, None, C.byref(n_segs)) in (0, -3)
        segs = np.zeros((max(1, n_segs.value), 5), dtype=np.int32)
        assert lib.pass_prefill_plan(cap, ip(lens_a), len(lens), n_segs.value, ip(segs), C.byref(n_segs)) == 0
        segs = segs[:n_segs.value]
        covered = [0] * len(lens)
        last_pass, used = -1, {}
        for ps, prompt, pos0, rows, base in segs.tolist():
            assert rows >= 1 and base % 128 == 0 and base + rows <= cap
            assert pos0 == covered[prompt]  # in position order, nothing skipped
            covered[prompt] += rows
            assert ps in (last_pass, last_pass + 1)
            if ps != last_pass:
                assert last_pass < 0 or used[last_pass] >= cap  # the previous pass was full (in whole blocks)
                last_pass, used[ps] = ps, 0
            assert base == used[ps]  # next free block: no overlap, no hole
            used[ps] = (base + rows + 127) // 128 * 128
        assert covered == [n - 1 for n in lens]
    one = np.array([5], dtype=np.int32)
    assert lib.pass_prefill_plan(100, ip(one), 1, 0, None, C.byref(n_segs)) == -1  # not a multiple of 128
    assert lib.pass_prefill_plan(128, ip(np.array([0], dtype=np.int32)), 1, 0, None, C.byref(n_segs)) == -1
