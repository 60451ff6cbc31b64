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
