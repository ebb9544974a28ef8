"""CPU-only checks of the C ABI: the shared library loads, exports every
function that include/moetuner.h declares, answers its size queries, and turns
bad scalar arguments into error codes (validation happens before any GPU call,
so no GPU is needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        for m in re.finditer(r"\b(moe_[a-z0-9_]+)\s*\(", text):
            names.add(m.group(1))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    from paper_2502_06643_amd import binding as B
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(B.lib(), n), f"{n} is declared in include/ but not exported"
        assert n in B.EXPORTS
    for n in B.EXPORTS:                      # and the binding names nothing the header lacks
        assert n in names
    assert "gfx950" in B.moe_version()


def test_python_binding_has_the_same_names():
    from paper_2502_06643_amd import binding as B
    for n in declared_functions():
        assert callable(getattr(B, n)), n


def test_size_queries():
    from paper_2502_06643_amd import binding as B
    assert B.moe_dispatch_workspace_bytes(4096, 8, 2) >= 8 * 8 * 4
    assert B.moe_dispatch_workspace_bytes(0, 8, 2) > 0
    assert B.moe_packed_weights_bytes(8, 4096, 14336, B.MOE_BF16) >= 8 * 3 * 4096 * 14336 * 2
    assert B.moe_packed_weights_bytes(8, 128, 256, B.MOE_F32) == 8 * 3 * 128 * 256 * 4
    assert B.moe_packed_weights_bytes(8, 100, 256, B.MOE_BF16) == 0          # d % 64 != 0 -> unsupported
    assert B.moe_ffn_workspace_bytes(8192, 4096, 14336, 8, B.MOE_BF16) >= 8192 * 14336 * 2


def test_bad_scalars_are_rejected_without_touching_the_gpu():
    from paper_2502_06643_amd import binding as B
    L = B.lib()
    one = ctypes.c_void_p(16)            # never dereferenced: validation fails first
    assert L.moe_topk_gate(one, -1, 8, 2, one, one, None) == -1
    assert b"T=" in L.moe_last_error()
    assert L.moe_topk_gate(one, 4, 8, 9, one, one, None) == -1
    assert L.moe_topk_gate(one, 4, 300, 2, one, one, None) == -1
    assert L.moe_topk_gate(None, 4, 8, 2, one, one, None) == -1
    assert L.moe_topk_gate(ctypes.c_void_p(20), 4, 8, 2, one, one, None) == -1     # misaligned
    assert L.moe_dispatch(None, 0, one, 4, 8, 8, 2, one, 0, None, one, one, one, one, one, one, one, 1 << 20, None) == -1   # G=0
    assert L.moe_dispatch(one, 1, one, 4, 12, 8, 2, one, 4, one, one, one, one, one, one, one, one, 1 << 20, None) == -1    # row not 16B multiple
    assert L.moe_dispatch(None, 1, one, 4000, 8, 8, 2, one, 4, None, one, one, one, one, one, one, one, 16, None) == -3     # workspace
    # the entry point with built-in scratch: same scalar checks, and sizes beyond its 256 KiB buffer are refused before any GPU call
    assert L.moe_dispatch_noalloc(None, 0, one, 4, 8, 8, 2, one, 0, None, one, one, one, one, one, one, None) == -1          # G=0
    assert L.moe_dispatch_static_scratch_bytes() == 256 << 10
    assert L.moe_dispatch_workspace_bytes(1 << 20, 256, 2) > L.moe_dispatch_static_scratch_bytes()
    assert L.moe_dispatch_noalloc(None, 1, one, 1 << 20, 8, 256, 2, one, 4, None, one, one, one, one, one, one, None) == -3
    assert b"moe_dispatch_noalloc" in L.moe_last_error() and b"scratch" in L.moe_last_error()
    assert L.moe_expert_ffn_grouped(one, 1, 8, 100, 256, 8, one, one, one, one, 0, one, one, 1 << 30, None) == -2           # bf16 d%64
    assert L.moe_expert_ffn_grouped(one, 1, 8, 128, 256, 8, one, one, one, one, -2, one, one, 1 << 30, None) == -1
    assert L.moe_expert_ffn_grouped(one, 1, 8, 128, 256, 8, one, one, one, one, 0, one, one, 16, None) == -3
    assert L.moe_combine(one, 1, one, one, one, None, 0, 4, 64, 8, 2, one, None) == -1                                   # placement needed
    assert L.moe_combine(one, 7, one, one, one, one, 0, 4, 64, 8, 2, one, None) == -1                                    # dtype
    assert L.moe_transition_counts(one, one, 4, 2, 2, 8, 8, None, None) == -1
    assert L.moe_transition_counts(one, one, 4, 9, 2, 8, 8, one, None) == -1
    assert L.moe_expert_ffn_segments(one, 1, 8, 128, 256, 8, one, -1, one, one, one, one, one, 1 << 30, None) == -1         # n_seg < 0
    assert L.moe_expert_ffn_segments(one, 1, 8, 128, 256, 8, one, 257, one, one, one, one, one, 1 << 30, None) == -1        # too many segments
    assert L.moe_expert_ffn_segments(one, 1, 8, 128, 256, 8, one, 4, one, one, one, one, one, 16, None) == -3               # workspace
    assert L.moe_expert_ffn_segments(None, 1, 8, 128, 256, 8, None, 0, None, None, None, None, None, 0, None) == 0          # no segment: nothing to do
    assert L.moe_topk_gate_norm(one, 4, 8, 2, 5, one, one, None) == -1                                                      # unknown norm
    assert L.moe_transition_counts_pairs(one, one, 4, 2, 2, 8, 8, 3, one, None) == -1                                       # unknown pair mode
    assert L.moe_receive_segments(one, one, 8, 4, 4, 8, one, one, one, None, None, None) == -1                              # dest outside [0,G)
    assert L.moe_receive_segments(one, one, 8, 4, 0, 257, one, one, one, None, None, None) == -1                            # more segments than the segment FFN takes
    assert L.moe_receive_segments(one, one, 8, 4, 0, 8, one, None, one, None, None, None) == -1                             # NULL table
    # the fused router and the placement evaluators
    assert L.moe_router_gate(one, 1, one, None, -1, 128, 8, 2, None, one, one, None) == -1                                  # T < 0
    assert L.moe_router_gate(one, 1, one, None, 4, 100, 8, 2, None, one, one, None) == -2                                   # bf16 needs d % 64 == 0
    assert L.moe_router_gate(one, 1, one, None, 4, 128, 8, 9, None, one, one, None) == -1                                   # k > E
    assert L.moe_router_gate(one, 1, None, None, 4, 128, 8, 2, None, one, one, None) == -1                                  # no packed router
    assert L.moe_router_packed_bytes(100, 8, 1) == 0 and L.moe_router_packed_bytes(128, 8, 1) >= 128 * 8 * 2
    assert L.moe_pack_router(one, 128, 8, 1, one, 16, None) == -3                                                           # packed buffer too small
    assert L.moe_accumulate_counts(one, 0, one, None) == -1
    assert L.moe_accumulate_counts(None, 8, one, None) == -1
    assert L.moe_placement_loads(one, one, 8, 0, one, None, None) == -1                                                     # G = 0
    assert L.moe_placement_loads(one, None, 8, 4, one, None, None) == -1
    assert L.moe_placement_traffic(one, one, one, 8, 300, 4, one, None, None, None) == -1                                   # E_l1 too large
    assert L.moe_placement_traffic(one, one, one, 8, 8, 4, None, None, None, None) == -1                                    # no output
    assert L.moe_timing_begin(1, 0) == -1
    # empty batches are fine and enqueue nothing
    assert L.moe_topk_gate(None, 0, 8, 2, None, None, None) == 0
    assert L.moe_combine(None, 1, None, None, None, None, -1, 0, 64, 8, 2, None, None) == 0
    assert L.moe_transition_counts(None, None, 0, 2, 2, 8, 8, one, None) == 0


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    """The product path has no fallback: importing the binding without the
    shared object is an ImportError."""
    import importlib.util
    src = os.path.join(ROOT, "paper_2502_06643_amd", "binding.py")
    dst = tmp_path / "binding_copy.py"
    dst.write_text(open(src).read())
    spec = importlib.util.spec_from_file_location("binding_copy", dst)
    mod = importlib.util.module_from_spec(spec)
    with pytest.raises(ImportError):
        spec.loader.exec_module(mod)
