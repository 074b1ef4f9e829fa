"""The C-ABI library loads, exports every symbol include/moe.h declares, and
its host-only entry points behave (no kernel is launched in this file)."""
import ctypes as C
import os
import re

import pytest

import paper_2504_14960_amd as moe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe.h")
GOLDEN = os.path.join(ROOT, "tests", "golden", "capacity_eq4.txt")


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_stage_calls():
    syms = _declared_symbols()
    for name in ("moe_router_topk", "moe_permute", "moe_grouped_gemm_swiglu", "moe_unpermute_combine",
                 "moe_layer_forward", "moe_last_error"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    L = C.CDLL(moe.lib_path())
    for name in _declared_symbols():
        assert hasattr(L, name), f"{name} declared in moe.h but not exported"


def test_capacity_matches_equation_four_values():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    for cf, T, K, E, Cap in rows:
        assert moe.capacity_from_factor(float(cf), int(T), int(K), int(E)) == int(Cap)
    assert moe.capacity_from_factor(0.0, 100, 2, 8) == 0


def test_max_rows_and_workspace_sizes():
    assert moe.max_rows(8192, 2, 8, 0) == 16384
    assert moe.max_rows(32768, 6, 64, 3072) == 196608
    assert moe.max_rows(100, 2, 4, 10) == 40
    assert moe.permute_workspace_bytes(8192, 2, 8) >= 16 * 8 * 4
    lay = moe.layer_workspace_layout(256, 128, 8, 2, 256, 0, 0, moe.MOE_F32)
    offs = list(lay.values())
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert moe.layer_workspace_bytes(256, 128, 8, 2, 256, 0, 0, moe.MOE_F32) >= offs[-1]
    # moe_workspace_bytes is moe_layer_workspace_bytes for a layer without a shared expert
    for T, H, E, K, F, cap, dt in ((256, 128, 8, 2, 256, 0, moe.MOE_F32), (8192, 6144, 8, 2, 16384, 0, moe.MOE_BF16),
                                   (32768, 4096, 64, 6, 1408, 3072, moe.MOE_BF16)):
        assert moe.workspace_bytes(T, H, E, K, F, cap, dt) == moe.layer_workspace_bytes(T, H, E, K, F, 0, cap, dt) > 0


def test_clock_sample_pointer_is_checked_on_the_host():
    import ctypes
    L = moe.lib()
    assert L.moe_gemm_clock_sample(ctypes.c_void_p(0)) == 0          # NULL switches the sampling off
    assert L.moe_gemm_clock_sample(ctypes.c_void_p(12)) != 0         # not 8-byte aligned: refused, nothing stored
    assert b"aligned" in L.moe_last_error()
    assert L.moe_gemm_clock_sample(ctypes.c_void_p(0)) == 0


def test_argument_errors_are_reported_on_the_host():
    L = moe.lib()
    # K > E
    st = L.moe_router_topk(None, None, None, None, 16, 64, 4, 5, 0, moe.MOE_BF16, None, None, None)
    assert st == 1 and b"exceeds E" in L.moe_last_error()
    # E above the limit
    st = L.moe_router_topk(None, None, None, None, 16, 64, 1000, 2, 0, moe.MOE_BF16, None, None, None)
    assert st == 2
    # H not a multiple of the vector width
    st = L.moe_permute(None, None, 16, 12, 4, 2, 0, moe.MOE_BF16, None, None, None, None, None, None, 0, None)
    assert st == 2
    # NULL outputs
    st = L.moe_permute(None, None, 16, 64, 4, 2, 0, moe.MOE_BF16, None, None, None, None, None, None, 0, None)
    assert st == 1 and b"NULL" in L.moe_last_error()
    # misaligned pointer
    st = L.moe_unpermute_combine(C.c_void_p(0x1004), C.c_void_p(0x1000), C.c_void_p(0x1000), None,
                                 4, 64, 2, 8, moe.MOE_BF16, C.c_void_p(0x1000), None)
    assert st == 1 and b"aligned" in L.moe_last_error()
    # workspace too small
    st = L.moe_layer_forward(*([C.c_void_p(0x1000)] * 3), *([C.c_void_p(0x1000)] * 3), None, None, None,
                             16, 64, 4, 2, 64, 0, 1, 0, moe.MOE_BF16, C.c_void_p(0x1000),
                             C.c_void_p(0x1000), 16, None)
    assert st == 3 and b"workspace" in L.moe_last_error()
    # unknown option
    with pytest.raises(moe.MoeError):
        moe.set_option("no_such_option", 1)
    # T == 0 is legal and launches nothing
    st = L.moe_router_topk(None, None, None, None, 0, 64, 4, 2, 0, moe.MOE_BF16, None, None, None)
    assert st == 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_14960_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in src.lower(), f"{fn} mentions the oracle"


def test_fp8_delayed_scale_closed_forms():
    assert moe.fp8_delayed_scale([1.0, 2.0, 0.5]) == 224.0            # 448 / largest amax
    assert moe.fp8_delayed_scale([1.0, 2.0, 0.5], 1) == 112.0         # one power of two of headroom
    assert moe.fp8_delayed_scale([0.0, 0.0]) == 1.0 and moe.fp8_delayed_scale([]) == 1.0   # nothing recorded yet
    assert moe.fp8_delayed_scale([float("inf"), 4.0]) == 112.0        # non-finite entries ignored
    assert moe.fp8_delayed_scale([float("nan"), 8.0]) == 56.0
