"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-only entry points (sizes, cost model, error strings) behave as documented.  Nothing
here launches a kernel."""
import ctypes
import os
import re
from ctypes import byref, c_size_t

import pytest

from paper_2305_17469_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gt_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(B.lib, n), n
    assert sorted(B.EXPORTS) == names


def test_status_strings_and_version():
    assert B.lib.gt_status_string(0) == b"GT_OK"
    assert B.lib.gt_status_string(3) == b"GT_ERR_WORKSPACE"
    assert b"gfx950" in B.lib.gt_version()


def test_plan_size_validation():
    n = c_size_t()
    assert B.lib.gt_graph_plan_size(10, 10, 50, 0, byref(n)) == B.GT_OK and n.value > 0
    small = n.value
    assert B.lib.gt_graph_plan_size(1 << 21, 1 << 21, 55_000_000, 1, byref(n)) == B.GT_OK and n.value > small
    assert B.lib.gt_graph_plan_size(-1, 10, 50, 0, byref(n)) == 1          # INVALID_ARG
    assert B.lib.gt_graph_plan_size(10, 10, 1 << 31, 0, byref(n)) == 2      # UNSUPPORTED: int32 indices
    assert B.lib.gt_graph_plan_size(10, 10, (1 << 31) - 1024, 0, byref(n)) == 2
    assert B.lib.gt_graph_plan_size(10, 10, (1 << 31) - 1025, 0, byref(n)) == B.GT_OK
    assert B.lib.gt_graph_plan_size(10, 10, 50, 0, None) == 1
    assert b"gt_graph_plan_size" in B.lib.gt_last_error()
    assert B.lib.gt_graph_plan_size(0, 0, 0, 0, byref(n)) == B.GT_OK        # empty graph is valid


def test_null_handles_are_rejected_without_touching_the_gpu():
    n = c_size_t()
    assert B.lib.gt_aggregate_ws_size(None, 16, byref(n)) == 1
    assert B.lib.gt_aggregate_fwd(None, 0, 0, 16, None, 16, None, 16, None, 0, None) == 1
    assert B.lib.gt_aggregate_bwd(None, 0, 0, 16, None, 16, None, 16, None, 0, None) == 1
    d = B.make_desc("sum", "f32", True, 8, 8)
    assert B.lib.gt_layer_decide(None, byref(d), None, None) == 1
    assert B.lib.gt_layer_ws_size(None, byref(d), None, None) == 1
    assert B.lib.gt_graph_outputs(None, None, None, None, None, None) == 1
    assert B.lib.gt_graph_destroy(None) == 0
    # combine: argument checks come before any launch
    assert B.lib.gt_combine(0, 0, 0, -1, 4, 4, None, 4, None, 4, None, 0, None, 4, 0, None, 0, None) == 1
    assert B.lib.gt_combine(0, 0, 0, 4, 4, 4, None, 4, None, 4, None, 0, None, 4, 0, None, 0, None) == 1   # C null
    assert B.lib.gt_combine(7, 0, 0, 4, 4, 4, None, 4, None, 4, None, 0, None, 4, 0, None, 0, None) == 1   # dtype
    assert B.lib.gt_combine(0, 0, 0, 0, 4, 4, None, 4, None, 4, None, 0, None, 4, 0, None, 0, None) == 0   # M == 0: no-op


def test_combine_ws_size_only_for_weight_gradient_shape():
    n = c_size_t()
    assert B.lib.gt_combine_ws_size(0, 0, 0, 1 << 18, 128, 602, byref(n)) == 0 and n.value == 0
    assert B.lib.gt_combine_ws_size(0, 1, 0, 602, 128, 1 << 18, byref(n)) == 0 and n.value >= 602 * 128 * 4 * 2


def test_cost_benefit_formulas_with_the_papers_constants():
    # Table "DKP cost model" with the coefficients printed beside it, evaluated by hand for
    # n_src 29,000, n_dst 8,000, n_edge 60,000, n_feat 4,353, n_hid 64.
    c = B.gt_cost_coeffs(6e-5, 1e-5, 1e-3, 1e-12, 1e-7, 4e-6, 1e-6, 1e-8)
    r = B.gt_cost_benefits(c, 29000, 8000, 60000, 4353, 64)
    assert r["aggr_fwd"] == pytest.approx(21000 * (6e-5 * 64 * 4353 + 1e-5 * 64), rel=1e-12)
    assert r["aggr_bwd"] == pytest.approx(21000 * (1e-7 * 64 * 4353 + 4e-6 * 4353), rel=1e-12)
    assert r["comb_fwd"] == pytest.approx(4289 * (1e-3 * 60000 + 1e-12 * 8000), rel=1e-12)
    assert r["comb_bwd"] == pytest.approx(4289 * (1e-6 * 60000 + 1e-8 * 29000), rel=1e-12)
    # first layer: the aggr-first BWP reduction factor becomes n_src
    r1 = B.gt_cost_benefits(c, 29000, 8000, 60000, 4353, 64, first_layer=True)
    assert r1["aggr_bwd"] == pytest.approx(29000 * (1e-7 * 64 * 4353 + 4e-6 * 4353), rel=1e-12)
    assert r1["aggr_fwd"] == r["aggr_fwd"] and r1["comb_bwd"] == r["comb_bwd"]


def test_cost_set_get_roundtrip_and_validation():
    old = [B.gt_cost_get_dtype(d) for d in ("f32", "bf16")]
    try:
        c = B.gt_cost_coeffs(1, 2, 3, 4, 5, 6, 7, 8)
        B.gt_cost_set(c)                                   # installs the set for every data type
        for g in (B.gt_cost_get(), B.gt_cost_get_dtype("f32"), B.gt_cost_get_dtype("bf16")):
            assert [getattr(g, f[0]) for f in g._fields_] == [1, 2, 3, 4, 5, 6, 7, 8, 0]
        B.gt_cost_set_dtype("bf16", B.gt_cost_coeffs(8, 7, 6, 5, 4, 3, 2, 1, 3e-6))   # one data type only
        g = B.gt_cost_get_dtype("bf16")
        assert [getattr(g, f[0]) for f in g._fields_] == [8, 7, 6, 5, 4, 3, 2, 1, 3e-6]
        g = B.gt_cost_get()
        assert [getattr(g, f[0]) for f in g._fields_] == [1, 2, 3, 4, 5, 6, 7, 8, 0]
        assert B.lib.gt_cost_set(byref(B.gt_cost_coeffs(1, 2, 3, 4, 5, 6, 7, 8, -1e-6))) == 1   # negative floor
        bad = B.gt_cost_coeffs(-1, 2, 3, 4, 5, 6, 7, 8)
        assert B.lib.gt_cost_set(byref(bad)) == 1
        assert B.lib.gt_cost_set_dtype(1, byref(bad)) == 1
        bad = B.gt_cost_coeffs(float("nan"), 2, 3, 4, 5, 6, 7, 8)
        assert B.lib.gt_cost_set(byref(bad)) == 1
        assert B.lib.gt_cost_set_dtype(7, byref(c)) == 1   # unknown data type
        assert B.lib.gt_cost_get_dtype(7, byref(c)) == 1
    finally:
        B.gt_cost_set_dtype("f32", old[0])
        B.gt_cost_set_dtype("bf16", old[1])


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2305_17469_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f
