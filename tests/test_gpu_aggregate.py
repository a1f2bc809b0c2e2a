"""gt_aggregate_fwd / gt_aggregate_bwd against the oracle, element by element.

Tolerances.  fp32: every output is a sum of at most GT_CHUNK fp32 fused multiply-adds per work
item plus the ordered sum of its partials, so |gpu - ref| <= 1e-5 * sum_e |c_e x_e| holds with a
wide margin (worst-case bound of sequential summation: n * 2^-24 per term); the tensor-level
metric max|gpu - ref| / max|ref| must be <= 1e-5.  bf16: the result is rounded once to bf16
(relative 2^-8), the oracle's fp64 result is rounded the same way, the two can differ by one
bf16 step when the fp32 sum sits next to a rounding boundary: |gpu - ref| <= 2^-7 |ref| + the
fp32 term; tensor-level <= 2e-2.
"""
import numpy as np
import pytest
import torch

import oracle
from gt_inputs import configs, graphs, tensors
from gpu_util import (announce, down, empty_feat, max_rel_err, pad_to, tol_for, up_feat, up_i32)

pytestmark = pytest.mark.gpu

WIDTHS = [1, 3, 16, 41, 47, 64, 100, 128, 256, 602, 1024]


def _graph_hubs():
    """4,096-vertex R-MAT plus two planted hub rows (2,000 and 700 in-edges) and a planted hub
    source, so split rows, near-threshold rows, empty rows and tiny rows all occur."""
    rp, ci = graphs.rmat_csr(12, 8, seed=31, self_loops=False)
    n = rp.size - 1
    dst = np.repeat(np.arange(n), np.diff(rp))
    rng = np.random.default_rng(8)
    extra_s = np.concatenate([rng.choice(n, 2000, replace=False), rng.choice(n, 700, replace=False),
                              np.full(1500, 5)])
    extra_d = np.concatenate([np.full(2000, 17), np.full(700, 900), rng.choice(n, 1500, replace=False)])
    rp, ci = graphs.csr_from_pairs(np.concatenate([ci, extra_s]), np.concatenate([dst, extra_d]), n, n)
    return rp, ci, n


def _check(got, ref, abs_terms, dtype, what):
    tol = tol_for(dtype)
    assert max_rel_err(got, ref) <= tol, (what, max_rel_err(got, ref))
    bound = 1e-5 * abs_terms + 1e-30
    if dtype == "bf16":
        bound = bound + 2.0 ** -7 * np.abs(ref)
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - ref).max()))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("F", WIDTHS)
def test_aggregate_widths_hub_graph(F, dtype):
    from paper_2305_17469_amd import binding as B
    rp, ci, n = _graph_hubs()
    g = B.Graph(up_i32(rp), up_i32(ci), n)
    X = tensors.normal((n, F), seed=100 + F)
    if dtype == "bf16":
        X = tensors.bf16_values(X)
    G = tensors.normal((n, F), seed=200 + F)
    if dtype == "bf16":
        G = tensors.bf16_values(G)
    for reduce in ("sum", "mean", "symnorm"):
        for ld in sorted({F, pad_to(F, dtype) + (8 if F % 2 else 0)}):
            announce("aggregate", dtype, "F", F, "ld", ld, reduce)
            Xd = up_feat(X, dtype, ld)
            Y = empty_feat(n, F, dtype, ld)
            B.gt_aggregate_fwd(g, reduce, Xd, out=Y)
            ref = oracle.aggregate_fwd(rp, ci, n, X, reduce)
            absr = oracle.aggregate_fwd(rp, ci, n, np.abs(X), reduce)
            if dtype == "bf16":
                ref = oracle.round_bf16(ref)
            _check(down(Y), ref, absr, dtype, ("fwd", reduce, F, ld))
            Gd = up_feat(G, dtype, ld)
            dX = empty_feat(n, F, dtype, ld)
            B.gt_aggregate_bwd(g, reduce, Gd, out=dX)
            ref = oracle.aggregate_bwd(rp, ci, n, G, reduce)
            absr = oracle.aggregate_bwd(rp, ci, n, np.abs(G), reduce)
            if dtype == "bf16":
                ref = oracle.round_bf16(ref)
            _check(down(dX), ref, absr, dtype, ("bwd", reduce, F, ld))
            if ld > F:   # padding columns of the outputs are never written
                assert torch.isnan(Y.as_strided((n, ld - F), (ld, 1), Y.storage_offset() + F)).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_aggregate_edge_weights_and_bipartite(dtype):
    from paper_2305_17469_amd import binding as B
    cfg = configs.sage_minibatch(12, 64)
    for blk in cfg["blocks"]:
        rp, ci, ns, nd = blk["rowptr"], blk["colidx"], blk["n_src"], blk["n_dst"]
        ew = np.random.default_rng(5).uniform(0.25, 2.0, ci.size).astype(np.float32)
        g = B.Graph(up_i32(rp), up_i32(ci), ns, torch.from_numpy(ew).cuda())
        F = 40
        X = tensors.normal((ns, F), seed=7)
        G = tensors.normal((nd, F), seed=8)
        if dtype == "bf16":
            X, G = tensors.bf16_values(X), tensors.bf16_values(G)
        for reduce in ("sum", "mean"):
            announce("aggregate weighted bipartite", dtype, reduce, nd, ns)
            Y = B.gt_aggregate_fwd(g, reduce, up_feat(X, dtype))
            ref = oracle.aggregate_fwd(rp, ci, ns, X, reduce, ew)
            absr = oracle.aggregate_fwd(rp, ci, ns, np.abs(X), reduce, ew)
            _check(down(Y), oracle.round_bf16(ref) if dtype == "bf16" else ref, absr, dtype, ("fwd", reduce))
            dX = B.gt_aggregate_bwd(g, reduce, up_feat(G, dtype))
            ref = oracle.aggregate_bwd(rp, ci, ns, G, reduce, ew)
            absr = oracle.aggregate_bwd(rp, ci, ns, np.abs(G), reduce, ew)
            _check(down(dX), oracle.round_bf16(ref) if dtype == "bf16" else ref, absr, dtype, ("bwd", reduce))
        with pytest.raises(B.GtError) as e:
            B.gt_aggregate_fwd(g, "symnorm", up_feat(X, dtype))
        assert e.value.status == 2   # UNSUPPORTED on a non-square graph


def test_exact_invariants_on_the_gpu():
    """sum of ones = in-degree exactly, mean of ones = 1 exactly (division, not reciprocal)."""
    from paper_2305_17469_amd import binding as B
    rp, ci, n = _graph_hubs()
    announce("aggregate invariants")
    g = B.Graph(up_i32(rp), up_i32(ci), n)
    ones = torch.ones((n, 8), dtype=torch.float32, device="cuda")
    deg = np.diff(rp).astype(np.float64)
    np.testing.assert_array_equal(down(B.gt_aggregate_fwd(g, "sum", ones)), np.repeat(deg[:, None], 8, 1))
    np.testing.assert_array_equal(down(B.gt_aggregate_fwd(g, "mean", ones)), np.repeat((deg > 0)[:, None], 8, 1) * 1.0)
    dout = np.bincount(ci, minlength=n).astype(np.float64)
    np.testing.assert_array_equal(down(B.gt_aggregate_bwd(g, "sum", ones)), np.repeat(dout[:, None], 8, 1))


def test_bitwise_reproducible_and_argument_errors():
    from paper_2305_17469_amd import binding as B
    rp, ci, n = _graph_hubs()
    announce("aggregate determinism + errors")
    g = B.Graph(up_i32(rp), up_i32(ci), n)
    X = up_feat(tensors.normal((n, 100), seed=3), "f32", 104)
    a = B.gt_aggregate_fwd(g, "symnorm", X).clone()
    b = B.gt_aggregate_fwd(g, "symnorm", X).clone()
    assert torch.equal(a, b)
    g2 = B.Graph(up_i32(rp), up_i32(ci), n)       # a second plan of the same graph gives the same bits
    assert torch.equal(a, B.gt_aggregate_fwd(g2, "symnorm", X))
    with pytest.raises(B.GtError) as e:           # in-place is rejected
        B.gt_aggregate_fwd(g, "sum", X, out=X)
    assert e.value.status == 1
    st = B.lib.gt_aggregate_fwd(g.handle, 0, 0, 100, X.data_ptr(), 50, a.data_ptr(), 100, None, 0, None)
    assert st == 1                                # ld < F
    need = g.aggregate_ws(100).numel()
    st = B.lib.gt_aggregate_fwd(g.handle, 0, 0, 100, X.data_ptr(), 104, a.data_ptr(), 100, None, 0, None)
    assert st == 3 and need > 256                 # split rows need the scratch buffer
    # zero-width and empty-graph calls are no-ops
    assert B.lib.gt_aggregate_fwd(g.handle, 0, 0, 0, None, 0, None, 0, None, 0, None) == 0
    g0 = B.Graph(up_i32(np.zeros(1, np.int32)), up_i32(np.zeros(0, np.int32)), 0)
    assert B.lib.gt_aggregate_fwd(g0.handle, 0, 0, 16, None, 16, None, 16, None, 0, None) == 0


def test_empty_rows_only():
    from paper_2305_17469_amd import binding as B
    announce("aggregate: graph without edges")
    g = B.Graph(up_i32(np.zeros(8, np.int32)), up_i32(np.zeros(0, np.int32)), 5)
    X = up_feat(tensors.normal((5, 12), seed=1), "f32")
    for reduce in ("sum", "mean"):
        assert torch.count_nonzero(B.gt_aggregate_fwd(g, reduce, X)) == 0
        assert torch.count_nonzero(B.gt_aggregate_bwd(g, reduce, up_feat(tensors.normal((7, 12), seed=2), "f32"))) == 0


def test_bf16_outputs_round_to_nearest_even_bit_for_bit():
    """Rows of two in-edges whose two bf16 terms differ by at most 8 binades: the fp32 sum is exact,
    so the bf16 output must be THE nearest-even rounding of the exact sum, ties included (a large
    share of such sums are ties), down to subnormal results and up to overflow."""
    from paper_2305_17469_amd import binding as B
    n, F = 8192, 8
    rng = np.random.default_rng(77)
    ea = rng.integers(90, 160, size=(n, F))
    ea[:64] = rng.integers(0, 3, size=(64, F))          # subnormal and smallest normal terms
    ea[64:128] = 254                                    # largest binade: same-sign sums overflow
    eb = np.maximum(ea - rng.integers(0, 9, size=(n, F)), 0)
    bits_a = (rng.integers(0, 2, size=(n, F)) << 15) | (ea << 7) | rng.integers(0, 128, size=(n, F))
    bits_b = (rng.integers(0, 2, size=(n, F)) << 15) | (eb << 7) | rng.integers(0, 128, size=(n, F))
    a = tensors.from_bf16_bits(bits_a.astype(np.uint16))
    b = tensors.from_bf16_bits(bits_b.astype(np.uint16))
    X = np.empty((2 * n, F), dtype=np.float32)
    X[0::2], X[1::2] = a, b
    assert np.array_equal(tensors.bf16_values(X), X)
    exact = a.astype(np.float64) + b.astype(np.float64)
    ref = oracle.round_bf16(exact)
    assert (ref != exact).mean() > 0.3                                  # most sums do need rounding
    g = B.Graph(up_i32(np.arange(0, 2 * n + 1, 2)), up_i32(np.arange(2 * n)), 2 * n)
    announce("aggregate bf16 rounding", n, F)
    got = down(B.gt_aggregate_fwd(g, "sum", up_feat(X, "bf16")))
    assert np.isinf(ref).any() and not np.isnan(ref).any()
    bad = got != ref
    assert not bad.any(), (int(bad.sum()), exact[bad][:4], got[bad][:4], ref[bad][:4])


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_aggregate_random_graphs(seed):
    """Seeded random bipartite and square graphs (empty graphs, single rows, empty rows, one row holding
    most of the edges so that it is split, duplicate-free random edges), random widths and strides,
    with and without per-edge weights, every reduction, both directions."""
    from paper_2305_17469_amd import binding as B
    rng = np.random.default_rng(seed)
    for it in range(24):
        n_dst = int(rng.choice([1, 2, 7, 64, 257, 1000, 5000]))
        n_src = n_dst if it % 3 == 0 else int(rng.choice([1, 3, 50, 333, 4096]))
        n_e = int(rng.choice([0, 1, 5, 200, 3000, 40000]))
        n_e = min(n_e, n_dst * n_src)
        src = rng.integers(0, n_src, n_e)
        dst = rng.integers(0, n_dst, n_e)
        if n_e >= 3000 and n_src >= 333:      # a hub: one destination takes a long run of distinct sources
            k = min(n_src, 2500)
            src = np.concatenate([src, rng.permutation(n_src)[:k]])
            dst = np.concatenate([dst, np.full(k, int(rng.integers(0, n_dst)))])
        rp, ci = graphs.csr_from_pairs(src, dst, n_dst, n_src)
        F = int(rng.choice([1, 2, 5, 8, 16, 31, 64, 100, 130, 256, 300]))
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        ld = F if rng.random() < 0.5 else pad_to(F, dtype) + int(rng.choice([0, 8]))
        ew = rng.uniform(0.25, 2.0, ci.size).astype(np.float32) if rng.random() < 0.5 else None
        g = B.Graph(up_i32(rp), up_i32(ci), n_src, None if ew is None else torch.from_numpy(ew).cuda())
        X = tensors.normal((n_src, F), seed=seed * 100 + it)
        G = tensors.normal((n_dst, F), seed=seed * 100 + it + 50)
        if dtype == "bf16":
            X, G = tensors.bf16_values(X), tensors.bf16_values(G)
        modes = ("sum", "mean", "symnorm") if n_src == n_dst else ("sum", "mean")
        for reduce in modes:
            announce("aggregate random", seed, it, dtype, (n_dst, n_src, int(ci.size)), "F", F, "ld", ld, reduce, "ew", ew is not None)
            Y = empty_feat(n_dst, F, dtype, ld)
            B.gt_aggregate_fwd(g, reduce, up_feat(X, dtype, ld), out=Y)
            ref = oracle.aggregate_fwd(rp, ci, n_src, X, reduce, ew)
            absr = oracle.aggregate_fwd(rp, ci, n_src, np.abs(X), reduce, ew)
            _check(down(Y), oracle.round_bf16(ref) if dtype == "bf16" else ref, absr, dtype, ("fwd", it, reduce))
            dX = empty_feat(n_src, F, dtype, ld)
            B.gt_aggregate_bwd(g, reduce, up_feat(G, dtype, ld), out=dX)
            ref = oracle.aggregate_bwd(rp, ci, n_src, G, reduce, ew)
            absr = oracle.aggregate_bwd(rp, ci, n_src, np.abs(G), reduce, ew)
            _check(down(dX), oracle.round_bf16(ref) if dtype == "bf16" else ref, absr, dtype, ("bwd", it, reduce))
