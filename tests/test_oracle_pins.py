"""Pins for the CPU oracle: every oracle function is checked against something other than
itself -- a dense-adjacency matmul built independently, a library routine, a closed form, an
invariant, brute force, finite differences, or the one value the paper prints."""
import os

import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
from gt_inputs import configs, graphs, tensors

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------------------------
# helpers that deliberately do NOT reuse oracle code
# --------------------------------------------------------------------------------------------

def tiny_graphs():
    """Hand-made and random tiny graphs: (name, rowptr, colidx, n_src)."""
    out = []
    # empty rows, a full row, duplicate edges, a self-loop
    rows = [[1, 2], [], [0, 1, 2, 3, 4, 5], [3, 3, 3], [], [0, 5]]
    rp = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    ci = np.array([c for r in rows for c in r], dtype=np.int32)
    out.append(("hand6", rp, ci, 6))
    # bipartite: 4 destinations, 9 sources
    rows = [[8, 0], [4], [], [1, 2, 3, 5, 6, 7]]
    rp = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    ci = np.array([c for r in rows for c in r], dtype=np.int32)
    out.append(("bip4x9", rp, ci, 9))
    rng = np.random.default_rng(7)
    for n, e in ((17, 60), (64, 700)):
        s = rng.integers(0, n, e)
        d = rng.integers(0, n, e)
        rp, ci = graphs.csr_from_pairs(s, d, n, n, self_loops=False)
        out.append(("rand%d" % n, rp, ci, n))
    rp, ci = graphs.rmat_csr(6, 8, seed=11, self_loops=True)
    out.append(("rmat64", rp, ci, 64))
    return out


def dense_adjacency(rp, ci, n_src, reduce, ew):
    """n_dst x n_src matrix with one added coefficient per edge (multiplicities kept)."""
    n_dst = rp.size - 1
    A = np.zeros((n_dst, n_src), dtype=np.float64)
    deg = [int(rp[v + 1] - rp[v]) for v in range(n_dst)]
    for v in range(n_dst):
        for e in range(int(rp[v]), int(rp[v + 1])):
            u = int(ci[e])
            c = 1.0 if ew is None else float(ew[e])
            if reduce == "mean":
                c /= deg[v]
            elif reduce == "symnorm":
                c /= np.sqrt(float(deg[u]) * float(deg[v])) if deg[u] > 0 else np.inf
            A[v, u] += c
    return A


def modes_for(n_dst, n_src):
    return ("sum", "mean", "symnorm") if n_dst == n_src else ("sum", "mean")


# --------------------------------------------------------------------------------------------
# the paper's printed example
# --------------------------------------------------------------------------------------------

def test_paper_five_vertex_example():
    rows = {}
    for line in open(os.path.join(GOLDEN, "toy5_spmm.txt")):
        if line.startswith("#") or not line.strip():
            continue
        d, s = line.split(":")
        rows[int(d)] = [int(t) for t in s.split()]
    rp = np.cumsum([0] + [len(rows[v]) for v in range(5)]).astype(np.int32)
    ci = np.array([c for v in range(5) for c in rows[v]], dtype=np.int32)
    E = np.random.default_rng(0).standard_normal((5, 7))
    Y = oracle.aggregate_fwd(rp, ci, 5, E, "sum")
    np.testing.assert_array_equal(Y[0], E[2] + E[3])      # "V0's result is E2 + E3"
    np.testing.assert_array_equal(Y[2], np.zeros(7))       # empty row


# --------------------------------------------------------------------------------------------
# aggregation forward
# --------------------------------------------------------------------------------------------

@pytest.mark.parametrize("use_ew", [False, True])
def test_aggregate_fwd_matches_dense_matmul(use_ew):
    rng = np.random.default_rng(3)
    for name, rp, ci, n_src in tiny_graphs():
        n_dst = rp.size - 1
        ew = rng.uniform(0.5, 2.0, ci.size).astype(np.float32) if use_ew else None
        X = rng.standard_normal((n_src, 5))
        for mode in modes_for(n_dst, n_src):
            if mode == "symnorm" and np.any(np.diff(rp)[ci] == 0):
                continue   # a source with in-degree 0 has coefficient 0 by the reading; below
            A = dense_adjacency(rp, ci, n_src, mode, ew)
            Y = oracle.aggregate_fwd(rp, ci, n_src, X, mode, ew)
            np.testing.assert_allclose(Y, A @ X, rtol=1e-12, atol=1e-12, err_msg=name + mode)


def test_symnorm_zero_degree_source_contributes_zero():
    # vertex 1 has no in-edges but is a source of vertex 0: its coefficient is defined as 0
    rp = np.array([0, 2, 2], dtype=np.int32)
    ci = np.array([0, 1], dtype=np.int32)
    X = np.array([[3.0], [100.0]])
    Y = oracle.aggregate_fwd(rp, ci, 2, X, "symnorm")
    np.testing.assert_allclose(Y, [[3.0 / 2.0], [0.0]])    # (1/sqrt2)(1/sqrt2)*3


def test_aggregate_fwd_matches_scipy_midsize():
    cfg = configs.tiny()
    blk = cfg["blocks"][0]
    rp, ci, n = blk["rowptr"], blk["colidx"], blk["n_src"]
    X = cfg["X"].astype(np.float64)
    ew = np.random.default_rng(5).uniform(0.1, 1.0, ci.size).astype(np.float32)
    deg = np.diff(rp).astype(np.float64)
    S = sp.csr_matrix((ew.astype(np.float64), ci, rp), shape=(n, n))
    np.testing.assert_allclose(oracle.aggregate_fwd(rp, ci, n, X, "sum", ew), S @ X, rtol=1e-11, atol=1e-11)
    Dm = sp.diags(1.0 / deg)
    np.testing.assert_allclose(oracle.aggregate_fwd(rp, ci, n, X, "mean", ew), Dm @ (S @ X), rtol=1e-11, atol=1e-11)
    Ds = sp.diags(deg ** -0.5)
    np.testing.assert_allclose(oracle.aggregate_fwd(rp, ci, n, X, "symnorm", ew), Ds @ (S @ (Ds @ X)),
                               rtol=1e-11, atol=1e-11)


def test_ones_give_degrees_and_mean_gives_ones():
    for name, rp, ci, n_src in tiny_graphs() + [("c1",) + tuple(configs.tiny()["blocks"][0][k] for k in ("rowptr", "colidx", "n_src"))]:
        ones = np.ones((n_src, 3), dtype=np.float32)
        deg = np.diff(rp)
        Y = oracle.aggregate_fwd(rp, ci, n_src, ones, "sum")
        np.testing.assert_array_equal(Y, np.repeat(deg[:, None], 3, 1).astype(np.float64))
        Ym = oracle.aggregate_fwd(rp, ci, n_src, ones, "mean")
        np.testing.assert_array_equal(Ym, np.repeat((deg > 0)[:, None], 3, 1).astype(np.float64))
        din, dout = oracle.degrees(rp, ci, n_src)
        np.testing.assert_array_equal(din, deg)
        np.testing.assert_array_equal(dout, np.bincount(ci, minlength=n_src))
        assert din.sum() == dout.sum() == ci.size


def test_symnorm_closed_form_sqrt_degree():
    # X[u] = sqrt(d(u))  =>  Y[v] = d(v)^-1/2 * sum_u d(u)^-1/2 d(u)^1/2 = sqrt(d(v))
    for scale in (6, 12):
        rp, ci = graphs.rmat_csr(scale, 8, seed=21, self_loops=True)
        n = rp.size - 1
        d = np.diff(rp).astype(np.float64)
        Y = oracle.aggregate_fwd(rp, ci, n, np.sqrt(d)[:, None], "symnorm")
        np.testing.assert_allclose(Y[:, 0], np.sqrt(d), rtol=1e-12)


def test_row_subset_equals_full():
    cfg = configs.tiny()
    blk = cfg["blocks"][0]
    rows = np.array([0, 5, 77, 4095, 1000], dtype=np.int64)
    for mode in ("sum", "mean", "symnorm"):
        full = oracle.aggregate_fwd(blk["rowptr"], blk["colidx"], blk["n_src"], cfg["X"], mode)
        sub = oracle.aggregate_fwd(blk["rowptr"], blk["colidx"], blk["n_src"], cfg["X"], mode, rows=rows)
        np.testing.assert_array_equal(sub, full[rows])


# --------------------------------------------------------------------------------------------
# aggregation backward, transposed structure
# --------------------------------------------------------------------------------------------

@pytest.mark.parametrize("use_ew", [False, True])
def test_aggregate_bwd_matches_dense_transpose(use_ew):
    rng = np.random.default_rng(4)
    for name, rp, ci, n_src in tiny_graphs():
        n_dst = rp.size - 1
        ew = rng.uniform(0.5, 2.0, ci.size).astype(np.float32) if use_ew else None
        G = rng.standard_normal((n_dst, 4))
        for mode in modes_for(n_dst, n_src):
            if mode == "symnorm" and np.any(np.diff(rp)[ci] == 0):
                continue
            A = dense_adjacency(rp, ci, n_src, mode, ew)
            dX = oracle.aggregate_bwd(rp, ci, n_src, G, mode, ew)
            np.testing.assert_allclose(dX, A.T @ G, rtol=1e-12, atol=1e-12, err_msg=name + mode)


def test_adjoint_identity_and_src_subset():
    cfg = configs.tiny()
    blk = cfg["blocks"][0]
    rp, ci, n = blk["rowptr"], blk["colidx"], blk["n_src"]
    rng = np.random.default_rng(9)
    X = rng.standard_normal((n, 6))
    G = rng.standard_normal((n, 6))
    ew = rng.uniform(0.1, 1.0, ci.size).astype(np.float32)
    for mode in ("sum", "mean", "symnorm"):
        Y = oracle.aggregate_fwd(rp, ci, n, X, mode, ew)
        dX = oracle.aggregate_bwd(rp, ci, n, G, mode, ew)
        lhs, rhs = np.sum(Y * G), np.sum(X * dX)
        assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), 1.0) * 10
        rows = np.array([3, 0, 4000, 17], dtype=np.int64)
        sub = oracle.aggregate_bwd(rp, ci, n, G, mode, ew, src_rows=rows)
        np.testing.assert_array_equal(sub, dX[rows])


def test_transpose_brute_force_and_properties():
    for name, rp, ci, n_src in tiny_graphs():
        n_dst = rp.size - 1
        rpt, cit, perm = oracle.transpose(rp, ci, n_src)
        # brute force: list (src, position e, dst) and sort by (src, e)
        trip = sorted((int(ci[e]), e, v) for v in range(n_dst) for e in range(int(rp[v]), int(rp[v + 1])))
        np.testing.assert_array_equal(cit, [t[2] for t in trip])
        np.testing.assert_array_equal(perm, [t[1] for t in trip])
        np.testing.assert_array_equal(np.diff(rpt), np.bincount(ci, minlength=n_src))
        assert rpt[0] == 0 and rpt[-1] == ci.size
    cfg = configs.tiny()
    blk = cfg["blocks"][0]
    rp, ci, n = blk["rowptr"], blk["colidx"], blk["n_src"]
    rpt, cit, perm = oracle.transpose(rp, ci, n)
    np.testing.assert_array_equal(np.sort(perm), np.arange(ci.size))
    row_t = np.repeat(np.arange(n), np.diff(rpt))
    np.testing.assert_array_equal(ci[perm], row_t)
    # rows are sorted by source, so transposing twice gives the graph back
    rp2, ci2, _ = oracle.transpose(rpt, cit, n)
    np.testing.assert_array_equal(rp2, rp)
    np.testing.assert_array_equal(ci2, ci)
    # library cross-check
    S = sp.csr_matrix((np.ones(ci.size), ci, rp), shape=(n, n)).T.tocsr()
    S.sort_indices()
    np.testing.assert_array_equal(S.indptr, rpt)
    np.testing.assert_array_equal(S.indices, cit)


# --------------------------------------------------------------------------------------------
# combination
# --------------------------------------------------------------------------------------------

def test_combine_hand_case():
    A = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    B = np.array([[1.0, 0.0, -1.0], [2.0, 1.0, 0.0]])
    bias = np.array([0.5, -20.0, 0.0])
    np.testing.assert_array_equal(oracle.combine(A, B), [[5, 2, -1], [11, 4, -3], [17, 6, -5]])
    np.testing.assert_array_equal(oracle.combine(A, B, bias, relu=True),
                                  [[5.5, 0, 0], [11.5, 0, 0], [17.5, 0, 0]])


def test_combine_matches_numpy_all_transposes():
    rng = np.random.default_rng(1)
    for (M, N, K) in ((7, 5, 3), (33, 17, 65), (1, 9, 4)):
        A = rng.standard_normal((M, K))
        B = rng.standard_normal((K, N))
        b = rng.standard_normal(N)
        ref = A @ B
        np.testing.assert_allclose(oracle.combine(A, B), ref, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(oracle.combine(A.T.copy(), B, transA=True), ref, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(oracle.combine(A, B.T.copy(), transB=True), ref, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(oracle.combine(A.T.copy(), B.T.copy(), transA=True, transB=True), ref,
                                   rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(oracle.combine(A, B, b, relu=True), np.maximum(ref + b, 0), rtol=1e-13, atol=1e-13)


# --------------------------------------------------------------------------------------------
# bf16 rounding
# --------------------------------------------------------------------------------------------

def test_round_bf16_ties_and_library():
    x = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -30, -0.0, 0.0,
                  3.0e38, 3.4e38, 2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -134])
    y = oracle.round_bf16(x)
    np.testing.assert_array_equal(y[:4], [1.0, 1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7])
    assert y[6] == float(torch.tensor(3.0e38).to(torch.bfloat16)) and np.isinf(y[7])
    np.testing.assert_array_equal(y[8:], [2.0 ** -133, 0.0, 2.0 ** -132])   # subnormal grid, ties to even
    r = np.random.default_rng(2).standard_normal(20000).astype(np.float32) * np.float32(37.0)
    lib = torch.from_numpy(r).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(oracle.round_bf16(r.astype(np.float64)), lib)
    np.testing.assert_array_equal(tensors.bf16_values(r).astype(np.float64), lib)   # generator's conversion


# --------------------------------------------------------------------------------------------
# layers: the two orders, finite differences
# --------------------------------------------------------------------------------------------

def small_cfgs():
    return [configs.tiny(8), configs.sage_minibatch(10, 16), configs.reorder_stress(8, True, "mean", 24, 5),
            configs.reorder_stress(8, False, "sum", 24, 5)]


def test_two_forward_orders_agree():
    # sigma(W f(h(X)) + b) == sigma(f(h(W X)) + b): aggregation is the linear map A
    for cfg in small_cfgs() + [configs.tiny()]:
        a = oracle.model_fwd(cfg, "agg_first", round_outputs=False)
        c = oracle.model_fwd(cfg, "comb_first", round_outputs=False)
        for sa, sc in zip(a, c):
            scale = np.abs(sa["Z"]).max()
            assert np.abs(sa["Z"] - sc["Z"]).max() <= 1e-12 * scale


def test_two_backward_orders_agree():
    for cfg in small_cfgs():
        st = oracle.model_fwd(cfg, "agg_first", round_outputs=False)
        ga = oracle.model_bwd(cfg, st, "agg_first", round_outputs=False)
        gc = oracle.model_bwd(cfg, st, "comb_first", round_outputs=False)
        for a, c in zip(ga, gc):
            for k in ("dW", "db", "dW_root", "dX"):
                if a[k] is None:
                    assert c[k] is None
                    continue
                assert np.abs(a[k] - c[k]).max() <= 1e-11 * max(np.abs(a[k]).max(), 1e-30), k


def _loss(cfg):
    st = oracle.model_fwd(cfg, "agg_first", round_outputs=False)
    return float(np.sum(np.asarray(cfg["G"], dtype=np.float64) * st[-1]["H"])), st


@pytest.mark.parametrize("which", [0, 1, 2])
def test_backward_matches_central_finite_differences(which):
    cfg = dict(small_cfgs()[which])
    cfg["X"] = cfg["X"].astype(np.float64)
    cfg["W"] = [w.astype(np.float64) for w in cfg["W"]]
    cfg["b"] = [np.random.default_rng(5 + i).standard_normal(b.size) * 0.1 for i, b in enumerate(cfg["b"])]
    if cfg["model"] == "sage":
        cfg["W_root"] = [w.astype(np.float64) for w in cfg["W_root"]]
    _, st = _loss(cfg)
    grads = oracle.model_bwd(cfg, st, "agg_first", round_outputs=False)
    # gradient w.r.t. the input features: run the first layer's backward with need_dx
    g0 = oracle.layer_bwd(cfg["blocks"][0], cfg["reduce"], st[0]["X"], cfg["W"][0], st[0]["Z"],
                          grads[1]["dX"] if len(st) > 1 else cfg["G"], len(st) > 1, "agg_first",
                          cfg["W_root"][0], None, need_dx=True)
    rng = np.random.default_rng(77)
    h = 1e-6

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + h
        lp, _ = _loss(cfg)
        arr[idx] = old - h
        lm, _ = _loss(cfg)
        arr[idx] = old
        return (lp - lm) / (2 * h)

    checks = []
    for l in range(len(cfg["W"])):
        for _ in range(4):
            i, j = rng.integers(cfg["W"][l].shape[0]), rng.integers(cfg["W"][l].shape[1])
            checks.append((fd(cfg["W"][l], (i, j)), grads[l]["dW"][i, j]))
            if cfg["model"] == "sage":
                checks.append((fd(cfg["W_root"][l], (i, j)), grads[l]["dW_root"][i, j]))
        j = rng.integers(cfg["b"][l].size)
        checks.append((fd(cfg["b"][l], j), grads[l]["db"][j]))
    for _ in range(6):
        i, j = rng.integers(cfg["X"].shape[0]), rng.integers(cfg["X"].shape[1])
        checks.append((fd(cfg["X"], (i, j)), g0["dX"][i, j]))
    # (a step of 1e-6 crosses a ReLU kink only where |Z| < ~1e-5; such a crossing would fail below)
    scale = max(abs(a) for _, a in checks)
    for num, ana in checks:
        assert abs(num - ana) <= 2e-6 * scale + 1e-7, (num, ana)


def test_stop_sets_cut_elements_out_of_the_gradient():
    """model_bwd(stop=...) zeroes the upstream gradient of the marked output elements.  Pins: an
    all-false set changes nothing; on the last layer it equals zeroing G there; on a hidden layer
    it is the gradient of the model in which those activations are held constant (checked by
    central differences on a forward pass that re-inserts the unperturbed values)."""
    cfg = dict(small_cfgs()[0])
    cfg["X"] = cfg["X"].astype(np.float64)
    cfg["W"] = [w.astype(np.float64) for w in cfg["W"]]
    L = len(cfg["W"])
    st = oracle.model_fwd(cfg, "agg_first", round_outputs=False)
    base = oracle.model_bwd(cfg, st, "agg_first", round_outputs=False)
    none = oracle.model_bwd(cfg, st, "agg_first", round_outputs=False,
                            stop=[np.zeros(s["H"].shape, bool) for s in st])
    for a, b in zip(base, none):
        assert np.array_equal(a["dW"], b["dW"]) and np.array_equal(a["db"], b["db"])
    rng = np.random.default_rng(3)
    S_last = rng.random(st[-1]["H"].shape) < 0.3
    cfg2 = dict(cfg)
    cfg2["G"] = np.where(S_last, 0.0, cfg["G"])
    a = oracle.model_bwd(cfg, st, "agg_first", round_outputs=False, stop=[None] * (L - 1) + [S_last])
    b = oracle.model_bwd(cfg2, st, "agg_first", round_outputs=False)
    for x, y in zip(a, b):
        assert np.array_equal(x["dW"], y["dW"]) and np.array_equal(x["db"], y["db"])
    # hidden layer 0: activations in S are constants of the loss
    S0 = rng.random(st[0]["H"].shape) < 0.3
    g = oracle.model_bwd(cfg, st, "agg_first", round_outputs=False, stop=[S0] + [None] * (L - 1))
    assert np.abs(g[0]["dW"] - base[0]["dW"]).max() > 1e-3 * np.abs(base[0]["dW"]).max()   # the set matters
    for l in range(1, L):
        assert np.array_equal(g[l]["dW"], base[l]["dW"])                 # layers above it are untouched
    H0_fixed = st[0]["H"]

    def loss():
        s0 = oracle.layer_fwd(cfg["blocks"][0], cfg["reduce"], cfg["X"], cfg["W"][0], cfg["b"][0], True)
        H = np.where(S0, H0_fixed, s0["H"])
        for l in range(1, L):
            H = oracle.layer_fwd(cfg["blocks"][l], cfg["reduce"], H, cfg["W"][l], cfg["b"][l], l < L - 1)["H"]
        return float(np.sum(np.asarray(cfg["G"], dtype=np.float64) * H))

    h = 1e-6
    scale = np.abs(g[0]["dW"]).max()
    for _ in range(5):
        i, j = rng.integers(cfg["W"][0].shape[0]), rng.integers(cfg["W"][0].shape[1])
        old = cfg["W"][0][i, j]
        cfg["W"][0][i, j] = old + h
        lp = loss()
        cfg["W"][0][i, j] = old - h
        lm = loss()
        cfg["W"][0][i, j] = old
        assert abs((lp - lm) / (2 * h) - g[0]["dW"][i, j]) <= 2e-6 * scale + 1e-7
