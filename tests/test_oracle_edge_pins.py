"""Pins for the oracle's edge-weighting functions (NeighborApply g, Pull with h and f): each is
checked against an independent formulation -- the paper's dense SDDMM form (D D^T) o S, numpy
gather expressions, brute-force loops, algebraic identities that reduce to the already pinned
aggregation, and central finite differences."""
import numpy as np
import pytest

import oracle
from gt_inputs import configs, graphs


def _graphs():
    out = []
    rows = [[1, 2], [], [0, 1, 2, 3, 4, 5], [3, 3, 3], [], [0, 5]]
    rp = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    ci = np.array([c for r in rows for c in r], dtype=np.int32)
    out.append((rp, ci, 6))
    rows = [[8, 0], [4], [], [1, 2, 3, 5, 6, 7]]          # bipartite 4 x 9
    rp = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    ci = np.array([c for r in rows for c in r], dtype=np.int32)
    out.append((rp, ci, 9))
    rp, ci = graphs.rmat_csr(6, 6, seed=5, self_loops=False)
    out.append((rp, ci, 64))
    return out


def _xs_xd(rp, n_src, F, seed, square_same=False):
    rng = np.random.default_rng(seed)
    Xs = rng.standard_normal((n_src, F))
    Xd = Xs[: rp.size - 1].copy() if square_same else rng.standard_normal((rp.size - 1, F))
    return Xs, Xd


def test_dot_is_the_dense_sddmm_of_the_paper():
    # (D D^T) o S: all pairwise products, then keep the entries of connected pairs
    for rp, ci, n_src in _graphs():
        Xs, Xd = _xs_xd(rp, n_src, 7, 1)
        dense = Xd @ Xs.T                                    # [n_dst, n_src]
        dst = np.repeat(np.arange(rp.size - 1), np.diff(rp))
        np.testing.assert_allclose(oracle.neighbor_apply(rp, ci, Xs, Xd, "dot"), dense[dst, ci], rtol=1e-13, atol=1e-13)


def test_mul_is_a_gathered_elementwise_product():
    for rp, ci, n_src in _graphs():
        Xs, Xd = _xs_xd(rp, n_src, 5, 2)
        dst = np.repeat(np.arange(rp.size - 1), np.diff(rp))
        np.testing.assert_array_equal(oracle.neighbor_apply(rp, ci, Xs, Xd, "mul"), Xs[ci] * Xd[dst])


@pytest.mark.parametrize("reduce", ["sum", "mean"])
def test_pull_brute_force(reduce):
    rng = np.random.default_rng(3)
    for rp, ci, n_src in _graphs():
        n_dst, F, E = rp.size - 1, 4, ci.size
        Xs = rng.standard_normal((n_src, F))
        for h in ("scale", "add", "mul"):
            W = rng.standard_normal(E if h == "scale" else (E, F))
            ref = np.zeros((n_dst, F))
            for v in range(n_dst):
                terms = []
                for e in range(rp[v], rp[v + 1]):
                    x = Xs[ci[e]]
                    terms.append(W[e] * x if h == "scale" else (x + W[e] if h == "add" else x * W[e]))
                if terms:
                    ref[v] = np.sum(terms, axis=0) / (len(terms) if reduce == "mean" else 1)
            np.testing.assert_allclose(oracle.pull(rp, ci, Xs, W, reduce, h), ref, rtol=1e-12, atol=1e-12)


def test_pull_reduces_to_the_plain_aggregation():
    cfg = configs.tiny(8)
    blk = cfg["blocks"][0]
    rp, ci, n = blk["rowptr"], blk["colidx"], blk["n_src"]
    X = np.random.default_rng(4).standard_normal((n, 6))
    E = ci.size
    for reduce in ("sum", "mean"):
        agg = oracle.aggregate_fwd(rp, ci, n, X, reduce)
        np.testing.assert_allclose(oracle.pull(rp, ci, X, np.ones(E), reduce, "scale"), agg, rtol=1e-13)
        np.testing.assert_allclose(oracle.pull(rp, ci, X, np.zeros((E, 6)), reduce, "add"), agg, rtol=1e-13)
        np.testing.assert_allclose(oracle.pull(rp, ci, X, np.ones((E, 6)), reduce, "mul"), agg, rtol=1e-13)
        w = np.random.default_rng(5).uniform(0.5, 2.0, E).astype(np.float32)
        np.testing.assert_allclose(oracle.pull(rp, ci, X, w, reduce, "scale"),
                                   oracle.aggregate_fwd(rp, ci, n, X, reduce, w), rtol=1e-13)


def test_ngcf_identity_factors_the_destination_out():
    # mean_e (x_u + x_u (.) x_v) = (1 + x_v) (.) mean_e x_u : NeighborApply(mul) + Pull(add, mean)
    cfg = configs.tiny(8)
    blk = cfg["blocks"][0]
    rp, ci, n = blk["rowptr"], blk["colidx"], blk["n_src"]
    X = np.random.default_rng(6).standard_normal((n, 5))
    W = oracle.neighbor_apply(rp, ci, X, X, "mul")
    Y = oracle.pull(rp, ci, X, W, "mean", "add")
    np.testing.assert_allclose(Y, (1.0 + X) * oracle.aggregate_fwd(rp, ci, n, X, "mean"), rtol=1e-12, atol=1e-13)


def _fd(fun, arr, idx, h=1e-6):
    old = arr[idx]
    arr[idx] = old + h
    lp = fun()
    arr[idx] = old - h
    lm = fun()
    arr[idx] = old
    return (lp - lm) / (2 * h)


@pytest.mark.parametrize("g", ["dot", "mul"])
def test_neighbor_apply_bwd_finite_differences(g):
    rng = np.random.default_rng(7)
    for rp, ci, n_src in _graphs():
        Xs, Xd = _xs_xd(rp, n_src, 3, 8)
        G = rng.standard_normal(ci.size if g == "dot" else (ci.size, 3))
        loss = lambda: float(np.sum(G * oracle.neighbor_apply(rp, ci, Xs, Xd, g)))
        dXs, dXd = oracle.neighbor_apply_bwd(rp, ci, G, Xs, Xd, g)
        for _ in range(5):
            i, j = rng.integers(n_src), rng.integers(3)
            assert abs(_fd(loss, Xs, (i, j)) - dXs[i, j]) <= 1e-6 * (1 + abs(dXs[i, j]))
            i, j = rng.integers(rp.size - 1), rng.integers(3)
            assert abs(_fd(loss, Xd, (i, j)) - dXd[i, j]) <= 1e-6 * (1 + abs(dXd[i, j]))


@pytest.mark.parametrize("h", ["scale", "add", "mul"])
@pytest.mark.parametrize("reduce", ["sum", "mean"])
def test_pull_bwd_finite_differences(h, reduce):
    rng = np.random.default_rng(9)
    for rp, ci, n_src in _graphs():
        n_dst, F, E = rp.size - 1, 3, ci.size
        Xs = rng.standard_normal((n_src, F))
        W = rng.standard_normal(E if h == "scale" else (E, F))
        G = rng.standard_normal((n_dst, F))
        loss = lambda: float(np.sum(G * oracle.pull(rp, ci, Xs, W, reduce, h)))
        dXs, dW = oracle.pull_bwd(rp, ci, G, Xs, W, reduce, h)
        for _ in range(5):
            i, j = rng.integers(n_src), rng.integers(F)
            assert abs(_fd(loss, Xs, (i, j)) - dXs[i, j]) <= 1e-6 * (1 + abs(dXs[i, j]))
            if E:
                idx = int(rng.integers(E)) if h == "scale" else (int(rng.integers(E)), int(rng.integers(F)))
                assert abs(_fd(loss, W, idx) - dW[idx]) <= 1e-6 * (1 + abs(dW[idx]))
