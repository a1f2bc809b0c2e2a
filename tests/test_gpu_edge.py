"""Edge weighting on the GPU (gt_neighbor_apply_fwd/bwd, gt_pull_fwd/bwd) against the oracle.

Tolerances as for the aggregation: fp32 sums of at most a chunk of fused multiply-adds per work
item, |gpu - ref| <= 1e-5 * (sum of the magnitudes of the terms) element-wise and
max|gpu - ref| / max|ref| <= 1e-5 per tensor; bf16 outputs are rounded once (2^-8 relative, one
step of slack against the oracle's rounding) and pass 2e-2 per tensor.
"""
import numpy as np
import pytest
import torch

import oracle
from gt_inputs import configs, graphs, tensors
from gpu_util import announce, down, max_rel_err, pad_to, tol_for, up_feat, up_i32

pytestmark = pytest.mark.gpu


def _hub_graph():
    rp, ci = graphs.rmat_csr(11, 8, seed=41, self_loops=False)
    n = rp.size - 1
    dst = np.repeat(np.arange(n), np.diff(rp))
    rng = np.random.default_rng(2)
    es = np.concatenate([rng.choice(n, 900, replace=False), np.full(600, 3)])
    ed = np.concatenate([np.full(900, 11), rng.choice(n, 600, replace=False)])
    rp, ci = graphs.csr_from_pairs(np.concatenate([ci, es]), np.concatenate([dst, ed]), n, n)
    return rp, ci, n


def _cases():
    rp, ci, n = _hub_graph()
    out = [("hub2048", rp, ci, n)]
    b = configs.sage_minibatch(12, 64)["blocks"][0]
    out.append(("bipartite", b["rowptr"], b["colidx"], b["n_src"]))
    return out


def _vals(shape, seed, dtype):
    x = tensors.normal(shape, seed=seed)
    return tensors.bf16_values(x) if dtype == "bf16" else x


def _check(got, ref, absr, dtype, rounded, what):
    tol = tol_for(dtype if rounded else "f32")
    assert max_rel_err(got, ref) <= tol, (what, max_rel_err(got, ref))
    bound = 1e-5 * absr + 1e-30 + (2.0 ** -7 * np.abs(ref) if rounded and dtype == "bf16" else 0.0)
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - ref).max()))


def _rnd(x, dtype):
    return oracle.round_bf16(x) if dtype == "bf16" else x


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("F", [1, 16, 41, 100, 256, 602])
def test_neighbor_apply_fwd_bwd(F, dtype):
    from paper_2305_17469_amd import binding as B
    for name, rp, ci, n_src in _cases():
        n_dst, E = rp.size - 1, ci.size
        g = B.Graph(up_i32(rp), up_i32(ci), n_src)
        Xs, Xd = _vals((n_src, F), 1, dtype), _vals((n_dst, F), 2, dtype)
        ld = pad_to(F, dtype)
        for ldx in sorted({F, ld}):
            Xs_d, Xd_d = up_feat(Xs, dtype, ldx), up_feat(Xd, dtype, ldx)
            for fn in ("dot", "mul"):
                announce("neighbor_apply", name, dtype, "F", F, "ld", ldx, fn)
                W = B.gt_neighbor_apply_fwd(g, fn, Xs_d, Xd_d)
                ref = oracle.neighbor_apply(rp, ci, Xs, Xd, fn)
                absr = oracle.neighbor_apply(rp, ci, np.abs(Xs), np.abs(Xd), fn)
                if fn == "dot":
                    _check(down(W), ref, absr, dtype, False, ("fwd", fn, name))
                else:
                    _check(down(W), _rnd(ref, dtype), absr, dtype, True, ("fwd", fn, name))
                dW = _vals((E,) if fn == "dot" else (E, F), 3, "f32" if fn == "dot" else dtype)
                dW_d = torch.from_numpy(dW).cuda() if fn == "dot" else up_feat(dW, dtype, ldx)
                dXs, dXd = B.gt_neighbor_apply_bwd(g, fn, dW_d, Xs_d, Xd_d)
                rs, rd = oracle.neighbor_apply_bwd(rp, ci, dW, Xs, Xd, fn)
                as_, ad = oracle.neighbor_apply_bwd(rp, ci, np.abs(dW), np.abs(Xs), np.abs(Xd), fn)
                _check(down(dXs), _rnd(rs, dtype), as_, dtype, True, ("dXs", fn, name))
                _check(down(dXd), _rnd(rd, dtype), ad, dtype, True, ("dXd", fn, name))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("F", [3, 64, 100, 602])
def test_pull_fwd_bwd(F, dtype):
    from paper_2305_17469_amd import binding as B
    for name, rp, ci, n_src in _cases():
        n_dst, E = rp.size - 1, ci.size
        g = B.Graph(up_i32(rp), up_i32(ci), n_src)
        Xs, G = _vals((n_src, F), 4, dtype), _vals((n_dst, F), 5, dtype)
        ld = pad_to(F, dtype)
        Xs_d, G_d = up_feat(Xs, dtype, ld), up_feat(G, dtype, ld)
        for h in ("scale", "add", "mul"):
            W = _vals((E,) if h == "scale" else (E, F), 6, "f32" if h == "scale" else dtype)
            W_d = torch.from_numpy(W).cuda() if h == "scale" else up_feat(W, dtype, ld)
            for reduce in ("sum", "mean"):
                announce("pull", name, dtype, "F", F, h, reduce)
                Y = B.gt_pull_fwd(g, reduce, h, Xs_d, W_d)
                ref = oracle.pull(rp, ci, Xs, W, reduce, h)
                absr = oracle.pull(rp, ci, np.abs(Xs), np.abs(W), reduce, h)
                _check(down(Y), _rnd(ref, dtype), absr, dtype, True, ("fwd", h, reduce, name))
                dXs, dW = B.gt_pull_bwd(g, reduce, h, G_d, Xs_d, W_d)
                rx, rw = oracle.pull_bwd(rp, ci, G, Xs, W, reduce, h)
                ax, aw = oracle.pull_bwd(rp, ci, np.abs(G), np.abs(Xs), np.abs(W), reduce, h)
                _check(down(dXs), _rnd(rx, dtype), ax, dtype, True, ("dXs", h, reduce, name))
                _check(down(dW), rw if h == "scale" else _rnd(rw, dtype), aw, dtype, h != "scale", ("dW", h, reduce, name))


def test_ngcf_layer_matches_its_factorised_form_and_is_reproducible():
    """NeighborApply(mul) + Pull(add, mean) -- the NGCF listing -- equals (1 + x_v) (.) mean_e x_u."""
    from paper_2305_17469_amd import binding as B
    cfg = configs.tiny()
    blk = cfg["blocks"][0]
    rp, ci, n = blk["rowptr"], blk["colidx"], blk["n_src"]
    announce("ngcf identity")
    g = B.Graph(up_i32(rp), up_i32(ci), n)
    X = up_feat(cfg["X"], "f32")
    W = B.gt_neighbor_apply_fwd(g, "mul", X, X)
    Y = B.gt_pull_fwd(g, "mean", "add", X, W)
    ref = (1.0 + cfg["X"].astype(np.float64)) * oracle.aggregate_fwd(rp, ci, n, cfg["X"], "mean")
    assert max_rel_err(down(Y), ref) <= 1e-5
    assert torch.equal(Y, B.gt_pull_fwd(g, "mean", "add", X, B.gt_neighbor_apply_fwd(g, "mul", X, X)))


def test_edge_entry_points_reject_bad_requests():
    from paper_2305_17469_amd import binding as B
    rp, ci, n = _hub_graph()
    announce("edge error paths")
    ew = torch.ones(ci.size, dtype=torch.float32, device="cuda")
    gw = B.Graph(up_i32(rp), up_i32(ci), n, ew)
    X = up_feat(tensors.normal((n, 8), seed=1), "f32")
    with pytest.raises(B.GtError) as e:
        B.gt_neighbor_apply_fwd(gw, "mul", X, X)
    assert e.value.status == 2                      # static edge weights in the plan
    g = B.Graph(up_i32(rp), up_i32(ci), n)
    W = torch.zeros((ci.size, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(B.GtError) as e:
        B.gt_pull_fwd(g, "symnorm", "add", X, W)
    assert e.value.status == 2
    wide = up_feat(tensors.normal((n, 1100), seed=5), "f32")           # wider than one column tile
    ref = oracle.neighbor_apply(rp, ci, down(wide), down(wide), "dot")
    assert max_rel_err(down(B.gt_neighbor_apply_fwd(g, "dot", wide, wide)), ref) <= 1e-5
    ws = g.aggregate_ws(8)
    st = B.lib.gt_pull_fwd(g.handle, 0, 1, 0, 8, X.data_ptr(), 4, W.data_ptr(), 8, W.data_ptr(), 8, ws.data_ptr(),
                           ws.numel(), None)
    assert st == 1                                  # ld < F
    st = B.lib.gt_pull_fwd(g.handle, 0, 1, 0, 8, X.data_ptr(), 8, W.data_ptr(), 8, W.data_ptr(), 8, None, 0, None)
    assert st == 3                                  # split rows need the scratch buffer
    g0 = B.Graph(up_i32(np.zeros(4, np.int32)), up_i32(np.zeros(0, np.int32)), 3)
    Y = B.gt_pull_fwd(g0, "mean", "add", up_feat(tensors.normal((3, 8), seed=2), "f32"),
                      torch.zeros((0, 8), dtype=torch.float32, device="cuda"))
    assert torch.count_nonzero(Y) == 0
