"""gt_layer_fwd / gt_layer_bwd (both placements, AUTO) on scaled-down versions of the five
workloads, against the oracle's model functions.  Tensor-level tolerance of the benchmark spec:
max|gpu - ref| / max|ref| <= 1e-5 (fp32), 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import oracle
from gt_inputs import configs, graphs, tensors
from gpu_util import announce, down, empty_feat, max_rel_err, pad_to, relu_rounding_sets, tol_for, up_feat, up_i32

pytestmark = pytest.mark.gpu


def small_workloads():
    return [configs.tiny(), configs.reddit_like(11), configs.products_like(12), configs.sage_minibatch(13, 128),
            configs.reorder_stress(11, True, "sum"), configs.reorder_stress(11, False, "mean"),
            configs.reorder_stress(11, True, "mean", 100, 47),
            # 16,384 vertices: tall enough for the weight-stationary, streaming and one-tile weight-gradient kernels
            configs.reorder_stress(14, True, "sum"), configs.reorder_stress(14, False, "mean"), configs.products_like(14)]


def run_model(cfg, fwd_order, bwd_order, pad=True, ref=None, fold=False):
    """The whole model through gt_layer_fwd / gt_layer_bwd, twice over:
      chained      forward with every layer reading the library's own previous output (what a user
                   runs); only its outputs are compared;
      layer-wise   every layer's forward on the ORACLE's input of that layer (exact in the working
                   type), then the backward chain through those layers: X, Y and `saved` of a layer
                   come from its layer-wise forward, the upstream gradient from the layer above,
                   zeroed on the oracle-made set of ReLU decisions that rounding may flip.
    `ref` = oracle_reference(cfg).  `fold`: the descriptors ask for the ReLU derivative to be
    folded into the kernel that produces the gradient (in_act / dy_is_dz).  Returns (chained
    outputs, layer-wise outputs, gradients, forward orders, backward orders)."""
    from paper_2305_17469_amd import binding as B
    st, stop = (ref or oracle_reference(cfg))[:2]
    dt = cfg["dtype"]
    L = len(cfg["W"])
    sage = cfg["model"] == "sage"
    graphs, seen = [], {}
    for blk in cfg["blocks"]:
        key = id(blk["rowptr"])
        if key not in seen:
            seen[key] = B.Graph(up_i32(blk["rowptr"]), up_i32(blk["colidx"]), blk["n_src"])
        graphs.append(seen[key])
    ld = (lambda F: pad_to(F, dt)) if pad else (lambda F: F)
    Ws = [up_feat(w, dt) for w in cfg["W"]]
    Wr = [up_feat(w, dt) if sage else None for w in cfg["W_root"]]
    bs = [torch.from_numpy(b).cuda() for b in cfg["b"]]
    descs = [B.make_desc(cfg["reduce"], dt, l < L - 1, cfg["dims"][l], cfg["dims"][l + 1], has_root=sage, need_dx=l > 0,
                         in_relu=fold and l > 0, dy_is_dz=fold and l < L - 1) for l in range(L)]
    bufs = [B.LayerBuffers(graphs[l], descs[l]) for l in range(L)]

    def fwd(l, Xin):
        out = up_feat(np.zeros((graphs[l].n_dst, cfg["dims"][l + 1]), np.float32), dt, ld(cfg["dims"][l + 1]))
        return B.gt_layer_fwd(graphs[l], descs[l], Xin, Ws[l], bs[l], bufs[l], fwd_order, Wr[l], out=out)

    Hc = [up_feat(cfg["X"], dt, ld(cfg["dims"][0]))]
    for l in range(L):
        Hc.append(fwd(l, Hc[-1])[0])
    Xin = [up_feat(st[l]["X"], dt, ld(cfg["dims"][l])) for l in range(L)]
    Hl, used_f = [], []
    for l in range(L):
        Y, used = fwd(l, Xin[l])
        Hl.append(Y)
        used_f.append(used)
    dH = up_feat(cfg["G"], dt, ld(cfg["dims"][-1]))
    grads, used_b = [None] * L, [None] * L
    for l in reversed(range(L)):
        out_dX = None
        if l > 0:
            out_dX = up_feat(np.zeros((graphs[l].n_src, cfg["dims"][l]), np.float32), dt, ld(cfg["dims"][l]))
        if stop[l] is not None:
            keep = dH                                 # dH is also a compared output: mask a copy of equal stride
            dH = torch.zeros((dH.shape[0], dH.stride(0)), dtype=dH.dtype, device=dH.device)[:, :dH.shape[1]]
            dH.copy_(keep)
            dH.masked_fill_(torch.from_numpy(stop[l]).cuda(), 0.0)
        r = B.gt_layer_bwd(graphs[l], descs[l], used_f[l], dH, Xin[l], Ws[l], None if descs[l].dy_is_dz else Hl[l],
                           bufs[l], bwd_order, Wr[l], out_dX=out_dX)
        grads[l] = r
        used_b[l] = r["used"]
        dH = r["dX"]
    torch.cuda.synchronize()
    return Hc[1:], Hl, grads, used_f, used_b


_ORACLE_CACHE = {}


def oracle_reference(cfg):
    """Everything the comparison needs, made by the oracle alone: forward states, the sets of
    ReLU decisions that rounding may flip (gpu_util.relu_rounding_sets), and the backward pass
    with its OWN decisions [Z > 0] and the upstream gradient zeroed on those sets."""
    key = cfg["name"] + str(cfg["X"].shape)
    if key not in _ORACLE_CACHE:
        st = oracle.model_fwd(cfg, "agg_first")
        stop, bounds = relu_rounding_sets(cfg, st)
        og = oracle.model_bwd(cfg, st, "agg_first", stop=stop)
        _ORACLE_CACHE[key] = (st, stop, bounds, og)
    return _ORACLE_CACHE[key]


def compare(cfg, Hc, Hl, grads, what, fold=False):
    """Outputs against the oracle's forward, gradients against the oracle's backward.  The ReLU
    derivative is a yes/no decision taken from a floating-point value (paper: "Training for GNNs",
    the activation's derivative): the library's decision [Y > 0] must equal the oracle's [Z > 0]
    everywhere outside the oracle-made rounding set, and inside that set the upstream gradient
    was zeroed on both sides (run_model, oracle.model_bwd(stop=...)), so no decision of the
    library enters the reference."""
    st, stop, bounds, og = oracle_reference(cfg)
    tol = tol_for(cfg["dtype"])
    L = len(st)
    errs, frac = {}, {}
    for l in range(L):
        Hg = down(Hl[l])
        if l < L - 1:
            bad = ((Hg > 0.0) != (st[l]["Z"] > 0.0)) & ~stop[l]
            assert not bad.any(), (what, "relu decision outside the rounding set", l, int(bad.sum()))
            frac[l] = float(stop[l].mean())
        errs["Hchain%d" % l] = max_rel_err(down(Hc[l]), st[l]["H"])
        errs["H%d" % l] = max_rel_err(Hg, st[l]["H"])
        errs["dW%d" % l] = max_rel_err(down(grads[l]["dW"]), og[l]["dW"])
        errs["db%d" % l] = max_rel_err(down(grads[l]["db"]), og[l]["db"])
        if og[l]["dW_root"] is not None:
            errs["dWr%d" % l] = max_rel_err(down(grads[l]["dW_root"]), og[l]["dW_root"])
        if l > 0:
            # folded: dX comes back multiplied by [X > 0], X being the oracle's activation given to the layer
            want = og[l]["dX"] * (st[l - 1]["H"] > 0.0) if fold else og[l]["dX"]
            errs["dX%d" % l] = max_rel_err(down(grads[l]["dX"]), want)
    assert max(errs.values()) <= tol, (what, errs)
    # the rounding sets must stay a small part of the outputs, or the gradient check would be hollow
    assert all(v <= (0.05 if cfg["dtype"] == "bf16" else 1e-3) for v in frac.values()), frac
    return errs


@pytest.mark.parametrize("cfg", small_workloads(), ids=lambda c: c["name"])
@pytest.mark.parametrize("orders", [("agg_first", "agg_first"), ("comb_first", "comb_first"),
                                    ("agg_first", "comb_first"), ("comb_first", "agg_first"), ("auto", "auto")])
@pytest.mark.parametrize("fold", [False, True], ids=["mask_pass", "mask_folded"])
def test_model_fwd_bwd_parity(cfg, orders, fold):
    if fold and len(cfg["W"]) == 1:
        pytest.skip("a single layer has no ReLU between layers")
    announce("layer parity", cfg["name"], orders, "folded" if fold else "")
    Hc, Hl, grads, uf, ub = run_model(cfg, *orders, fold=fold)
    if orders[0] != "auto":
        assert all(u == orders[0] for u in uf)
        # the first layer has no dX: its backward order is reported as the forward's
        assert all(u == orders[1] for u in ub[1:])
    compare(cfg, Hc, Hl, grads, (cfg["name"], orders, fold), fold=fold)


def test_unpadded_strides_take_the_elementwise_path():
    cfg = configs.reorder_stress(11, True, "mean", 100, 47)
    cfg = dict(cfg)
    cfg["dims"] = list(cfg["dims"])
    announce("layer parity unpadded ld", cfg["name"])
    cfg2 = dict(configs.reddit_like(11))       # 602 -> 128 -> 41, ld = 602 and 41: not multiples of 4
    for c in (cfg, cfg2):
        for fold in (False, True):
            Hc, Hl, grads, _, _ = run_model(c, "auto", "auto", pad=False, fold=fold)
            compare(c, Hc, Hl, grads, (c["name"], "unpadded", fold), fold=fold)


def test_auto_matches_decide_and_expected_orders():
    from paper_2305_17469_amd import binding as B
    announce("layer decide")
    cfg = configs.reddit_like(11)
    blk = cfg["blocks"][0]
    g = B.Graph(up_i32(blk["rowptr"]), up_i32(blk["colidx"]), blk["n_src"])
    # full graph (n_src == n_dst): aggregation-first has no benefit, so the width decides
    assert B.gt_layer_decide(g, B.make_desc("symnorm", "f32", True, 602, 128, need_dx=False)) == ("comb_first", "comb_first")
    assert B.gt_layer_decide(g, B.make_desc("symnorm", "f32", False, 128, 41)) == ("comb_first", "comb_first")
    assert B.gt_layer_decide(g, B.make_desc("symnorm", "f32", True, 16, 1024)) == ("agg_first", "agg_first")
    assert B.gt_layer_decide(g, B.make_desc("symnorm", "f32", True, 64, 64)) == ("agg_first", "agg_first")   # tie
    # sampled block with far fewer destinations than sources: row reduction wins over 256 -> 47
    c4 = configs.sage_minibatch(13, 128)
    b2 = c4["blocks"][1]
    g2 = B.Graph(up_i32(b2["rowptr"]), up_i32(b2["colidx"]), b2["n_src"])
    f, _ = B.gt_layer_decide(g2, B.make_desc("mean", "f32", False, 256, 47, has_root=True))
    assert f == "agg_first"


def test_first_layer_agg_first_backward_launches_no_aggregation():
    """With need_dx = 0 and an aggregation-first forward, dW = (A X)^T dZ needs no transposed
    aggregation (paper: cost-model paragraph on the first GNN layer).  Checked by poisoning the
    transposed structure: the backward must not read it."""
    from paper_2305_17469_amd import binding as B
    cfg = configs.tiny()
    blk = cfg["blocks"][0]
    announce("first layer: no backward aggregation")
    g = B.Graph(up_i32(blk["rowptr"]), up_i32(blk["colidx"]), blk["n_src"])
    d = B.make_desc("symnorm", "f32", True, 64, 64, need_dx=False)
    bufs = B.LayerBuffers(g, d)
    X, W, b = up_feat(cfg["X"], "f32"), up_feat(cfg["W"][0], "f32"), torch.from_numpy(cfg["b"][0]).cuda()
    Y, used = B.gt_layer_fwd(g, d, X, W, b, bufs, "agg_first")
    st = oracle.layer_fwd(blk, "symnorm", cfg["X"], cfg["W"][0], cfg["b"][0], True)
    one = dict(cfg, blocks=cfg["blocks"][:1], W=cfg["W"][:1], W_root=cfg["W_root"][:1], b=cfg["b"][:1])
    _, bounds = relu_rounding_sets(one, [dict(st, X=np.asarray(cfg["X"], np.float64))])
    amb = np.abs(st["Z"]) <= bounds[0]          # decisions rounding may flip: no gradient flows there
    dYh = np.where(amb, 0.0, 1.0).astype(np.float32)
    dY = up_feat(dYh, "f32")
    # the first region of the scratch is where A^T dZ would be written: fill it with a sentinel
    n_bytes = g.n_src * 64 * 4
    bufs.scratch[:n_bytes].fill_(0xAB)
    r1 = B.gt_layer_bwd(g, d, used, dY, X, W, Y, bufs, "auto")
    torch.cuda.synchronize()
    assert r1["used"] == "agg_first"
    assert bool((bufs.scratch[:n_bytes] == 0xAB).all())
    assert not (((down(Y) > 0) != (st["Z"] > 0)) & ~amb).any()
    og = oracle.layer_bwd(blk, "symnorm", cfg["X"], cfg["W"][0], st["Z"], dYh.astype(np.float64), True, need_dx=False)
    assert max_rel_err(down(r1["dW"]), og["dW"]) <= 1e-5


def test_layer_calls_check_buffer_sizes_and_overlap_before_launching():
    """Undersized `saved` / `scratch` give GT_ERR_WORKSPACE, overlapping X / Y GT_ERR_INVALID_ARG;
    all checks precede the first launch (the output stays untouched)."""
    from paper_2305_17469_amd import binding as B
    cfg = configs.tiny()
    blk = cfg["blocks"][0]
    announce("layer argument checks")
    g = B.Graph(up_i32(blk["rowptr"]), up_i32(blk["colidx"]), blk["n_src"])
    d = B.make_desc("symnorm", "f32", True, 64, 64)
    bufs = B.LayerBuffers(g, d)
    need_saved, need_scratch = B.gt_layer_ws_size(g, d)
    X, W, b = up_feat(cfg["X"], "f32"), up_feat(cfg["W"][0], "f32"), torch.from_numpy(cfg["b"][0]).cuda()
    Y = torch.full((g.n_dst, 64), 7.0, device="cuda")
    dX = torch.full((g.n_src, 64), 7.0, device="cuda")
    dW = torch.empty((64, 64), device="cuda")
    used = B.c_int()

    def fwd(saved_bytes, scratch_bytes, y=Y, order=B.GT_AGG_FIRST):
        return B.lib.gt_layer_fwd(g.handle, B.byref(d), order, X.data_ptr(), 64, W.data_ptr(), None, b.data_ptr(),
                                  y.data_ptr(), 64, bufs.saved.data_ptr(), saved_bytes, bufs.scratch.data_ptr(),
                                  scratch_bytes, B.byref(used), None)

    def bwd(saved_bytes, scratch_bytes, dx=dX):
        return B.lib.gt_layer_bwd(g.handle, B.byref(d), B.GT_AGG_FIRST, B.GT_AUTO, Y.data_ptr(), 64, X.data_ptr(), 64,
                                  W.data_ptr(), None, Y.data_ptr(), 64, bufs.saved.data_ptr(), saved_bytes,
                                  bufs.scratch.data_ptr(), scratch_bytes, dx.data_ptr(), 64, dW.data_ptr(), None, None,
                                  B.byref(used), None)

    assert fwd(need_saved, need_scratch - 1) == 3 and b"scratch_bytes" in B.lib.gt_last_error()
    assert fwd(need_saved - 1, need_scratch) == 3 and b"saved_bytes" in B.lib.gt_last_error()
    assert fwd(0, need_scratch, order=B.GT_COMB_FIRST) == 0          # `saved` is not written in this order
    Y.fill_(7.0)
    assert fwd(need_saved, need_scratch, y=X) == 1 and b"overlap" in B.lib.gt_last_error()
    assert bwd(need_saved, need_scratch - 1) == 3
    assert bwd(need_saved - 1, need_scratch) == 3
    assert bwd(need_saved, need_scratch, dx=X) == 1
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all()) and bool((dX == 7.0).all())
    assert fwd(need_saved, need_scratch) == 0 and bwd(need_saved, need_scratch) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,in_dim,out_dim", [("bf16", 64, 47), ("bf16", 47, 100), ("f32", 64, 41), ("f32", 41, 18)])
def test_pad_writable_touches_only_the_rest_of_a_rows_last_vector(dtype, in_dim, out_dim):
    """gt_layer_desc.pad_writable: the logical outputs are bit for bit what they are without it, the
    padding columns up to the next multiple of 16 bytes hold zeros afterwards or are untouched, every
    column beyond that (and, without the flag, all padding) is left as it was.  16,384 vertices, so that the
    tall-product kernels with the staged epilogues run."""
    from paper_2305_17469_amd import binding as B
    rp, ci = graphs.rmat_csr(14, 8, seed=77)
    n = rp.size - 1
    g = B.Graph(up_i32(rp), up_i32(ci), n)
    v = 8 if dtype == "bf16" else 4
    X = tensors.normal((n, in_dim), seed=1)
    W = tensors.glorot(in_dim, out_dim, seed=2)
    dY = tensors.normal((n, out_dim), seed=3)
    if dtype == "bf16":
        X, W, dY = tensors.bf16_values(X), tensors.bf16_values(W), tensors.bf16_values(dY)
    bias = torch.from_numpy(tensors.normal((out_dim,), seed=4)).cuda()
    Xd, Wd, dYd = up_feat(X, dtype, pad_to(in_dim, dtype)), up_feat(W, dtype), up_feat(dY, dtype, pad_to(out_dim, dtype))
    ldy, ldx = pad_to(out_dim, dtype) + 2 * v, pad_to(in_dim, dtype) + 2 * v
    for order in ("agg_first", "comb_first"):
        res = {}
        for flag in (False, True):
            announce("pad_writable", dtype, in_dim, out_dim, order, flag)
            d = B.make_desc("sum", dtype, True, in_dim, out_dim, in_relu=True, pad_writable=flag)
            bufs = B.LayerBuffers(g, d)
            Y = empty_feat(n, out_dim, dtype, ldy)
            dX = empty_feat(n, in_dim, dtype, ldx)
            _, used = B.gt_layer_fwd(g, d, Xd, Wd, bias, bufs, order, out=Y)
            r = B.gt_layer_bwd(g, d, used, dYd, Xd, Wd, Y, bufs, order, out_dX=dX)
            torch.cuda.synchronize()
            res[flag] = (Y.clone(), dX.clone(), r["dW"].clone(), r["db"].clone())
            for T, F, ld in ((Y, out_dim, ldy), (dX, in_dim, ldx)):
                full = T.as_strided((n, ld), (ld, 1), T.storage_offset()).float()
                edge = pad_to(F, dtype) if flag else F
                assert not torch.isnan(full[:, :F]).any()
                rest = full[:, F:edge]                               # the rest of the row's last vector: zeros, or untouched
                assert bool(((rest == 0) | torch.isnan(rest)).all())
                assert bool(torch.isnan(full[:, edge:]).all())       # nothing beyond it was written
                # the aggregation kernel writes these two (Y of a combination-first forward, dX of an
                # aggregation-first backward) and does store the zeros
                if flag and ((T is Y and order == "comb_first") or (T is dX and order == "agg_first")):
                    assert bool((rest == 0).all())
        for a, b in zip(res[False], res[True]):
            assert torch.equal(a, b)
