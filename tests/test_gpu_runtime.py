"""Run-time facilities around the kernels: coefficient calibration, per-kernel event timing, and
replay of a whole fwd+bwd step from a captured HIP graph (the layer calls allocate nothing, never
synchronise and record no memset nodes, so a caller may capture them)."""
import numpy as np
import pytest
import torch

from gt_inputs import configs
from gpu_util import announce, pad_to, up_feat, up_i32

pytestmark = pytest.mark.gpu


def _stack(cfg, dev):
    from paper_2305_17469_amd.stack import LayerStack
    dt = cfg["dtype"]
    blocks, seen = [], {}
    for blk in cfg["blocks"]:
        if id(blk["rowptr"]) not in seen:
            seen[id(blk["rowptr"])] = dict(rowptr=up_i32(blk["rowptr"]), colidx=up_i32(blk["colidx"]),
                                           n_dst=blk["n_dst"], n_src=blk["n_src"])
        blocks.append(seen[id(blk["rowptr"])])
    sage = cfg["model"] == "sage"
    W = [up_feat(w, dt) for w in cfg["W"]]
    Wr = [up_feat(w, dt) for w in cfg["W_root"]] if sage else None
    bs = [torch.from_numpy(b).to(dev) for b in cfg["b"]]
    return LayerStack(blocks, cfg["dims"], dt, cfg["reduce"], W, bs, Wr)


def test_calibrate_fits_positive_coefficients_and_keeps_decisions():
    from paper_2305_17469_amd import binding as B
    announce("gt_calibrate")
    old = [B.gt_cost_get_dtype(d) for d in ("f32", "bf16")]
    try:
        c = B.gt_calibrate()                       # fits bf16, then fp32; returns the fp32 set
        fitted = {"f32": B.gt_cost_get_dtype("f32"), "bf16": B.gt_cost_get_dtype("bf16")}
        assert fitted["f32"].gamma_fwd == c.gamma_fwd and fitted["f32"].alpha_bwd == c.alpha_bwd   # installed
        for dt, cc in fitted.items():
            vals = {f[0]: getattr(cc, f[0]) for f in cc._fields_}
            print(dt, vals)
            assert all(np.isfinite(v) and v >= 0 for v in vals.values())
            assert vals["gamma_fwd"] > 0 and vals["gamma_bwd"] > 0 and vals["alpha_fwd"] > 0 and vals["alpha_bwd"] > 0
            # a gather of one feature takes between 0.05 and 50 ps on this class of device
            assert 5e-14 < vals["gamma_fwd"] < 5e-11 and 5e-14 < vals["gamma_bwd"] < 5e-11
            # the floor of an aggregation launch: a few microseconds
            assert 1e-6 <= vals["aggr_floor"] <= 2e-5
        # bf16 rows are half as long: gathering one feature must not cost more than in fp32
        assert fitted["bf16"].gamma_fwd <= 1.1 * fitted["f32"].gamma_fwd
        one = B.gt_calibrate_dtype("bf16")         # one data type alone leaves the other set untouched
        assert B.gt_cost_get_dtype("bf16").gamma_fwd == one.gamma_fwd
        assert B.gt_cost_get_dtype("f32").gamma_fwd == c.gamma_fwd
        # (2^14 vertices: on a few thousand vertices every kernel sits at its launch floor and the two
        # orders tie within the noise of a fit)
        cfg = configs.reddit_like(14)
        blk = cfg["blocks"][0]
        g = B.Graph(up_i32(blk["rowptr"]), up_i32(blk["colidx"]), blk["n_src"])
        for dt in ("f32", "bf16"):
            assert B.gt_layer_decide(g, B.make_desc("symnorm", dt, True, 602, 128, need_dx=False))[0] == "comb_first"
            assert B.gt_layer_decide(g, B.make_desc("symnorm", dt, True, 16, 1024))[0] == "agg_first"
    finally:
        B.gt_cost_set_dtype("f32", old[0])
        B.gt_cost_set_dtype("bf16", old[1])


def test_kernel_trace_records_every_gather_and_combine_launch():
    from paper_2305_17469_amd import binding as B
    announce("gt_trace")
    dev = torch.device("cuda:0")
    cfg = configs.tiny()
    m = _stack(cfg, dev)
    X, G = up_feat(cfg["X"], "f32"), up_feat(cfg["G"], "f32")
    m.step(X, G)
    B.gt_trace_reset()
    B.gt_trace_enable(True)
    m.step(X, G, "comb_first", "comb_first")
    torch.cuda.synchronize()
    B.gt_trace_enable(False)
    recs = B.gt_trace_records()
    B.gt_trace_reset()
    kinds = [r[0] for r in recs]
    # per layer: 1 forward gather, 1 transposed gather (A^T dZ), 3 combinations (X W, dW, dX) -- the
    # first layer has no dX
    assert kinds.count(0) == 2 and kinds.count(1) == 2 and kinds.count(2) == 5
    assert all(r[4] > 0 for r in recs)
    assert {r[1] for r in recs if r[0] == 0} == {64, 16}
    m.step(X, G)
    assert B.gt_trace_records() == []            # disabled: nothing recorded


@pytest.mark.parametrize("which", ["tiny", "sage"])
def test_step_replays_from_a_captured_graph(which):
    announce("graph capture of a fwd+bwd step:", which)
    dev = torch.device("cuda:0")
    cfg = configs.tiny() if which == "tiny" else configs.sage_minibatch(13, 128)
    m = _stack(cfg, dev)
    X, G = up_feat(cfg["X"], "f32"), up_feat(cfg["G"], "f32")
    m.step(X, G)                                  # eager reference (also fixes the AUTO orders)
    torch.cuda.synchronize()
    ref_out = m.H[-1].clone()
    ref_dW = [w.clone() for w in m.dW]
    ref_db = [b.clone() for b in m.db]
    graph = m.capture(X, G)
    torch.cuda.synchronize()
    for rep in range(4):
        # eager work and a synchronisation between replays; outputs are clobbered first
        m.H[-1].zero_()
        for w in m.dW:
            w.fill_(float(rep))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(m.H[-1], ref_out), rep
        for a, b in zip(m.dW, ref_dW):
            assert torch.equal(a, b), rep
        for a, b in zip(m.db, ref_db):
            assert torch.equal(a, b), rep


def test_weight_stationary_combination_replays_from_a_captured_graph():
    """The tall-product kernel needs more than 64 KB of LDS for a 256 x 256 bf16 weight matrix,
    which has to be allowed per kernel on the host; that must also work when the launch is
    captured, and every replay must reproduce the eager result bit for bit."""
    from paper_2305_17469_amd import binding as B
    announce("graph capture of the weight-stationary combination (154 KB of LDS)")
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(3)
    A = torch.randn((8200, 256), device=dev, generator=g).to(torch.bfloat16)
    W = torch.randn((256, 256), device=dev, generator=g).to(torch.bfloat16)
    bias = torch.randn(256, device=dev, generator=g)
    ref = B.gt_combine(A, W, bias, relu=True)
    torch.cuda.synchronize()
    out = torch.zeros_like(ref)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.gt_combine(A, W, bias, relu=True, out=out)
    torch.cuda.synchronize()
    for rep in range(3):
        out.fill_(float(rep))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), rep


def _time_step(m, X, G, fo, bo, reps=6):
    for _ in range(2):
        m.step(X, G, fo, bo)
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(3):                            # best of three timed groups: box noise only adds
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            m.step(X, G, fo, bo)
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps)
    return best


@pytest.mark.parametrize("which", ["c2_scale16", "c5a_scale18", "c5b_scale18", "c6a"])
def test_auto_placement_is_the_measured_faster_order(which):
    """Dynamic kernel placement under test: for every layer, both placements (aggregation-first and
    combination-first, forward and backward alike) are forced and timed; where they differ by more
    than 20 % AUTO must have picked the faster one (paper: the placement is chosen from the cost
    model so that the cheaper order runs)."""
    from paper_2305_17469_amd import binding as B
    cfg = {"c2_scale16": lambda: configs.reddit_like(16), "c5a_scale18": lambda: configs.reorder_stress(18, True, "sum"),
           "c5b_scale18": lambda: configs.reorder_stress(18, False, "sum"), "c6a": lambda: configs.paper_batch("light")}[which]()
    dev = torch.device("cuda:0")
    announce("placement under test:", cfg["name"])
    m = _stack(cfg, dev)
    dt = cfg["dtype"]
    X, G = up_feat(cfg["X"], dt, pad_to(cfg["dims"][0], dt)), up_feat(cfg["G"], dt, pad_to(cfg["dims"][-1], dt))
    m.step(X, G)
    auto_f, auto_b = list(m.used_fwd), list(m.used_bwd)
    decided = 0
    for l in range(m.L):
        t = {}
        for o in ("agg_first", "comb_first"):
            fo, bo = list(auto_f), list(auto_b)
            fo[l], bo[l] = o, o
            t[o] = _time_step(m, X, G, fo, bo)
        fast = min(t, key=t.get)
        slow = max(t, key=t.get)
        print(cfg["name"], "layer", l, cfg["dims"][l], "->", cfg["dims"][l + 1], t, "auto", auto_f[l], auto_b[l])
        if t[slow] > 1.2 * t[fast]:
            decided += 1
            assert auto_f[l] == fast, (cfg["name"], l, t, auto_f[l])
            if l > 0:
                assert auto_b[l] == fast, (cfg["name"], l, t, auto_b[l])
    assert decided >= 1, "no layer of this workload separates the two orders by 20 %"
