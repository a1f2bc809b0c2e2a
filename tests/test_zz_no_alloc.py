"""gt_aggregate_fwd_static (the entry point that allocates nothing: partial rows of split long
rows go to a fixed array inside the library) against gt_aggregate_fwd with a caller workspace:
same kernels, so the outputs must agree bit for bit, and both must match the oracle.  Two calls in
a row share the array; the second, on a smaller input, must not be disturbed by what the first
left there."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from gt_inputs import graphs, tensors
from gpu_util import announce, down, empty_feat, max_rel_err, tol_for, up_feat, up_i32

pytestmark = pytest.mark.gpu


def _hub_graph(scale, hubs, seed):
    """R-MAT graph plus planted hub rows of the given in-degrees (split into chunk work items)."""
    rp, ci = graphs.rmat_csr(scale, 8, seed=seed, self_loops=False)
    n = rp.size - 1
    dst = np.repeat(np.arange(n), np.diff(rp))
    rng = np.random.default_rng(seed)
    es = np.concatenate([rng.choice(n, h, replace=False) for h in hubs])
    ed = np.concatenate([np.full(h, 11 + 97 * i) for i, h in enumerate(hubs)])
    rp, ci = graphs.csr_from_pairs(np.concatenate([ci, es]), np.concatenate([dst, ed]), n, n)
    return rp, ci, n


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_scratch_entry_point_matches_workspace_entry_point(dtype):
    from paper_2305_17469_amd import binding as B
    cap = ctypes.c_size_t()
    assert B.lib.gt_aggregate_static_capacity(ctypes.byref(cap)) == 0 and cap.value == 32 << 20
    cases = [(_hub_graph(13, (3000, 1500, 700), 41), 200), (_hub_graph(11, (900,), 42), 40)]   # second: smaller
    for (rp, ci, n), F in cases:
        g = B.Graph(up_i32(rp), up_i32(ci), n)
        assert g.info()["fwd_split_rows"] >= 1
        need = ctypes.c_size_t()
        assert B.lib.gt_aggregate_ws_size(g.handle, F, ctypes.byref(need)) == 0 and 0 < need.value <= cap.value
        X = tensors.normal((n, F), seed=300 + F)
        if dtype == "bf16":
            X = tensors.bf16_values(X)
        Xd = up_feat(X, dtype)
        for reduce in ("sum", "mean", "symnorm"):
            announce("static scratch:", dtype, "n", n, "F", F, reduce)
            ref_gpu = B.gt_aggregate_fwd(g, reduce, Xd)
            out = empty_feat(n, F, dtype)
            B.gt_aggregate_fwd_static(g, reduce, Xd, out)
            torch.cuda.synchronize()
            assert torch.equal(out, ref_gpu), (dtype, F, reduce)
            ref = oracle.aggregate_fwd(rp, ci, n, X, reduce)
            if dtype == "bf16":
                ref = oracle.round_bf16(ref)
            assert max_rel_err(down(out), ref) <= tol_for(dtype), (dtype, F, reduce)


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2305_17469_amd import binding as B
    announce("static scratch: capacity check")
    rp, ci, n = _hub_graph(11, (1800, 900), 43)
    g = B.Graph(up_i32(rp), up_i32(ci), n)
    F = 1 << 20                       # partial rows of this width cannot fit 32 MiB
    need = ctypes.c_size_t()
    assert B.lib.gt_aggregate_ws_size(g.handle, F, ctypes.byref(need)) == 0 and need.value > 32 << 20
    st = B.lib.gt_aggregate_fwd_static(g.handle, 0, 0, F, ctypes.c_void_p(256), F, ctypes.c_void_p(512), F, None)
    assert st == 3 and b"exceed" in B.lib.gt_last_error()     # GT_ERR_WORKSPACE, nothing launched
    assert B.lib.gt_aggregate_fwd_static(None, 0, 0, 8, None, 8, None, 8, None) == 1
