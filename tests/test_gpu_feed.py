"""Batch preparation on the GPU (gt_sample_neighbors, gt_reindex, gt_lookup) against the oracle in
oracle/feed.py.  Integer and copy work: every comparison is bit-exact.

Inputs: R-MAT graphs (hubs far above the fanout, many vertices below it, isolated vertices),
destination sets that always contain the largest hubs, fanouts on both sides of the 64-entry
boundary between the two permutation constructions.
"""
import numpy as np
import pytest
import torch

from gt_inputs import graphs, tensors
from gpu_util import announce, dev, up_feat, up_i32
from oracle import feed as ofeed

pytestmark = pytest.mark.gpu


def _graph(scale=13, draws=20, seed=31):
    return graphs.rmat_csr(scale, draws, seed=seed, self_loops=False)


def _dst_with_hubs(rp, n, rng):
    deg = np.diff(rp)
    hubs = np.argsort(-deg)[:8]
    rest = rng.choice(np.setdiff1d(np.arange(rp.size - 1), hubs), n - hubs.size, replace=False)
    dst = np.concatenate([hubs, rest])
    rng.shuffle(dst)
    return dst


@pytest.mark.parametrize("fanout", [1, 5, 25, 64, 100, 4000])
def test_sampling_matches_oracle(fanout):
    from paper_2305_17469_amd import binding as B
    rp, ci = _graph()
    deg = np.diff(rp)
    assert deg.max() > 1000 and (deg == 0).any() and ((deg > 1) & (deg <= 64)).any()
    rng = np.random.default_rng(fanout)
    dst = _dst_with_hubs(rp, 700, rng)
    announce("sample", fanout, "n_dst", dst.size, "max degree", int(deg.max()))
    ptr, picked = B.gt_sample_neighbors(up_i32(rp), up_i32(ci), up_i32(dst), fanout, seed=17, stream_id=3)
    optr, opicked = ofeed.sample_neighbors(rp, ci, dst, fanout, seed=17, stream=3)
    assert np.array_equal(ptr.cpu().numpy(), optr)
    assert np.array_equal(picked.cpu().numpy(), opicked)
    # another seed or stream gives other picks
    _, other = B.gt_sample_neighbors(up_i32(rp), up_i32(ci), up_i32(dst), fanout, seed=18, stream_id=3)
    if fanout < deg.max():
        assert not np.array_equal(other.cpu().numpy(), opicked)


def test_sampling_edge_cases():
    from paper_2305_17469_amd import binding as B
    rp, ci = _graph(10, 8, 5)
    drp, dci = up_i32(rp), up_i32(ci)
    announce("sample: empty batch")
    ptr, picked = B.gt_sample_neighbors(drp, dci, up_i32(np.zeros(0)), 5, 1, 0)
    assert ptr.cpu().tolist() == [0] and picked.numel() == 0
    announce("sample: ids outside the graph give empty rows")
    dst = np.array([3, -1, rp.size - 1, 7, 1 << 30])
    ptr, picked = B.gt_sample_neighbors(drp, dci, up_i32(dst), 4, 1, 0)
    optr, opicked = ofeed.sample_neighbors(rp, ci, np.array([3, 7]), 4, 1, 0)
    p = ptr.cpu().numpy()
    assert p[1] == p[2] == p[3] and p[4] == p[5]          # rows 1, 2 and 4 are empty
    assert np.array_equal(picked.cpu().numpy(), opicked)
    announce("sample: argument checks")
    with pytest.raises(B.GtError):
        B.gt_sample_neighbors(drp, dci, up_i32(dst), 0, 1, 0)


@pytest.mark.parametrize("n_dst,n_picked,universe", [(0, 0, 10), (1, 0, 10), (0, 50, 20), (5, 40, 12), (300, 9000, 4000),
                                                       (5000, 120000, 1 << 20), (70000, 500000, 1 << 17),
                                                       # around the single-launch sort's capacity of 16,384 pairs,
                                                       # ids of one to four bytes, and the one-launch pass (<= 32 K)
                                                       (150, 16234, 200), (384, 16000, 1 << 30), (1000, 15384, 70000),
                                                       (1000, 15385, 70000), (2000, 30000, 1 << 25), (1, 1023, 1 << 16)])
def test_reindex_matches_oracle(n_dst, n_picked, universe):
    from paper_2305_17469_amd import binding as B
    rng = np.random.default_rng(n_dst + n_picked)
    dst = rng.choice(universe, n_dst, replace=False)
    picked = rng.integers(0, universe, n_picked)
    announce("reindex", n_dst, n_picked, universe)
    src, local = B.gt_reindex(up_i32(dst), up_i32(picked), universe)
    osrc, olocal = ofeed.reindex(dst, picked)
    assert np.array_equal(src.cpu().numpy(), osrc)
    assert np.array_equal(local.cpu().numpy(), olocal)


def test_reindex_reports_repeated_destinations():
    from paper_2305_17469_amd import binding as B
    announce("reindex: repeated destination")
    with pytest.raises(ValueError):
        B.gt_reindex(up_i32(np.array([3, 4, 3])), up_i32(np.array([1])), 10)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("F", [1, 3, 4, 100, 602])
def test_lookup_matches_oracle(F, dtype):
    from paper_2305_17469_amd import binding as B
    n_rows, n = 3000, 5000
    table = tensors.normal((n_rows, F), seed=F)
    if dtype == "bf16":
        table = tensors.bf16_values(table)
    ids = np.random.default_rng(F).integers(0, n_rows, n)
    ref = ofeed.lookup(table, ids)
    v = 8 if dtype == "bf16" else 4
    for ld in (F, (F + v - 1) // v * v + v):
        announce("lookup", dtype, F, "ld", ld)
        T = up_feat(table, dtype, ld)
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        buf = torch.full((n, ld + 1), 7.0, dtype=tdt, device=dev())
        out = buf[:, :F]
        B.gt_lookup(T, up_i32(ids), out=out)
        assert np.array_equal(out.float().cpu().numpy(), ref)
        assert (buf[:, F:] == 7.0).all()                 # nothing outside the F logical columns
    announce("lookup: id outside the table gives zeros", dtype, F)
    bad = up_i32(np.array([0, n_rows, -1, 5]))
    out = B.gt_lookup(up_feat(table, dtype), bad).float().cpu().numpy()
    assert np.array_equal(out[0], table[0]) and np.array_equal(out[3], table[5])
    assert (out[1] == 0).all() and (out[2] == 0).all()


def test_layer_chain_matches_oracle_and_feeds_the_model():
    """S and R chained over two layers on a graph with 2^18 vertices, 300 seeds as in the paper's
    evaluation; the blocks must equal the oracle's, pass the library's own structure check, and
    the embeddings fetched for the outermost sources must be the table's rows."""
    from paper_2305_17469_amd import binding as B, feed
    rp, ci = graphs.rmat_csr(18, 16, seed=2, self_loops=False)
    seeds = np.random.default_rng(8).choice(rp.size - 1, 300, replace=False)
    fanouts = (25, 10)
    announce("feed chain: 300 seeds, fanouts", fanouts)
    table = tensors.normal((rp.size - 1, 100), seed=9)
    T = up_feat(table, "f32")
    blocks, X = feed.prepare_batch(up_i32(rp), up_i32(ci), T, up_i32(seeds), fanouts, seed=5)
    oblocks = ofeed.sample_blocks(rp, ci, seeds, fanouts, seed=5)
    assert len(blocks) == len(oblocks) == 2
    for blk, oblk in zip(blocks, oblocks):
        assert (blk["n_dst"], blk["n_src"]) == (oblk["n_dst"], oblk["n_src"])
        for k in ("rowptr", "colidx", "src_global"):
            assert np.array_equal(blk[k].cpu().numpy(), oblk[k]), k
        g = B.Graph(blk["rowptr"], blk["colidx"], blk["n_src"])
        assert g.validate() == 0
    assert np.array_equal(X.cpu().numpy(), ofeed.lookup(table, oblocks[0]["src_global"]))
