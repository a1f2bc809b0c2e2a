"""Pins for the batch-preparation oracle (oracle/feed.py): what the paper's "Preprocessing for
GNNs" section and plain mathematics fix about sampling (S), renumbering (R) and lookup (K).

  * the mixer is a bijection (checked against its inverse, written here from modular
    inverses), hence picks within a row cannot collide;
  * the keyed position map is a permutation of 0..d-1 for every d (brute force);
  * "unique random": every position, every unordered pair and every first pick is chosen
    equally often over many rows (chi-square against the uniform law, fixed keys);
  * S returns min(degree, n) distinct true in-neighbours and does not depend on the rest of the
    batch;
  * R is the unique renumbering with: destinations first, ids in first-met order, exact round
    trip (brute force through numpy.unique, a different algorithm from the oracle's table walk);
  * the paper's worked example (preprocessing figure: V5 <- {V8, V9}, then V8 <- {V9, new}).
"""
import numpy as np
import pytest

from gt_inputs import graphs
from oracle import feed

M32 = 0xFFFFFFFF


def _unxorshift(x, s):
    y = x
    k = s
    while k < 32:
        y = x ^ (y >> s)
        k += s
    return y & M32


def _mix32_inverse(y):
    y = _unxorshift(y, 16)
    y = (y * pow(0x846CA68B, -1, 1 << 32)) & M32
    y = _unxorshift(y, 15)
    y = (y * pow(0x7FEB352D, -1, 1 << 32)) & M32
    y = _unxorshift(y, 16)
    return y


def test_mixer_is_a_bijection():
    rng = np.random.default_rng(0)
    xs = np.concatenate([np.arange(0, 70000), rng.integers(0, 1 << 32, 30000)]).astype(np.uint64)
    ys = feed.mix32(xs)
    assert np.unique(ys[:70000]).size == 70000
    back = np.array([_mix32_inverse(int(y)) for y in ys[::37]], dtype=np.uint64)
    assert (back == xs[::37]).all()
    # scalar definition, written out once more with Python integers
    x = 0x12345678
    r = x ^ (x >> 16)
    r = (r * 0x7FEB352D) & M32
    r ^= r >> 15
    r = (r * 0x846CA68B) & M32
    r ^= r >> 16
    assert int(feed.mix32(x)) == r


@pytest.mark.parametrize("d", [2, 3, 4, 5, 7, 8, 9, 16, 17, 31, 33, 64, 100, 257, 1000, 4097, 65539])
def test_position_map_is_a_permutation(d):
    for rk in (0, 1, 0xDEADBEEF, 12345):
        p = feed.permute_positions(np.arange(d), d, rk)
        assert p.min() == 0 and p.max() == d - 1 and np.unique(p).size == d


def _chi2_ok(counts, expected):
    df = counts.size - 1
    stat = float(((counts - expected) ** 2 / expected).sum())
    return stat < df + 6.0 * np.sqrt(2.0 * df) + 6.0, stat


@pytest.mark.parametrize("d,f", [(3, 1), (3, 2), (5, 2), (8, 3), (17, 5), (64, 10), (65, 10), (129, 7), (300, 25),
                                 (1000, 3), (5000, 2)])
def test_every_position_is_picked_equally_often(d, f):
    n_rows = 30000 if d < 1000 else 200000
    p = feed.permute_positions(np.arange(f), d, feed.row_key(7, 1, np.arange(n_rows)))
    assert p.shape == (n_rows, f)
    assert np.array_equal(p[123], feed.permute_positions(np.arange(f), d, feed.row_key(7, 1, 123)))
    counts = np.bincount(p.ravel(), minlength=d).astype(float)
    first = np.bincount(p[:, 0], minlength=d).astype(float)
    ok, stat = _chi2_ok(counts, n_rows * f / d)
    assert ok, ("positions", d, f, stat)
    ok, stat = _chi2_ok(first, n_rows / d)
    assert ok, ("first pick", d, f, stat)


@pytest.mark.parametrize("d", [4, 5, 7, 65, 70])
def test_every_pair_is_picked_equally_often(d):
    n_rows = 20000 if d < 10 else 60000
    p = feed.permute_positions(np.arange(2), d, feed.row_key(3, 0, np.arange(n_rows)))
    pairs = np.zeros((d, d))
    np.add.at(pairs, (p.min(axis=1), p.max(axis=1)), 1)
    iu = np.triu_indices(d, 1)
    ok, stat = _chi2_ok(pairs[iu], n_rows / iu[0].size)
    assert ok, (d, stat)


def test_keys_separate_seeds_streams_and_vertices():
    base = feed.permute_positions(np.arange(8), 1000, feed.row_key(1, 0, 42))
    assert not np.array_equal(base, feed.permute_positions(np.arange(8), 1000, feed.row_key(2, 0, 42)))
    assert not np.array_equal(base, feed.permute_positions(np.arange(8), 1000, feed.row_key(1, 1, 42)))
    assert not np.array_equal(base, feed.permute_positions(np.arange(8), 1000, feed.row_key(1, 0, 43)))


def _graph():
    return graphs.rmat_csr(10, 12, seed=21, self_loops=False)


def test_sampling_returns_distinct_true_neighbours():
    rp, ci = _graph()
    rng = np.random.default_rng(1)
    dst = rng.choice(rp.size - 1, 200, replace=False)
    for fanout in (1, 4, 10, 1000):
        ptr, picked = feed.sample_neighbors(rp, ci, dst, fanout, seed=5, stream=0)
        assert ptr[0] == 0 and ptr[-1] == picked.size
        for i, v in enumerate(dst):
            nb = ci[rp[v]:rp[v + 1]]
            row = picked[ptr[i]:ptr[i + 1]]
            assert row.size == min(nb.size, fanout)
            assert np.unique(row).size == row.size
            assert np.isin(row, nb).all()
            if nb.size <= fanout:
                assert np.array_equal(row, nb)          # whole list, list order


def test_sampling_of_a_vertex_does_not_depend_on_the_batch():
    rp, ci = _graph()
    dst = np.array([5, 17, 300, 9, 511])
    ptr, picked = feed.sample_neighbors(rp, ci, dst, 3, seed=9, stream=2)
    perm = np.array([4, 2, 0, 1, 3])
    ptr2, picked2 = feed.sample_neighbors(rp, ci, dst[perm], 3, seed=9, stream=2)
    for k, i in enumerate(perm):
        assert np.array_equal(picked[ptr[i]:ptr[i + 1]], picked2[ptr2[k]:ptr2[k + 1]])
    _, other = feed.sample_neighbors(rp, ci, dst, 3, seed=10, stream=2)
    assert not np.array_equal(picked, other)


def _first_met_brute_force(dst, picked):
    seq = np.concatenate([dst, picked])
    uniq, first = np.unique(seq, return_index=True)
    return uniq[np.argsort(first, kind="stable")]


def test_renumbering_is_first_met_order_and_round_trips():
    rng = np.random.default_rng(2)
    for n_dst, e, universe in ((1, 0, 10), (5, 40, 12), (50, 700, 300), (300, 5000, 100000)):
        dst = rng.choice(universe, n_dst, replace=False)
        picked = rng.integers(0, universe, e)
        src, local = feed.reindex(dst, picked)
        assert np.array_equal(src[:n_dst], dst)                 # destination i keeps id i
        assert np.unique(src).size == src.size
        assert np.array_equal(src[local], picked)               # exact round trip
        assert np.array_equal(src, _first_met_brute_force(dst, picked))


def test_renumbering_rejects_repeated_destinations():
    with pytest.raises(ValueError):
        feed.reindex(np.array([3, 4, 3]), np.array([1]))


def test_paper_worked_example():
    """Preprocessing figure: the batch holds V5; its sampled neighbours V8 and V9 receive the next
    new ids; for the next layer V8 draws V9 (already in the table: no new id) and one vertex not
    seen before (any id, here V2), which receives the next id."""
    src2, local2 = feed.reindex(np.array([5]), np.array([8, 9]))
    assert src2.tolist() == [5, 8, 9] and local2.tolist() == [1, 2]
    # layer 1: destinations are the layer-2 sources; V5 keeps {8, 9}, V8 draws {9, 2}, V9 draws {8}
    src1, local1 = feed.reindex(src2, np.array([8, 9, 9, 2, 8]))
    assert src1.tolist() == [5, 8, 9, 2]
    assert local1.tolist() == [1, 2, 2, 3, 1]


def test_lookup_fetches_the_named_rows():
    table = np.arange(40, dtype=np.float32).reshape(10, 4)
    ids = np.array([9, 0, 3, 3])
    out = feed.lookup(table, ids)
    assert out.shape == (4, 4) and out.dtype == np.float32
    for i, v in enumerate(ids):
        assert out[i].tolist() == [4.0 * v, 4.0 * v + 1, 4.0 * v + 2, 4.0 * v + 3]
    perm = np.random.default_rng(3).permutation(10)
    inv = np.argsort(perm)
    assert np.array_equal(feed.lookup(feed.lookup(table, perm), inv), table)


def test_layer_chain_is_consistent_with_the_graph():
    rp, ci = _graph()
    seeds = np.random.default_rng(4).choice(rp.size - 1, 16, replace=False)
    blocks = feed.sample_blocks(rp, ci, seeds, (5, 3), seed=11)
    assert len(blocks) == 2
    inner, outer = blocks[1], blocks[0]
    assert np.array_equal(inner["src_global"][:16], seeds)
    assert outer["n_dst"] == inner["n_src"]
    assert np.array_equal(outer["src_global"][:outer["n_dst"]], inner["src_global"])
    for blk, fanout in ((inner, 5), (outer, 3)):
        sg = blk["src_global"]
        for i in range(blk["n_dst"]):
            v = sg[i]
            nb = ci[rp[v]:rp[v + 1]]
            row = sg[blk["colidx"][blk["rowptr"][i]:blk["rowptr"][i + 1]]]
            assert row.size == min(nb.size, fanout) and np.isin(row, nb).all()
