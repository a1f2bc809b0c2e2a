"""Seeded synthetic graph generators (inputs only; none of the method's arithmetic lives here).

All generators return an in-edge CSR in the paper's sense (Preliminaries, "Data representation"):
a pointer array indexed by destination vertex and a vertex array holding source ids, as int32
numpy arrays.  Rows are de-duplicated and sorted by source id.  Randomness comes from
numpy's counter-based Philox bit generator keyed by the given seed, so the same seed gives the
same arrays on every machine that has this numpy.
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def rmat_edges(scale: int, n_draws: int, seed: int, a=0.57, b=0.19, c=0.19, d=0.05):
    """R-MAT (src, dst) draws on 2**scale vertices.

    At each of `scale` bit levels one quadrant is drawn with probabilities (a, b, c, d) for
    (src-bit, dst-bit) = (0,0), (0,1), (1,0), (1,1); no noise is added to the probabilities.
    Returns two int64 arrays of length n_draws (duplicates and self-pairs still present).
    """
    assert abs(a + b + c + d - 1.0) < 1e-9
    rng = _rng(seed, 1)
    src = np.zeros(n_draws, dtype=np.int64)
    dst = np.zeros(n_draws, dtype=np.int64)
    t_ab = np.float32(a + b)
    t_a = np.float32(a)
    t_abc = np.float32(a + b + c)
    for _ in range(scale):
        r = rng.random(n_draws, dtype=np.float32)
        src_bit = r >= t_ab                       # quadrants c, d
        dst_bit = ((r >= t_a) & (r < t_ab)) | (r >= t_abc)   # quadrants b, d
        src <<= 1
        dst <<= 1
        src |= src_bit
        dst |= dst_bit
    return src, dst


def uniform_edges(n: int, n_draws: int, seed: int):
    """Erdos-Renyi style: n_draws independent uniform (src, dst) pairs on n vertices."""
    rng = _rng(seed, 2)
    src = rng.integers(0, n, size=n_draws, dtype=np.int64)
    dst = rng.integers(0, n, size=n_draws, dtype=np.int64)
    return src, dst


def csr_from_pairs(src, dst, n_dst: int, n_src: int, self_loops: bool = False):
    """De-duplicate (src, dst) pairs, optionally add the missing (v, v) pairs, and build the
    in-edge CSR: rowptr[n_dst+1], colidx[E] (sources of each destination, ascending)."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    if self_loops:
        assert n_dst == n_src
        loops = np.arange(n_dst, dtype=np.int64)
        src = np.concatenate([src, loops])
        dst = np.concatenate([dst, loops])
    key = dst * np.int64(n_src) + src
    key = np.unique(key)                          # sorted by (dst, src), duplicates dropped
    d = key // np.int64(n_src)
    colidx = (key - d * np.int64(n_src)).astype(np.int32)
    counts = np.bincount(d, minlength=n_dst)
    rowptr = np.zeros(n_dst + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] == colidx.size and rowptr[-1] < 2**31
    return rowptr.astype(np.int32), colidx


def rmat_csr(scale: int, avg_draws: int, seed: int, self_loops: bool = True):
    n = 1 << scale
    s, d = rmat_edges(scale, avg_draws * n, seed)
    return csr_from_pairs(s, d, n, n, self_loops=self_loops)


def er_csr(scale: int, avg_draws: float, seed: int):
    n = 1 << scale
    s, d = uniform_edges(n, int(avg_draws * n), seed)
    return csr_from_pairs(s, d, n, n, self_loops=False)


def sample_blocks(rowptr, colidx, n_seeds: int, fanouts, seed: int):
    """Uniform neighbour sampling into bipartite CSR blocks (one per GNN layer).

    `fanouts` is given from the seed hop outwards, e.g. (25, 10): the block nearest the seeds
    (used by the LAST layer) draws up to 25 distinct in-neighbours per destination, the next
    block up to 10.  In every block the destinations are the first n_dst local source ids and
    further sources get local ids in first-seen order (cf. the paper's "Preprocessing for
    GNNs": new ids are handed out from 0 in insertion order).

    Returns a list ordered by LAYER (outermost hop first); each entry is a dict with
    rowptr, colidx (local ids), n_dst, n_src and `src_global` (global id of each local source).
    """
    rng = _rng(seed, 3)
    n = rowptr.size - 1
    seeds = rng.choice(n, size=n_seeds, replace=False).astype(np.int64)
    blocks = []
    dst_global = seeds
    for fanout in fanouts:
        picked = []
        counts = np.zeros(dst_global.size, dtype=np.int64)
        for i, v in enumerate(dst_global):
            nb = colidx[rowptr[v]:rowptr[v + 1]]
            if nb.size > fanout:
                nb = nb[np.sort(rng.choice(nb.size, size=fanout, replace=False))]
            picked.append(nb.astype(np.int64))
            counts[i] = nb.size
        flat = np.concatenate(picked) if picked else np.zeros(0, dtype=np.int64)
        seen = np.concatenate([dst_global, flat])
        uniq, first = np.unique(seen, return_index=True)
        order = np.argsort(first, kind="stable")
        src_global = uniq[order]                  # first-seen order; destinations come first
        local_of = np.empty(uniq.size, dtype=np.int64)
        local_of[order] = np.arange(uniq.size)
        local = local_of[np.searchsorted(uniq, flat)]
        rp = np.zeros(dst_global.size + 1, dtype=np.int64)
        np.cumsum(counts, out=rp[1:])
        # sort each row by local source id so rows are canonical
        row_of = np.repeat(np.arange(dst_global.size, dtype=np.int64), counts)
        key = np.sort(row_of * np.int64(uniq.size) + local)
        local = (key - (key // np.int64(uniq.size)) * np.int64(uniq.size))
        blocks.append(dict(rowptr=rp.astype(np.int32), colidx=local.astype(np.int32),
                           n_dst=int(dst_global.size), n_src=int(src_global.size),
                           src_global=src_global))
        dst_global = src_global
    blocks.reverse()
    return blocks


def drawn_blocks(scale: int, n_seeds: int, fanouts, seed: int):
    """Sampled bipartite blocks drawn directly, without a base graph: every destination draws
    `fanout` in-neighbours from the source marginal of the R-MAT generator on 2**scale vertices
    (popular vertices are drawn often, as in a sampled power-law graph) and duplicates within a
    row are dropped.  Same conventions as `sample_blocks`: fanouts from the seed hop outwards,
    destinations are the first local source ids, new sources get ids in first-seen order, the
    list is ordered by layer.  Stands in for the paper's sampled batches (dataset table, "Sampled
    graph" columns), whose sampler settings are not given.
    """
    rng = _rng(seed, 4)
    n = 1 << scale
    dst_global = rng.choice(n, size=n_seeds, replace=False).astype(np.int64)
    blocks = []
    for hop, fanout in enumerate(fanouts):
        nd = dst_global.size
        flat, _ = rmat_edges(scale, nd * fanout, seed * 131 + hop)
        row_of = np.repeat(np.arange(nd, dtype=np.int64), fanout)
        key = np.unique(row_of * np.int64(n) + flat)          # per-row duplicates dropped
        row_of = key // np.int64(n)
        flat = key - row_of * np.int64(n)
        counts = np.bincount(row_of, minlength=nd)
        seen = np.concatenate([dst_global, flat])
        uniq, first = np.unique(seen, return_index=True)
        order = np.argsort(first, kind="stable")
        src_global = uniq[order]
        local_of = np.empty(uniq.size, dtype=np.int64)
        local_of[order] = np.arange(uniq.size)
        local = local_of[np.searchsorted(uniq, flat)]
        key = np.sort(row_of * np.int64(uniq.size) + local)   # rows canonical: ascending local id
        local = key - (key // np.int64(uniq.size)) * np.int64(uniq.size)
        rp = np.zeros(nd + 1, dtype=np.int64)
        np.cumsum(counts, out=rp[1:])
        blocks.append(dict(rowptr=rp.astype(np.int32), colidx=local.astype(np.int32),
                           n_dst=int(nd), n_src=int(src_global.size), src_global=src_global))
        dst_global = src_global
    blocks.reverse()
    return blocks
