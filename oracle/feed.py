"""CPU oracle (TEST INFRASTRUCTURE) for the batch preparation steps of the paper's
"Preprocessing for GNNs" section: neighbour sampling (S), renumbering through the table of
sampled vertices (R) and embedding lookup (K).  Plain numpy / Python, one destination at a time.

What the paper fixes: S picks at most n distinct in-neighbours of every destination vertex of
the batch at random ("unique random"); every vertex that enters the subgraph receives a new id,
handed out from zero in the order the vertices are first met; R rewrites the subgraph in the new
ids; K fetches the embedding rows of the sampled vertices.  One subgraph is prepared per GNN
layer, the layer nearest the seeds first.

What the paper leaves open and this file defines (the GPU library defines the same, in code of
its own): the random choice.  It is a keyed pseudo-random permutation pi of the positions 0..d-1
of a destination's in-neighbour list (d = its in-degree); the picks are pi(0), ..., pi(n-1):
  * mix32 is an invertible 32-bit integer mixer (xor-shift / odd-multiply rounds);
  * the row key depends on (seed, stream, global destination id) only, so a vertex draws the
    same neighbours whatever else is in the batch;
  * short lists (d <= SMALL): position j gets the key mix32(row key + GOLD * (j + 1)), distinct
    for distinct j because mix32 is a bijection, and pi lists the positions by ascending key;
  * long lists: pi is a balanced Feistel network of ROUNDS rounds on 2h bits, h = ceil(b/2)
    for b the bit length of d-1, followed by cycle walking (re-apply until the value is < d);
    a Feistel network is a bijection whatever its round function is, so the n picks are
    distinct, and walking the cycle keeps it a bijection on 0..d-1.  (On very small domains a
    Feistel network reaches too few permutations to look uniform, hence the split.)
Destinations with d <= n keep their whole list in list order; the others list their picks in
the order t = 0..n-1.

Uniformity is a statistical property of this construction, not an identity: it is pinned by
chi-square tests in tests/test_oracle_feed_pins.py.
"""
from __future__ import annotations

import numpy as np

GOLD = 0x9E3779B9
ROUNDS = 6
SMALL = 64          # lists up to this length are ordered by per-position keys
_M32 = 0xFFFFFFFF


def mix32(x):
    """Invertible mixer on uint32 (array or scalar): x ^= x>>16; x *= 0x7feb352d; x ^= x>>15;
    x *= 0x846ca68b; x ^= x>>16 (all modulo 2^32)."""
    x = np.asarray(x, dtype=np.uint64) & _M32
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & _M32
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & _M32
    x ^= x >> np.uint64(16)
    return x


def row_key(seed: int, stream: int, v):
    """Key of destination v (scalar or array of global ids) under (seed, stream)."""
    s = int(mix32((int(seed) + GOLD * int(stream)) & _M32))
    k = mix32(np.uint64(s) ^ (np.asarray(v, dtype=np.uint64) & _M32))
    return int(k) if k.ndim == 0 else k


def _feistel_positions(t, d: int, rk):
    # t: [f] positions, rk: [n] row keys -> [n, f]
    b = int(d - 1).bit_length()
    h = (b + 1) // 2
    mask = np.uint64((1 << h) - 1)
    keys = [mix32((rk + np.uint64(GOLD * (r + 1))) & _M32)[:, None] for r in range(ROUNDS)]
    x = np.broadcast_to(t[None, :], (rk.size, t.size)).copy()
    todo = np.ones(x.shape, dtype=bool)
    while todo.any():
        L = x >> np.uint64(h)
        R = x & mask
        for r in range(ROUNDS):
            L, R = R, L ^ (mix32(R ^ keys[r]) & mask)
        x = np.where(todo, (L << np.uint64(h)) | R, x)
        todo = x >= d
    return x.astype(np.int64)


def permute_positions(t, d: int, rk):
    """pi(t) for an array of t in [0, d): the keyed permutation of 0..d-1 described above.
    rk is one row key (result has t's shape) or an array of n row keys (result [n, len(t)])."""
    t = np.asarray(t, dtype=np.int64)
    assert d >= 2 and t.ndim == 1 and (t >= 0).all() and (t < d).all()
    rks = np.atleast_1d(np.asarray(rk, dtype=np.uint64))
    if d <= SMALL:
        j1 = np.arange(1, d + 1, dtype=np.uint64)
        keys = mix32((rks[:, None] + np.uint64(GOLD) * j1[None, :]) & _M32)
        out = np.argsort(keys, axis=1, kind="stable")[:, t].astype(np.int64)
    else:
        out = _feistel_positions(t.astype(np.uint64), d, rks)
    return out[0] if np.ndim(rk) == 0 else out


def sample_neighbors(rowptr, colidx, dst, fanout: int, seed: int, stream: int):
    """S for one layer.  rowptr/colidx: in-edge CSR of the whole graph (global ids); dst: the
    layer's destination vertices (global ids).  Returns (rowptr_out[n_dst+1], picked global
    ids), row i holding min(deg(dst[i]), fanout) entries."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx)
    dst = np.asarray(dst, dtype=np.int64)
    assert fanout >= 1
    out_ptr = np.zeros(dst.size + 1, dtype=np.int64)
    rows = []
    for i, v in enumerate(dst):
        nb = colidx[rowptr[v]:rowptr[v + 1]]
        d = nb.size
        if d > fanout:
            pos = permute_positions(np.arange(fanout), d, row_key(seed, stream, int(v)))
            nb = nb[pos]
        rows.append(np.asarray(nb, dtype=np.int64))
        out_ptr[i + 1] = out_ptr[i] + rows[-1].size
    picked = np.concatenate(rows) if rows else np.zeros(0, dtype=np.int64)
    return out_ptr, picked


def reindex(dst, picked):
    """R: the table of sampled vertices.  Walk dst then picked in order; a global id met for the
    first time receives the next new id (from 0).  dst must hold distinct ids, so destination i
    gets new id i.  Returns (src_global[n_src], colidx_local[len(picked)])."""
    table = {}
    src_global = []
    for v in np.asarray(dst).tolist():
        if v in table:
            raise ValueError("destination ids must be distinct")
        table[v] = len(src_global)
        src_global.append(v)
    local = np.empty(len(picked), dtype=np.int64)
    for k, u in enumerate(np.asarray(picked).tolist()):
        nid = table.get(u)
        if nid is None:
            nid = len(src_global)
            table[u] = nid
            src_global.append(u)
        local[k] = nid
    return np.asarray(src_global, dtype=np.int64), local


def lookup(table, ids):
    """K: row ids[i] of the embedding table for every i."""
    table = np.asarray(table)
    out = np.empty((len(ids), table.shape[1]), dtype=table.dtype)
    for i, v in enumerate(np.asarray(ids).tolist()):
        out[i, :] = table[v, :]
    return out


def sample_blocks(rowptr, colidx, seeds, fanouts, seed: int):
    """The per-layer chain: S then R for the layer nearest the seeds (fanouts[0], stream 0), its
    sources become the destinations of the next layer outwards, and so on.  Returns the blocks
    ordered by layer (outermost first), each a dict(rowptr, colidx (new ids), n_dst, n_src,
    src_global)."""
    blocks = []
    dst = np.asarray(seeds, dtype=np.int64)
    for hop, fanout in enumerate(fanouts):
        ptr, picked = sample_neighbors(rowptr, colidx, dst, fanout, seed, hop)
        src_global, local = reindex(dst, picked)
        blocks.append(dict(rowptr=ptr, colidx=local, n_dst=int(dst.size), n_src=int(src_global.size),
                           src_global=src_global))
        dst = src_global
    blocks.reverse()
    return blocks
