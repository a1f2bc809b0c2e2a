"""The five benchmark workloads as seeded synthetic inputs (shapes of the paper's dataset table;
the public graphs themselves are not used).  `scale` can be lowered for tests: the recipe stays
the same, only the vertex count changes.

Every workload is a dict:
  name, dtype ("f32" | "bf16"), model ("gcn" | "sage"), reduce ("sum"|"mean"|"symnorm"),
  blocks : list (one per layer) of dict(rowptr, colidx, n_dst, n_src)
  dims   : [F_in, hidden..., F_out]
  X      : fp32 [n_src(layer 1), F_in]   (bf16-representable values when dtype == "bf16")
  W, b   : per layer fp32 Glorot [F_l, F_{l+1}] / bias 0.1 N(0,1) [F_{l+1}] (non-zero, so that a
           dropped or misplaced bias shows in every comparison);  W_root for "sage"
  G      : fp32 upstream gradient of the linear probe loss L = <G, Out>, shape of the output
"""
from __future__ import annotations

import functools

import numpy as np

from . import graphs, tensors


def _dense(seed, n_rows, dims, dtype, sage=False, n_out=None):
    X = tensors.normal((n_rows, dims[0]), seed, 10)
    W, Wr, b = [], [], []
    for l in range(len(dims) - 1):
        w = tensors.glorot(dims[l], dims[l + 1], seed, 20 + l)
        wr = tensors.glorot(dims[l], dims[l + 1], seed, 40 + l) if sage else None
        if dtype == "bf16":
            w = tensors.bf16_values(w)
        W.append(w)
        Wr.append(wr)
        b.append((0.1 * tensors.normal((dims[l + 1],), seed, 50 + l)).astype(np.float32))
    if dtype == "bf16":
        X = tensors.bf16_values(X)
    G = tensors.normal((n_out if n_out is not None else n_rows, dims[-1]), seed, 30)
    if dtype == "bf16":
        G = tensors.bf16_values(G)
    return X, W, Wr, b, G


def _full_graph_cfg(name, rowptr, colidx, dims, dtype, reduce, seed):
    n = rowptr.size - 1
    blk = dict(rowptr=rowptr, colidx=colidx, n_dst=n, n_src=n)
    X, W, Wr, b, G = _dense(seed, n, dims, dtype)
    return dict(name=name, dtype=dtype, model="gcn", reduce=reduce,
                blocks=[blk] * (len(dims) - 1), dims=list(dims), X=X, W=W, W_root=Wr, b=b, G=G)


@functools.lru_cache(maxsize=4)
def tiny(scale: int = 12):
    """Config 1: R-MAT, 16 draws per vertex, dedup, self-loops; fp32 dim 64; GCN 64-64-16."""
    rp, ci = graphs.rmat_csr(scale, 16, seed=1, self_loops=True)
    return _full_graph_cfg("c1_tiny", rp, ci, (64, 64, 16), "f32", "symnorm", 1)


@functools.lru_cache(maxsize=2)
def reddit_like(scale: int = 18):
    """Config 2: R-MAT, 50 draws per vertex, self-loops; fp32 dim 602; GCN 602-128-41."""
    rp, ci = graphs.rmat_csr(scale, 50, seed=2, self_loops=True)
    return _full_graph_cfg("c2_rmat18_f602", rp, ci, (602, 128, 41), "f32", "symnorm", 2)


@functools.lru_cache(maxsize=2)
def products_like(scale: int = 21):
    """Config 3: R-MAT, 25 draws per vertex, self-loops, heavy hubs; bf16 dim 100;
    GCN 100-256-256-47 with fp32 accumulation."""
    rp, ci = graphs.rmat_csr(scale, 25, seed=3, self_loops=True)
    return _full_graph_cfg("c3_rmat21_bf16", rp, ci, (100, 256, 256, 47), "bf16", "symnorm", 3)


@functools.lru_cache(maxsize=2)
def sage_minibatch(scale: int = 21, n_seeds: int = 1024):
    """Config 4: 1,024 seeds, fanout (25, 10) on the config-3 style base graph (no self-loops
    needed: the root linear carries the vertex's own row); mean aggregation + root linear;
    fp32 256-256-47."""
    rp, ci = graphs.rmat_csr(scale, 25, seed=3, self_loops=False)
    blocks = graphs.sample_blocks(rp, ci, n_seeds, (25, 10), seed=4)
    dims = (256, 256, 47)
    X, W, Wr, b, G = _dense(4, blocks[0]["n_src"], dims, "f32", sage=True,
                            n_out=blocks[-1]["n_dst"])
    return dict(name="c4_sage_minibatch", dtype="f32", model="sage", reduce="mean",
                blocks=blocks, dims=list(dims), X=X, W=W, W_root=Wr, b=b, G=G)


@functools.lru_cache(maxsize=2)
def paper_batch(kind: str = "light", n_seeds: int = 300, scale: int | None = None):
    """The paper's own training regime (Evaluation, "GNN models" and "Workloads and datasets"):
    a batch of 300 seed vertices, two GCN layers with mean aggregation and hidden width 64.
    Two shapes from the dataset table's "Sampled graph" columns:
      "light": the reddit2 row  (feature 602, 41 outputs, about 185 K sampled vertices, 57 K
               destinations, 0.9 M edges),
      "heavy": the wiki-talk row (feature 4353, 2 outputs, about 29 K vertices, 8 K
               destinations, 60 K edges).
    The sampler's fanouts are not given in the paper; they are chosen here so that the drawn
    blocks come out near those sizes (light: 91 K vertices, 44 K destinations, 0.88 M edges;
    heavy: 34 K vertices, 7 K destinations, 52 K edges)."""
    if kind == "light":
        sc, fanouts, dims, seed = scale or 18, (600, 16), (602, 64, 41), 6
    elif kind == "heavy":
        sc, fanouts, dims, seed = scale or 21, (27, 6), (4353, 64, 2), 7
    else:
        raise ValueError(kind)
    blocks = graphs.drawn_blocks(sc, n_seeds, fanouts, seed)
    X, W, Wr, b, G = _dense(seed, blocks[0]["n_src"], dims, "f32", n_out=blocks[-1]["n_dst"])
    return dict(name="c6_paper_batch_%s" % kind, dtype="f32", model="gcn", reduce="mean",
                blocks=blocks, dims=list(dims), X=X, W=W, W_root=Wr, b=b, G=G)


@functools.lru_cache(maxsize=4)
def reorder_stress(scale: int = 20, wide_to_narrow: bool = True, reduce: str = "sum",
                   wide: int = 1024, narrow: int = 16):
    """Config 5: uniform random graph, 16 draws per vertex, no self-loops; one GCN layer
    wide->narrow or narrow->wide, sum or mean."""
    rp, ci = graphs.er_csr(scale, 16, seed=5)
    dims = (wide, narrow) if wide_to_narrow else (narrow, wide)
    name = "c5_er%d_%dto%d_%s" % (scale, dims[0], dims[1], reduce)
    return _full_graph_cfg(name, rp, ci, dims, "f32", reduce, 5)
