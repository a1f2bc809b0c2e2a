"""Batch preparation driver: chains the library's S (sampling), R (renumbering) and K (lookup)
entry points into per-layer blocks, the way the paper's preprocessing does for every batch
(Preliminaries, "Preprocessing for GNNs"): the layer nearest the seeds first, each layer's source
list becoming the next layer's destinations, embeddings fetched for the outermost sources.

Marshalling only; all work happens in the library's kernels on the current torch stream.
"""
from __future__ import annotations

from . import binding as B


def sample_blocks(rowptr, colidx, seeds, fanouts, seed):
    """rowptr, colidx: int32 device tensors (whole graph, in-edge CSR); seeds: int32 device
    tensor of distinct global ids; fanouts from the seed hop outwards.  Returns the blocks
    ordered by layer (outermost first): dict(rowptr, colidx (new ids), n_dst, n_src, src_global),
    all device tensors."""
    n_vertices = rowptr.numel() - 1
    blocks = []
    dst = seeds
    for hop, fanout in enumerate(fanouts):
        ptr, picked = B.gt_sample_neighbors(rowptr, colidx, dst, fanout, seed, hop)
        src_global, local = B.gt_reindex(dst, picked, n_vertices)
        blocks.append(dict(rowptr=ptr, colidx=local, n_dst=int(dst.numel()), n_src=int(src_global.numel()),
                           src_global=src_global))
        dst = src_global
    blocks.reverse()
    return blocks


def prepare_batch(rowptr, colidx, table, seeds, fanouts, seed):
    """S and R for every layer, then K on the outermost source list.  Returns (blocks, X)."""
    blocks = sample_blocks(rowptr, colidx, seeds, fanouts, seed)
    X = B.gt_lookup(table, blocks[0]["src_global"])
    return blocks, X
