"""A multi-layer GNN driven through gt_layer_fwd / gt_layer_bwd with every buffer allocated once.

Marshalling only: which kernels run, and in which order, is decided inside the library
(gt_layer_decide); this class keeps the device tensors alive and passes pointers.
"""
from __future__ import annotations

import torch

from . import binding as B


def _pad(F, dtype):
    v = 8 if dtype == "bf16" else 4
    return (F + v - 1) // v * v


class LayerStack:
    """`blocks`: per-layer dict(rowptr, colidx, n_dst, n_src) of device int32 tensors (a full
    graph repeats the same dict).  Weights are device tensors of the layer dtype, biases fp32.
    Hidden layers use ReLU, the last layer none; the first layer produces no input gradient."""

    def __init__(self, blocks, dims, dtype, reduce, W, b, W_root=None, pad=True, fold_relu_grad=True):
        self.dtype, self.reduce, self.dims = dtype, reduce, list(dims)
        self.tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.L = len(dims) - 1
        self.W, self.b = W, b
        self.W_root = W_root if W_root is not None else [None] * self.L
        self.graphs, seen = [], {}
        for blk in blocks:
            key = blk["rowptr"].data_ptr()
            if key not in seen:
                seen[key] = B.Graph(blk["rowptr"], blk["colidx"], blk["n_src"], blk.get("edge_weight"))
            self.graphs.append(seen[key])
        dev = self.graphs[0].device
        ld = (lambda F: _pad(F, dtype)) if pad else (lambda F: F)

        # one zero-filled slab per element type (one fill launch instead of one per tensor);
        # every tensor starts on a 256-byte boundary
        def carve(shapes, tdt):
            es = torch.empty((), dtype=tdt).element_size()
            offs, off = [], 0
            for sh in shapes:
                offs.append(off)
                n = 1
                for v in sh:
                    n *= v
                off += (n * es + 255) // 256 * 256 // es
            slab = torch.zeros(max(off, 1), dtype=tdt, device=dev)
            return [slab[o:o + sh[0] * sh[1]].view(sh) if len(sh) == 2 else slab[o:o + sh[0]] for o, sh in zip(offs, shapes)]

        self.descs, self.bufs = [], []
        feat_shapes, f32_shapes = [], []
        for l in range(self.L):
            g = self.graphs[l]
            # hidden layers end in a ReLU: the layer above folds its derivative into the gradient it
            # hands down (in_relu), and the layer itself then takes that gradient as dZ (dy_is_dz)
            d = B.make_desc(reduce, dtype, l < self.L - 1, dims[l], dims[l + 1], has_root=self.W_root[l] is not None,
                            need_dx=l > 0, in_relu=fold_relu_grad and l > 0, dy_is_dz=fold_relu_grad and l < self.L - 1,
                            pad_writable=pad)   # H and dH below are this class's own padded buffers
            self.descs.append(d)
            self.bufs.append(B.LayerBuffers(g, d))
            feat_shapes += [(g.n_dst, ld(dims[l + 1])), (g.n_src if l > 0 else 0, ld(dims[l]))]
            f32_shapes += [(dims[l], dims[l + 1]), (dims[l], dims[l + 1]) if self.W_root[l] is not None else (0, 1),
                           (dims[l + 1],)]
        feat = carve(feat_shapes, self.tdt)
        f32 = carve(f32_shapes, torch.float32)
        self.H = [feat[2 * l][:, :dims[l + 1]] for l in range(self.L)]
        self.dH = [feat[2 * l + 1][:, :dims[l]] if l > 0 else None for l in range(self.L)]
        self.dW = [f32[3 * l] for l in range(self.L)]
        self.dW_root = [f32[3 * l + 1] if self.W_root[l] is not None else None for l in range(self.L)]
        self.db = [f32[3 * l + 2] for l in range(self.L)]
        self.used_fwd = [None] * self.L
        self.used_bwd = [None] * self.L

    def forward(self, X, order="auto"):
        orders = order if isinstance(order, (list, tuple)) else [order] * self.L
        self.X = X
        h = X
        for l in range(self.L):
            _, self.used_fwd[l] = B.gt_layer_fwd(self.graphs[l], self.descs[l], h, self.W[l], self.b[l], self.bufs[l],
                                                 orders[l], self.W_root[l], out=self.H[l])
            h = self.H[l]
        return h

    def backward(self, dOut, order="auto"):
        orders = order if isinstance(order, (list, tuple)) else [order] * self.L
        dh = dOut
        stream = B._stream()
        for l in reversed(range(self.L)):
            g, d = self.graphs[l], self.descs[l]
            x = self.X if l == 0 else self.H[l - 1]
            dX = self.dH[l]
            used = B.c_int()
            B._check(B.lib.gt_layer_bwd(g.handle, B.byref(d), B.ORDER[self.used_fwd[l]], B.ORDER[orders[l]],
                                        B._ptr(dh), dh.stride(0), B._ptr(x), x.stride(0), B._ptr(self.W[l]),
                                        B._ptr(self.W_root[l]), B._ptr(self.H[l]), self.H[l].stride(0),
                                        B._ptr(self.bufs[l].saved), self.bufs[l].saved.numel(),
                                        B._ptr(self.bufs[l].scratch), self.bufs[l].scratch.numel(),
                                        B._ptr(dX), dX.stride(0) if dX is not None else 0, B._ptr(self.dW[l]),
                                        B._ptr(self.dW_root[l]), B._ptr(self.db[l]), B.byref(used), stream))
            self.used_bwd[l] = B.ORDER_NAME[used.value]
            dh = dX
        return self.dW, self.db

    def step(self, X, dOut, fwd_order="auto", bwd_order="auto"):
        self.forward(X, fwd_order)
        self.backward(dOut, bwd_order)

    def capture(self, X, dOut, fwd_order="auto", bwd_order="auto"):
        """One fwd+bwd step recorded into a HIP graph (for launch-bound workloads): the layer calls
        allocate nothing and never synchronise, so the whole step is capturable.  Runs the step once
        eagerly on a side stream first (placement decisions are taken there), then records it.
        Returns the graph; `graph.replay()` re-runs the step on the same buffers (X, dOut, the
        stack's outputs and gradients)."""
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step(X, dOut, fwd_order, bwd_order)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                self.step(X, dOut, fwd_order, bwd_order)
        torch.cuda.current_stream().wait_stream(side)
        return graph
