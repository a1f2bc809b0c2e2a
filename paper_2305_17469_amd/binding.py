"""ctypes binding of libgt.so: the same entry points as include/gt.h, taking torch tensors.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.  torch
is used for device memory and for the current stream.  There is no CPU fallback: importing this
module fails if the library has not been built (`python -m paper_2305_17469_amd.build`).
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgt.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libgt.so is not built; run `python -m paper_2305_17469_amd.build` "
                      "(there is no fallback implementation)")
lib = ctypes.CDLL(LIB_PATH)

GT_OK = 0
GT_F32, GT_BF16 = 0, 1
GT_SUM, GT_MEAN, GT_SYMNORM = 0, 1, 2
GT_AUTO, GT_AGG_FIRST, GT_COMB_FIRST = 0, 1, 2
GT_ACT_NONE, GT_ACT_RELU = 0, 1
REDUCE = {"sum": GT_SUM, "mean": GT_MEAN, "symnorm": GT_SYMNORM}
ORDER = {"auto": GT_AUTO, "agg_first": GT_AGG_FIRST, "comb_first": GT_COMB_FIRST}
ORDER_NAME = {v: k for k, v in ORDER.items()}
STATUS_NAME = {0: "GT_OK", 1: "GT_ERR_INVALID_ARG", 2: "GT_ERR_UNSUPPORTED", 3: "GT_ERR_WORKSPACE",
               4: "GT_ERR_HIP", 5: "GT_ERR_INTERNAL"}


class gt_layer_desc(ctypes.Structure):
    _fields_ = [("reduce", c_int), ("dtype", c_int), ("act", c_int), ("in_dim", c_int64), ("out_dim", c_int64),
                ("has_root", c_int), ("need_dx", c_int), ("in_act", c_int), ("dy_is_dz", c_int),
                ("pad_writable", c_int)]


class gt_cost_coeffs(ctypes.Structure):
    _fields_ = [(n, c_double) for n in ("alpha_fwd", "beta_fwd", "gamma_fwd", "delta_fwd",
                                        "alpha_bwd", "beta_bwd", "gamma_bwd", "delta_bwd", "aggr_floor")]


class GtError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("%s: %s" % (STATUS_NAME.get(status, status), msg))
        self.status = status


EXPORTS = ["gt_graph_plan_size", "gt_graph_create", "gt_graph_destroy", "gt_graph_outputs", "gt_graph_info",
           "gt_graph_validate", "gt_aggregate_ws_size", "gt_aggregate_fwd", "gt_aggregate_bwd",
           "gt_aggregate_static_capacity", "gt_aggregate_fwd_static", "gt_aggregate_combine_supported",
           "gt_aggregate_combine_fwd", "gt_combine_ws_size",
           "gt_combine", "gt_neighbor_apply_fwd", "gt_neighbor_apply_bwd", "gt_pull_fwd", "gt_pull_bwd", "gt_cost_get", "gt_cost_set", "gt_cost_get_dtype", "gt_cost_set_dtype", "gt_cost_benefits", "gt_layer_decide", "gt_layer_ws_size",
           "gt_layer_fwd", "gt_layer_bwd", "gt_calibrate_ws_size", "gt_calibrate", "gt_calibrate_dtype", "gt_trace_enable", "gt_trace_reset",
           "gt_trace_count", "gt_trace_get", "gt_trace_get_variant", "gt_sample_ws_size", "gt_sample_neighbors", "gt_reindex_ws_size",
           "gt_reindex", "gt_lookup", "gt_status_string",
           "gt_last_error", "gt_version"]

for _n in EXPORTS:
    getattr(lib, _n).restype = c_int
lib.gt_status_string.restype = ctypes.c_char_p
lib.gt_last_error.restype = ctypes.c_char_p
lib.gt_version.restype = ctypes.c_char_p
lib.gt_graph_plan_size.argtypes = [c_int64, c_int64, c_int64, c_int, POINTER(c_size_t)]
lib.gt_graph_create.argtypes = [POINTER(c_void_p), c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                c_size_t, c_void_p]
lib.gt_graph_destroy.argtypes = [c_void_p]
lib.gt_graph_outputs.argtypes = [c_void_p] + [POINTER(c_void_p)] * 5
lib.gt_graph_info.argtypes = [c_void_p] + [POINTER(c_int64)] * 7
lib.gt_graph_validate.argtypes = [c_void_p, POINTER(c_int64), c_void_p]
lib.gt_aggregate_ws_size.argtypes = [c_void_p, c_int64, POINTER(c_size_t)]
_AGG = [c_void_p, c_int, c_int, c_int64, c_void_p, c_int64, c_void_p, c_int64, c_void_p, c_size_t, c_void_p]
lib.gt_aggregate_fwd.argtypes = _AGG
lib.gt_aggregate_bwd.argtypes = _AGG
lib.gt_aggregate_static_capacity.argtypes = [POINTER(c_size_t)]
lib.gt_aggregate_fwd_static.argtypes = _AGG[:8] + [c_void_p]
lib.gt_aggregate_combine_supported.argtypes = [c_int, c_int64, c_int64, POINTER(c_int)]
lib.gt_aggregate_combine_fwd.argtypes = [c_void_p, c_int, c_int, c_int64, c_int64, c_void_p, c_int64, c_void_p, c_void_p, c_int,
                                         c_void_p, c_int64, c_void_p, c_size_t, c_void_p]
lib.gt_combine_ws_size.argtypes = [c_int, c_int, c_int, c_int64, c_int64, c_int64, POINTER(c_size_t)]
lib.gt_combine.argtypes = [c_int, c_int, c_int, c_int64, c_int64, c_int64, c_void_p, c_int64, c_void_p, c_int64,
                           c_void_p, c_int, c_void_p, c_int64, c_int, c_void_p, c_size_t, c_void_p]
lib.gt_neighbor_apply_fwd.argtypes = [c_void_p, c_int, c_int, c_int64, c_void_p, c_int64, c_void_p, c_int64, c_void_p,
                                      c_int64, c_void_p]
lib.gt_neighbor_apply_bwd.argtypes = [c_void_p, c_int, c_int, c_int64, c_void_p, c_int64, c_void_p, c_int64, c_void_p,
                                      c_int64, c_void_p, c_int64, c_void_p, c_int64, c_void_p, c_size_t, c_void_p]
lib.gt_pull_fwd.argtypes = [c_void_p, c_int, c_int, c_int, c_int64, c_void_p, c_int64, c_void_p, c_int64, c_void_p,
                            c_int64, c_void_p, c_size_t, c_void_p]
lib.gt_pull_bwd.argtypes = [c_void_p, c_int, c_int, c_int, c_int64, c_void_p, c_int64, c_void_p, c_int64, c_void_p,
                            c_int64, c_void_p, c_int64, c_void_p, c_int64, c_void_p, c_size_t, c_void_p]
lib.gt_cost_get.argtypes = [POINTER(gt_cost_coeffs)]
lib.gt_cost_set.argtypes = [POINTER(gt_cost_coeffs)]
lib.gt_cost_get_dtype.argtypes = [c_int, POINTER(gt_cost_coeffs)]
lib.gt_cost_set_dtype.argtypes = [c_int, POINTER(gt_cost_coeffs)]
lib.gt_cost_benefits.argtypes = [POINTER(gt_cost_coeffs), c_int64, c_int64, c_int64, c_int64, c_int64, c_int] + \
    [POINTER(c_double)] * 4
lib.gt_layer_decide.argtypes = [c_void_p, POINTER(gt_layer_desc), POINTER(c_int), POINTER(c_int)]
lib.gt_layer_ws_size.argtypes = [c_void_p, POINTER(gt_layer_desc), POINTER(c_size_t), POINTER(c_size_t)]
lib.gt_layer_fwd.argtypes = [c_void_p, POINTER(gt_layer_desc), c_int, c_void_p, c_int64, c_void_p, c_void_p, c_void_p,
                             c_void_p, c_int64, c_void_p, c_size_t, c_void_p, c_size_t, POINTER(c_int), c_void_p]
lib.gt_layer_bwd.argtypes = [c_void_p, POINTER(gt_layer_desc), c_int, c_int, c_void_p, c_int64, c_void_p, c_int64,
                             c_void_p, c_void_p, c_void_p, c_int64, c_void_p, c_size_t, c_void_p, c_size_t, c_void_p,
                             c_int64, c_void_p, c_void_p, c_void_p, POINTER(c_int), c_void_p]
lib.gt_trace_enable.argtypes = [c_int]
lib.gt_trace_reset.argtypes = []
lib.gt_trace_count.argtypes = [POINTER(c_int64)]
lib.gt_trace_get.argtypes = [c_int64, POINTER(c_int), POINTER(c_int64), POINTER(c_int64), POINTER(c_int64),
                             POINTER(c_double)]
lib.gt_trace_get_variant.argtypes = [c_int64] + [POINTER(c_int)] * 5
lib.gt_calibrate_ws_size.argtypes = [POINTER(c_size_t)]
lib.gt_calibrate.argtypes = [c_void_p, c_size_t, POINTER(gt_cost_coeffs), c_void_p]
lib.gt_calibrate_dtype.argtypes = [c_int, c_void_p, c_size_t, POINTER(gt_cost_coeffs), c_void_p]


lib.gt_sample_ws_size.argtypes = [c_int64, POINTER(c_size_t)]
lib.gt_sample_neighbors.argtypes = [c_void_p, c_void_p, c_int64, c_void_p, c_int64, c_int32, ctypes.c_uint32,
                                    ctypes.c_uint32, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
lib.gt_reindex_ws_size.argtypes = [c_int64, c_int64, POINTER(c_size_t)]
lib.gt_reindex.argtypes = [c_void_p, c_int64, c_void_p, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                           c_size_t, c_void_p]
lib.gt_lookup.argtypes = [c_int, c_void_p, c_int64, c_int64, c_void_p, c_int64, c_int64, c_void_p, c_int64, c_void_p]


def _check(status):
    if status != GT_OK:
        raise GtError(status, lib.gt_last_error().decode())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _dtype(t):
    if t.dtype == torch.float32:
        return GT_F32
    if t.dtype == torch.bfloat16:
        return GT_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _ws(nbytes, device):
    """Device scratch of at least nbytes (torch allocations are 256-byte aligned or better)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _rows2d(t):
    assert t.dim() == 2 and t.stride(1) == 1, "row-major 2-D tensor expected"
    return t.stride(0)


class Graph:
    """gt_graph handle plus the torch tensors it borrows (rowptr, colidx, weights, plan workspace)."""

    def __init__(self, rowptr, colidx, n_src, edge_weight=None):
        assert rowptr.dtype == torch.int32 and colidx.dtype == torch.int32 and rowptr.is_cuda and colidx.is_cuda
        self.rowptr, self.colidx, self.edge_weight = rowptr.contiguous(), colidx.contiguous(), edge_weight
        if edge_weight is not None:
            assert edge_weight.dtype == torch.float32 and edge_weight.is_cuda
            self.edge_weight = edge_weight.contiguous()
        self.n_dst, self.n_src, self.n_edges = rowptr.numel() - 1, int(n_src), colidx.numel()
        self.device = rowptr.device
        need = c_size_t()
        _check(lib.gt_graph_plan_size(self.n_dst, self.n_src, self.n_edges, int(edge_weight is not None), byref(need)))
        self.plan_bytes = need.value
        self.ws = _ws(need.value, self.device)
        h = c_void_p()
        _check(lib.gt_graph_create(byref(h), self.n_dst, self.n_src, self.n_edges, _ptr(self.rowptr), _ptr(self.colidx),
                                   _ptr(self.edge_weight), _ptr(self.ws), self.ws.numel(), _stream()))
        self.handle = h
        self._agg_ws = None

    def __del__(self):
        h = getattr(self, "handle", None)
        if h and lib is not None:       # `lib` is already gone at interpreter shutdown
            lib.gt_graph_destroy(h)
            self.handle = None

    def info(self):
        v = [c_int64() for _ in range(7)]
        _check(lib.gt_graph_info(self.handle, *[byref(x) for x in v]))
        keys = ("n_dst", "n_src", "n_edges", "fwd_items", "fwd_split_rows", "bwd_items", "bwd_split_rows")
        return {k: x.value for k, x in zip(keys, v)}

    def outputs(self):
        """Views (no copies) of in_deg, out_deg, rowptr_t, colidx_t, perm inside the plan workspace."""
        p = [c_void_p() for _ in range(5)]
        _check(lib.gt_graph_outputs(self.handle, *[byref(x) for x in p]))
        sizes = (self.n_dst, self.n_src, self.n_src + 1, self.n_edges, self.n_edges)
        base = self.ws.data_ptr()
        out = []
        for ptr, n in zip(p, sizes):
            off = (ptr.value or base) - base
            out.append(self.ws[off:off + 4 * n].view(torch.int32))
        return out

    def validate(self):
        n = c_int64()
        _check(lib.gt_graph_validate(self.handle, byref(n), _stream()))
        return n.value

    def aggregate_ws(self, F):
        need = c_size_t()
        _check(lib.gt_aggregate_ws_size(self.handle, int(F), byref(need)))
        if self._agg_ws is None or self._agg_ws.numel() < need.value:
            self._agg_ws = _ws(need.value, self.device)
        return self._agg_ws


def gt_aggregate_fwd(g: Graph, reduce, X, out=None, F=None):
    """Y[n_dst, F] = A X.  `out` may be a preallocated (possibly wider-strided) tensor."""
    F = X.shape[1] if F is None else F
    Y = torch.empty((g.n_dst, F), dtype=X.dtype, device=X.device) if out is None else out
    ws = g.aggregate_ws(F)
    _check(lib.gt_aggregate_fwd(g.handle, REDUCE[reduce], _dtype(X), F, _ptr(X), _rows2d(X), _ptr(Y), _rows2d(Y),
                                _ptr(ws), ws.numel(), _stream()))
    return Y


def gt_aggregate_fwd_static(g: Graph, reduce, X, out):
    """gt_aggregate_fwd without a workspace argument (the library's built-in scratch); `out` must be
    preallocated by the caller, this wrapper allocates nothing either."""
    _check(lib.gt_aggregate_fwd_static(g.handle, REDUCE[reduce], _dtype(X), X.shape[1], _ptr(X), _rows2d(X), _ptr(out),
                                       _rows2d(out), _stream()))
    return out


def gt_aggregate_combine_supported(dtype, in_dim, out_dim):
    yes = c_int()
    _check(lib.gt_aggregate_combine_supported(_dtype_code(dtype), int(in_dim), int(out_dim), byref(yes)))
    return bool(yes.value)


def gt_aggregate_combine_fwd(g: Graph, reduce, X, W, b=None, relu=False, out=None):
    """Y = act((A X) W + b) in one fused kernel (inference: A X is not kept)."""
    fi, fo = W.shape
    Y = torch.empty((g.n_dst, fo), dtype=X.dtype, device=X.device) if out is None else out
    ws = g.aggregate_ws(fi)
    assert W.is_contiguous()
    _check(lib.gt_aggregate_combine_fwd(g.handle, REDUCE[reduce], _dtype(X), fi, fo, _ptr(X), _rows2d(X), _ptr(W), _ptr(b),
                                        GT_ACT_RELU if relu else GT_ACT_NONE, _ptr(Y), _rows2d(Y), _ptr(ws), ws.numel(),
                                        _stream()))
    return Y


def gt_aggregate_bwd(g: Graph, reduce, dY, out=None, F=None):
    """dX[n_src, F] = A^T dY."""
    F = dY.shape[1] if F is None else F
    dX = torch.empty((g.n_src, F), dtype=dY.dtype, device=dY.device) if out is None else out
    ws = g.aggregate_ws(F)
    _check(lib.gt_aggregate_bwd(g.handle, REDUCE[reduce], _dtype(dY), F, _ptr(dY), _rows2d(dY), _ptr(dX), _rows2d(dX),
                                _ptr(ws), ws.numel(), _stream()))
    return dX


def gt_combine(A, B, bias=None, relu=False, transA=False, transB=False, out=None, out_dtype=None):
    """C = act(op(A) op(B) + bias)."""
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    K2, N = (B.shape[1], B.shape[0]) if transB else B.shape
    assert K == K2 and A.dtype == B.dtype
    cdt = out_dtype or (out.dtype if out is not None else A.dtype)
    C = torch.empty((M, N), dtype=cdt, device=A.device) if out is None else out
    need = c_size_t()
    _check(lib.gt_combine_ws_size(_dtype(A), int(transA), int(transB), M, N, K, byref(need)))
    ws = _ws(need.value, A.device)
    _check(lib.gt_combine(_dtype(A), int(transA), int(transB), M, N, K, _ptr(A), _rows2d(A), _ptr(B), _rows2d(B),
                          _ptr(bias), GT_ACT_RELU if relu else GT_ACT_NONE, _ptr(C), _rows2d(C), _dtype(C),
                          _ptr(ws), ws.numel(), _stream()))
    return C


EDGE_FN = {"dot": 0, "mul": 1}
WEIGHT_FN = {"scale": 0, "add": 1, "mul": 2}


def _ld(t):
    return t.stride(0) if t.dim() == 2 else 0


def gt_neighbor_apply_fwd(g: Graph, fn, Xs, Xd, out=None):
    """W_e = g(Xs[src], Xd[dst]): float32 [E] for 'dot', [E, F] of the input dtype for 'mul'."""
    F = Xs.shape[1]
    if out is None:
        out = torch.empty((g.n_edges,), dtype=torch.float32, device=Xs.device) if fn == "dot" else \
            torch.empty((g.n_edges, F), dtype=Xs.dtype, device=Xs.device)
    _check(lib.gt_neighbor_apply_fwd(g.handle, EDGE_FN[fn], _dtype(Xs), F, _ptr(Xs), _rows2d(Xs), _ptr(Xd), _rows2d(Xd),
                                     _ptr(out), _ld(out), _stream()))
    return out


def gt_neighbor_apply_bwd(g: Graph, fn, dW, Xs, Xd, out_dXs=None, out_dXd=None):
    F = Xs.shape[1]
    dXs = torch.empty((g.n_src, F), dtype=Xs.dtype, device=Xs.device) if out_dXs is None else out_dXs
    dXd = torch.empty((g.n_dst, F), dtype=Xs.dtype, device=Xs.device) if out_dXd is None else out_dXd
    ws = g.aggregate_ws(F)
    _check(lib.gt_neighbor_apply_bwd(g.handle, EDGE_FN[fn], _dtype(Xs), F, _ptr(dW), _ld(dW), _ptr(Xs), _rows2d(Xs),
                                     _ptr(Xd), _rows2d(Xd), _ptr(dXs), _rows2d(dXs), _ptr(dXd), _rows2d(dXd),
                                     _ptr(ws), ws.numel(), _stream()))
    return dXs, dXd


def gt_pull_fwd(g: Graph, reduce, h, Xs, W, out=None):
    F = Xs.shape[1]
    Y = torch.empty((g.n_dst, F), dtype=Xs.dtype, device=Xs.device) if out is None else out
    ws = g.aggregate_ws(F)
    _check(lib.gt_pull_fwd(g.handle, REDUCE[reduce], WEIGHT_FN[h], _dtype(Xs), F, _ptr(Xs), _rows2d(Xs), _ptr(W), _ld(W),
                           _ptr(Y), _rows2d(Y), _ptr(ws), ws.numel(), _stream()))
    return Y


def gt_pull_bwd(g: Graph, reduce, h, dY, Xs, W, out_dXs=None, out_dW=None):
    F = Xs.shape[1]
    dXs = torch.empty((g.n_src, F), dtype=Xs.dtype, device=Xs.device) if out_dXs is None else out_dXs
    dW = torch.empty_like(W) if out_dW is None else out_dW
    ws = g.aggregate_ws(F)
    _check(lib.gt_pull_bwd(g.handle, REDUCE[reduce], WEIGHT_FN[h], _dtype(Xs), F, _ptr(dY), _rows2d(dY), _ptr(Xs),
                           _rows2d(Xs), _ptr(W), _ld(W), _ptr(dXs), _rows2d(dXs), _ptr(dW), _ld(dW), _ptr(ws),
                           ws.numel(), _stream()))
    return dXs, dW


def make_desc(reduce, dtype, relu, in_dim, out_dim, has_root=False, need_dx=True, in_relu=False, dy_is_dz=False,
              pad_writable=False):
    d = gt_layer_desc()
    d.reduce = REDUCE[reduce]
    if dtype in (torch.bfloat16, "bf16"):
        d.dtype = GT_BF16
    elif dtype in (torch.float32, "f32"):
        d.dtype = GT_F32
    else:
        raise TypeError("dtype must be torch.float32/'f32' or torch.bfloat16/'bf16'")
    d.act = GT_ACT_RELU if relu else GT_ACT_NONE
    d.in_dim, d.out_dim = int(in_dim), int(out_dim)
    d.has_root, d.need_dx = int(has_root), int(need_dx)
    d.in_act, d.dy_is_dz = (GT_ACT_RELU if in_relu else GT_ACT_NONE), int(dy_is_dz)
    d.pad_writable = int(pad_writable)
    return d


def gt_layer_decide(g: Graph, desc):
    f, b = c_int(), c_int()
    _check(lib.gt_layer_decide(g.handle, byref(desc), byref(f), byref(b)))
    return ORDER_NAME[f.value], ORDER_NAME[b.value]


def gt_layer_ws_size(g: Graph, desc):
    s, t = c_size_t(), c_size_t()
    _check(lib.gt_layer_ws_size(g.handle, byref(desc), byref(s), byref(t)))
    return s.value, t.value


class LayerBuffers:
    """saved / scratch device buffers of one layer, allocated once and reused every step."""

    def __init__(self, g: Graph, desc):
        s, t = gt_layer_ws_size(g, desc)
        self.saved = _ws(s, g.device)
        self.scratch = _ws(t, g.device)


def gt_layer_fwd(g: Graph, desc, X, W, b, bufs: LayerBuffers, order="auto", W_root=None, out=None, inference=False):
    """`inference=True` passes no `saved` buffer: forward only, no backward call may follow."""
    tdt = torch.bfloat16 if desc.dtype == GT_BF16 else torch.float32
    Y = torch.empty((g.n_dst, desc.out_dim), dtype=tdt, device=X.device) if out is None else out
    used = c_int()
    saved = None if inference else bufs.saved
    _check(lib.gt_layer_fwd(g.handle, byref(desc), ORDER[order], _ptr(X), _rows2d(X), _ptr(W), _ptr(W_root), _ptr(b),
                            _ptr(Y), _rows2d(Y), _ptr(saved), 0 if inference else saved.numel(), _ptr(bufs.scratch),
                            bufs.scratch.numel(), byref(used), _stream()))
    return Y, ORDER_NAME[used.value]


def gt_layer_bwd(g: Graph, desc, fwd_used, dY, X, W, Y, bufs: LayerBuffers, order="auto", W_root=None,
                 want_db=True, out_dX=None):
    dev = X.device
    tdt = torch.bfloat16 if desc.dtype == GT_BF16 else torch.float32
    dX = None
    if desc.need_dx:
        dX = torch.empty((g.n_src, desc.in_dim), dtype=tdt, device=dev) if out_dX is None else out_dX
    dW = torch.empty((desc.in_dim, desc.out_dim), dtype=torch.float32, device=dev)
    dWr = torch.empty_like(dW) if desc.has_root else None
    db = torch.empty((desc.out_dim,), dtype=torch.float32, device=dev) if want_db else None
    used = c_int()
    _check(lib.gt_layer_bwd(g.handle, byref(desc), ORDER[fwd_used], ORDER[order], _ptr(dY), _rows2d(dY), _ptr(X),
                            _rows2d(X), _ptr(W), _ptr(W_root), _ptr(Y), _rows2d(Y) if Y is not None else 0,
                            _ptr(bufs.saved), bufs.saved.numel(), _ptr(bufs.scratch), bufs.scratch.numel(),
                            _ptr(dX), _rows2d(dX) if dX is not None else 0,
                            _ptr(dW), _ptr(dWr), _ptr(db), byref(used), _stream()))
    return dict(dX=dX, dW=dW, dW_root=dWr, db=db, used=ORDER_NAME[used.value])


def gt_cost_get():
    c = gt_cost_coeffs()
    _check(lib.gt_cost_get(byref(c)))
    return c


def gt_cost_set(c):
    _check(lib.gt_cost_set(byref(c)))


def _dtype_code(dtype):
    if dtype in (torch.bfloat16, "bf16"):
        return 1
    if dtype in (torch.float32, "f32"):
        return 0
    raise ValueError("dtype must be f32 or bf16")


def gt_cost_get_dtype(dtype):
    c = gt_cost_coeffs()
    _check(lib.gt_cost_get_dtype(_dtype_code(dtype), byref(c)))
    return c


def gt_cost_set_dtype(dtype, c):
    _check(lib.gt_cost_set_dtype(_dtype_code(dtype), byref(c)))


def gt_cost_benefits(c, n_src, n_dst, n_edge, n_feat, n_hid, first_layer=False):
    v = [c_double() for _ in range(4)]
    _check(lib.gt_cost_benefits(byref(c), n_src, n_dst, n_edge, n_feat, n_hid, int(first_layer), *[byref(x) for x in v]))
    return dict(aggr_fwd=v[0].value, aggr_bwd=v[1].value, comb_fwd=v[2].value, comb_bwd=v[3].value)


def gt_calibrate(device="cuda"):
    need = c_size_t()
    _check(lib.gt_calibrate_ws_size(byref(need)))
    ws = _ws(need.value, device)
    c = gt_cost_coeffs()
    _check(lib.gt_calibrate(_ptr(ws), ws.numel(), byref(c), _stream()))
    return c


def gt_calibrate_dtype(dtype, device="cuda"):
    need = c_size_t()
    _check(lib.gt_calibrate_ws_size(byref(need)))
    ws = _ws(need.value, device)
    c = gt_cost_coeffs()
    _check(lib.gt_calibrate_dtype(_dtype_code(dtype), _ptr(ws), ws.numel(), byref(c), _stream()))
    return c


def gt_trace_enable(on):
    _check(lib.gt_trace_enable(int(on)))


def gt_trace_reset():
    _check(lib.gt_trace_reset())


def gt_trace_records():
    """[(kind, width, rows, work, ms)] of every kernel launch recorded since the last reset."""
    n = c_int64()
    _check(lib.gt_trace_count(byref(n)))
    out = []
    for i in range(n.value):
        k, w, r, wk, ms = c_int(), c_int64(), c_int64(), c_int64(), c_double()
        _check(lib.gt_trace_get(i, byref(k), byref(w), byref(r), byref(wk), byref(ms)))
        out.append((k.value, w.value, r.value, wk.value, ms.value))
    return out


def gt_trace_variants():
    """[(V, G, NP, U, masked)] of every record: the aggregation kernel's template arguments (zeros for a combination)."""
    n = c_int64()
    _check(lib.gt_trace_count(byref(n)))
    out = []
    for i in range(n.value):
        v = [c_int() for _ in range(5)]
        _check(lib.gt_trace_get_variant(i, *[byref(x) for x in v]))
        out.append(tuple(x.value for x in v))
    return out


def gt_sample_neighbors(rowptr, colidx, dst, fanout, seed, stream_id):
    """S for one layer: (out_rowptr[n_dst + 1], picked global ids).  rowptr / colidx: int32 device
    tensors of the whole graph's in-edge CSR; dst: int32 device tensor of global ids.  Reads the
    number of picks back from the device (one stream synchronisation) to trim the result."""
    n_vertices, n_dst = rowptr.numel() - 1, dst.numel()
    need = c_size_t()
    _check(lib.gt_sample_ws_size(n_dst, byref(need)))
    ws = _ws(need.value, dst.device)
    out_rowptr = torch.empty(n_dst + 1, dtype=torch.int32, device=dst.device)
    out_nbr = torch.empty(max(n_dst * int(fanout), 1), dtype=torch.int32, device=dst.device)
    _check(lib.gt_sample_neighbors(_ptr(rowptr), _ptr(colidx), n_vertices, _ptr(dst), n_dst, int(fanout),
                                   int(seed) & 0xFFFFFFFF, int(stream_id) & 0xFFFFFFFF, _ptr(out_rowptr),
                                   _ptr(out_nbr), _ptr(ws), ws.numel(), _stream()))
    n_picked = int(out_rowptr[-1].item())
    return out_rowptr, out_nbr[:n_picked]


def gt_reindex(dst, picked, n_vertices):
    """R: (src_global[n_src], colidx_local[n_picked]); raises if dst holds a repeated id."""
    n_dst, n_picked = dst.numel(), picked.numel()
    need = c_size_t()
    _check(lib.gt_reindex_ws_size(n_dst, n_picked, byref(need)))
    ws = _ws(need.value, dst.device)
    src_global = torch.empty(max(n_dst + n_picked, 1), dtype=torch.int32, device=dst.device)
    colidx_local = torch.empty(max(n_picked, 1), dtype=torch.int32, device=dst.device)
    counts = torch.empty(2, dtype=torch.int32, device=dst.device)
    _check(lib.gt_reindex(_ptr(dst), n_dst, _ptr(picked), n_picked, int(n_vertices), _ptr(src_global),
                          _ptr(colidx_local), _ptr(counts), _ptr(ws), ws.numel(), _stream()))
    n_src, n_dst_distinct = counts.tolist()
    if n_dst_distinct != n_dst:
        raise ValueError("gt_reindex: destination ids must be distinct (%d distinct of %d)" % (n_dst_distinct, n_dst))
    return src_global[:n_src], colidx_local[:n_picked]


def gt_lookup(table, ids, out=None, F=None):
    """K: out[i, :F] = table[ids[i], :F]."""
    F = table.shape[1] if F is None else F
    if out is None:
        out = torch.empty((ids.numel(), F), dtype=table.dtype, device=table.device)
    _check(lib.gt_lookup(_dtype(table), _ptr(table), table.shape[0], _rows2d(table), _ptr(ids), ids.numel(), F,
                         _ptr(out), _rows2d(out), _stream()))
    return out


def gt_version():
    return lib.gt_version().decode()
