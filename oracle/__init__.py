"""CPU oracle (TEST INFRASTRUCTURE): plain fp64 definitions of the aggregation / combination
path, used only by tests/, the smoke check and the benchmark's cpu_baseline leg.  It imports
nothing from the GPU package and the GPU package imports nothing from here.

Primitives are the C loops in gt_oracle.c (compiled on demand with gcc); the layer and model
functions below chain them in the order the paper gives:
  aggregation-first  sigma(W f(h(X)) + b)   and   combination-first  sigma(f(h(W X)) + b)
(GNN Kernel Orchestrator section), written here nodes x features:  act(A X W + b).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gt_oracle.c")
_LIB = os.path.join(_HERE, "libgt_oracle.so")
_lib = None

REDUCE = {"sum": 0, "mean": 1, "symnorm": 2}


def build(force: bool = False) -> str:
    """Compile gt_oracle.c with gcc (OpenMP over independent outputs)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.gto_aggregate_fwd.restype = ctypes.c_int
        _lib.gto_aggregate_bwd.restype = ctypes.c_int
        _lib.gto_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


def _feat(a):
    """Feature-like input: keep fp32 as is (read as fp32, widened per element), else fp64."""
    a = np.asarray(a)
    if a.dtype == np.float32:
        return np.ascontiguousarray(a), 1
    return np.ascontiguousarray(a, dtype=np.float64), 0


def num_threads() -> int:
    return int(lib().gto_num_threads())


def degrees(rowptr, colidx, n_src):
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n_dst = rowptr.size - 1
    din = np.empty(n_dst, dtype=np.int32)
    dout = np.empty(n_src, dtype=np.int32)
    lib().gto_degrees(ctypes.c_int64(n_dst), ctypes.c_int64(n_src), _p(rowptr), _p(colidx), _p(din), _p(dout))
    return din, dout


def transpose(rowptr, colidx, n_src):
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n_dst = rowptr.size - 1
    rpt = np.empty(n_src + 1, dtype=np.int32)
    cit = np.empty(colidx.size, dtype=np.int32)
    perm = np.empty(colidx.size, dtype=np.int32)
    lib().gto_transpose(ctypes.c_int64(n_dst), ctypes.c_int64(n_src), _p(rowptr), _p(colidx), _p(rpt), _p(cit), _p(perm))
    return rpt, cit, perm


def aggregate_fwd(rowptr, colidx, n_src, X, reduce="sum", ew=None, rows=None):
    """fp64 Y[n_rows, F]: aggregation of every destination (or of the listed `rows`)."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n_dst = rowptr.size - 1
    X, is32 = _feat(X)
    assert X.ndim == 2 and X.shape[0] == n_src
    F = X.shape[1]
    ew = None if ew is None else np.ascontiguousarray(ew, dtype=np.float32)
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = n_dst if rows is None else rows_a.size
    Y = np.empty((n_rows, F), dtype=np.float64)
    rc = lib().gto_aggregate_fwd(ctypes.c_int64(n_dst), ctypes.c_int64(n_src), _p(rowptr), _p(colidx), _p(ew),
                                 ctypes.c_int(REDUCE[reduce]), ctypes.c_int64(F), _p(X), ctypes.c_int(is32),
                                 ctypes.c_int64(X.strides[0] // X.itemsize), _p(Y), ctypes.c_int64(F),
                                 _p(rows_a), ctypes.c_int64(n_rows))
    if rc != 0:
        raise ValueError("unsupported aggregation request (symnorm needs a square graph)")
    return Y


def aggregate_bwd(rowptr, colidx, n_src, dY, reduce="sum", ew=None, src_rows=None):
    """fp64 dX[n_src (or len(src_rows)), F] = A^T dY by scattering over destination rows."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n_dst = rowptr.size - 1
    dY, is32 = _feat(dY)
    assert dY.ndim == 2 and dY.shape[0] == n_dst
    F = dY.shape[1]
    ew = None if ew is None else np.ascontiguousarray(ew, dtype=np.float32)
    sr = None if src_rows is None else np.ascontiguousarray(src_rows, dtype=np.int64)
    n_out = n_src if sr is None else sr.size
    dX = np.empty((n_out, F), dtype=np.float64)
    rc = lib().gto_aggregate_bwd(ctypes.c_int64(n_dst), ctypes.c_int64(n_src), _p(rowptr), _p(colidx), _p(ew),
                                 ctypes.c_int(REDUCE[reduce]), ctypes.c_int64(F), _p(dY), ctypes.c_int(is32),
                                 ctypes.c_int64(dY.strides[0] // dY.itemsize), _p(dX), ctypes.c_int64(F),
                                 _p(sr), ctypes.c_int64(n_out))
    if rc != 0:
        raise ValueError("unsupported aggregation request (symnorm needs a square graph)")
    return dX


def combine(A, B, bias=None, relu=False, transA=False, transB=False):
    """fp64 C = op(A) op(B) (+bias) (ReLU): plain triple loop."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    K2, N = (B.shape[1], B.shape[0]) if transB else B.shape
    assert K == K2, (A.shape, B.shape, transA, transB)
    bias = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    C = np.empty((M, N), dtype=np.float64)
    lib().gto_combine(ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), _p(A), ctypes.c_int64(A.shape[1]),
                      ctypes.c_int(int(transA)), _p(B), ctypes.c_int64(B.shape[1]), ctypes.c_int(int(transB)),
                      _p(bias), ctypes.c_int(int(relu)), _p(C), ctypes.c_int64(N))
    return C


def round_bf16(x):
    """Nearest bf16 value (ties to even) of every element, as fp64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    lib().gto_round_bf16(ctypes.c_int64(x.size), _p(x), _p(y))
    return y


EDGE_FN = {"dot": 0, "mul": 1}
WEIGHT_FN = {"scale": 0, "add": 1, "mul": 2}


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def neighbor_apply(rowptr, colidx, Xs, Xd, g="mul"):
    """Edge weights W = g(Xs[src], Xd[dst]) per edge: [E] for 'dot', [E, F] for 'mul'."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    Xs, Xd = _f64(Xs), _f64(Xd)
    n_dst, F = rowptr.size - 1, Xs.shape[1]
    assert Xd.shape == (n_dst, F)
    W = np.empty(colidx.size if g == "dot" else (colidx.size, F), dtype=np.float64)
    lib().gto_neighbor_apply(ctypes.c_int64(n_dst), _p(rowptr), _p(colidx), ctypes.c_int(EDGE_FN[g]), ctypes.c_int64(F),
                             _p(Xs), _p(Xd), _p(W))
    return W


def neighbor_apply_bwd(rowptr, colidx, dW, Xs, Xd, g="mul"):
    """(dXs, dXd) for upstream dW."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    Xs, Xd, dW = _f64(Xs), _f64(Xd), _f64(dW)
    n_dst, (n_src, F) = rowptr.size - 1, Xs.shape
    dXs, dXd = np.empty((n_src, F)), np.empty((n_dst, F))
    lib().gto_neighbor_apply_bwd(ctypes.c_int64(n_dst), ctypes.c_int64(n_src), _p(rowptr), _p(colidx),
                                 ctypes.c_int(EDGE_FN[g]), ctypes.c_int64(F), _p(dW), _p(Xs), _p(Xd), _p(dXs), _p(dXd))
    return dXs, dXd


def pull(rowptr, colidx, Xs, W, reduce="mean", h="add"):
    """Y[v] = f over in-edges of h(Xs[src], W_e); reduce in {'sum','mean'}."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    Xs, W = _f64(Xs), _f64(W)
    n_dst, F = rowptr.size - 1, Xs.shape[1]
    Y = np.empty((n_dst, F))
    lib().gto_pull(ctypes.c_int64(n_dst), _p(rowptr), _p(colidx), ctypes.c_int(int(reduce == "mean")),
                   ctypes.c_int(WEIGHT_FN[h]), ctypes.c_int64(F), _p(Xs), _p(W), _p(Y))
    return Y


def pull_bwd(rowptr, colidx, dY, Xs, W, reduce="mean", h="add"):
    """(dXs, dW) for upstream dY."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    Xs, W, dY = _f64(Xs), _f64(W), _f64(dY)
    n_dst, (n_src, F) = rowptr.size - 1, Xs.shape
    dXs, dW = np.empty((n_src, F)), np.empty_like(W)
    lib().gto_pull_bwd(ctypes.c_int64(n_dst), ctypes.c_int64(n_src), _p(rowptr), _p(colidx),
                       ctypes.c_int(int(reduce == "mean")), ctypes.c_int(WEIGHT_FN[h]), ctypes.c_int64(F), _p(dY),
                       _p(Xs), _p(W), _p(dXs), _p(dW))
    return dXs, dW


# ------------------------------------------------------------------------------------------
# Layers and models (fp64).  `blk` is a dict(rowptr, colidx, n_dst, n_src).
# ------------------------------------------------------------------------------------------

def layer_fwd(blk, reduce, X, W, b, relu, order="agg_first", W_root=None, ew=None):
    """One GNN layer, H' = act(A X W (+ X[:n_dst] W_root) + b), in the requested order.
    Returns dict(M=A X or None, Z=pre-activation, H=output)."""
    rp, ci, ns, nd = blk["rowptr"], blk["colidx"], blk["n_src"], blk["n_dst"]
    X = np.asarray(X, dtype=np.float64)
    M = None
    if order == "agg_first":
        M = aggregate_fwd(rp, ci, ns, X, reduce, ew)
        Z = combine(M, W)
    elif order == "comb_first":
        T = combine(X, W)
        Z = aggregate_fwd(rp, ci, ns, T, reduce, ew)
    else:
        raise ValueError(order)
    if W_root is not None:
        Z = Z + combine(X[:nd], W_root)
    Z = Z + np.asarray(b, dtype=np.float64)[None, :]
    H = np.maximum(Z, 0.0) if relu else Z
    return dict(M=M, Z=Z, H=H)


def layer_bwd(blk, reduce, X, W, Z, dH, relu, order="agg_first", W_root=None, ew=None, need_dx=True):
    """Gradients of one layer for upstream dH: dZ = dH * [Z > 0] (the activation's derivative,
    "Training for GNNs"; ReLU'(0) = 0, always decided from this function's own Z); db = column
    sums of dZ; dW = (A X)^T dZ; dX = A^T (dZ W^T) ["agg_first": the transposed aggregation runs
    at width F_in] or (A^T dZ) W^T ["comb_first": at width F_out]; the root term adds
    X[:n_dst]^T dZ and dZ W_root^T on the first n_dst rows."""
    rp, ci, ns, nd = blk["rowptr"], blk["colidx"], blk["n_src"], blk["n_dst"]
    X = np.asarray(X, dtype=np.float64)
    dZ = np.asarray(dH, dtype=np.float64)
    if relu:
        dZ = dZ * (np.asarray(Z) > 0.0)
    db = dZ.sum(axis=0)
    out = dict(dZ=dZ, db=db, dW_root=None, dX=None)
    if order == "agg_first":
        M = aggregate_fwd(rp, ci, ns, X, reduce, ew)
        out["dW"] = combine(M, dZ, transA=True)
        if need_dx:
            dM = combine(dZ, W, transB=True)
            out["dX"] = aggregate_bwd(rp, ci, ns, dM, reduce, ew)
    else:
        S = aggregate_bwd(rp, ci, ns, dZ, reduce, ew)
        out["dW"] = combine(X, S, transA=True)
        if need_dx:
            out["dX"] = combine(S, W, transB=True)
    if W_root is not None:
        out["dW_root"] = combine(X[:nd], dZ, transA=True)
        if need_dx:
            out["dX"][:nd] += combine(dZ, W_root, transB=True)
    return out


def model_fwd(cfg, order="agg_first", round_outputs=None):
    """All layers of a workload dict (gt_inputs.configs).  Hidden layers ReLU, last layer none.
    In bf16 workloads each layer output is rounded to bf16 where it crosses the library
    boundary (`round_outputs` defaults to cfg['dtype'] == 'bf16')."""
    rnd = (cfg["dtype"] == "bf16") if round_outputs is None else round_outputs
    H = np.asarray(cfg["X"], dtype=np.float64)
    states = []
    L = len(cfg["W"])
    orders = order if isinstance(order, (list, tuple)) else [order] * L
    for l in range(L):
        relu = l < L - 1
        st = layer_fwd(cfg["blocks"][l], cfg["reduce"], H, cfg["W"][l], cfg["b"][l], relu, orders[l],
                       cfg["W_root"][l], cfg.get("ew"))
        st["X"] = H
        if rnd:
            st["H"] = round_bf16(st["H"])
        states.append(st)
        H = st["H"]
    return states


def model_bwd(cfg, states, order="agg_first", round_outputs=None, stop=None):
    """Backward of the linear probe loss L = <G, Out>: dOut = G.  The first layer's dX is not
    needed (only parameter gradients are; cf. the cost-model paragraph on the first layer).
    `stop` (optional, one boolean array or None per layer, shape of that layer's output) marks
    output elements whose upstream gradient is taken as zero before the layer's backward: the
    gradient of the same model with those elements cut out of the loss.  It is an input of the
    computation like G; the ReLU decisions stay this function's own."""
    rnd = (cfg["dtype"] == "bf16") if round_outputs is None else round_outputs
    L = len(cfg["W"])
    orders = order if isinstance(order, (list, tuple)) else [order] * L
    dH = np.asarray(cfg["G"], dtype=np.float64)
    grads = [None] * L
    for l in reversed(range(L)):
        relu = l < L - 1
        st = states[l]
        if stop is not None and stop[l] is not None:
            dH = np.where(np.asarray(stop[l], dtype=bool), 0.0, dH)
        g = layer_bwd(cfg["blocks"][l], cfg["reduce"], st["X"], cfg["W"][l], st["Z"], dH, relu, orders[l],
                      cfg["W_root"][l], cfg.get("ew"), need_dx=(l > 0))
        if l > 0 and rnd:
            g["dX"] = round_bf16(g["dX"])
        grads[l] = g
        dH = g["dX"]
    return grads
