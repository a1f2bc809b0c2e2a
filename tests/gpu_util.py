"""Helpers for the GPU parity tests: upload seeded inputs, call the library through the binding,
compare with the oracle.  Each case announces itself (flushed) before touching the GPU."""
import sys

import numpy as np
import torch

from gt_inputs import tensors


def announce(*what):
    print("[gpu-case]", *what, flush=True)
    sys.stdout.flush()


def dev():
    return torch.device("cuda:0")


def up_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev())


def up_feat(a, dtype, ld=None):
    """fp32 numpy [n, F] -> device tensor of `dtype` ('f32'|'bf16') viewed [n, F] with row stride ld."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    n, F = a.shape
    ld = F if ld is None else ld
    if dtype == "bf16":
        bits = tensors.to_bf16_bits(a).view(np.int16)
        host = torch.from_numpy(bits).view(torch.bfloat16)
    else:
        host = torch.from_numpy(a)
    buf = torch.zeros((n, ld), dtype=host.dtype, device=dev())
    buf[:, :F] = host.to(dev())
    return buf[:, :F]


def empty_feat(n, F, dtype, ld=None, fill=float("nan")):
    ld = F if ld is None else ld
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    buf = torch.full((n, ld), fill, dtype=tdt, device=dev())
    return buf[:, :F]


def down(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def pad_to(F, dtype):
    v = 8 if dtype == "bf16" else 4
    return (F + v - 1) // v * v


def max_rel_err(got, ref):
    """max |got - ref| / max |ref| over the tensor (the tolerance metric of the benchmark spec)."""
    den = np.abs(ref).max()
    if den == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / den)


FP32_TOL = 1e-5
BF16_TOL = 2e-2


def tol_for(dtype):
    return BF16_TOL if dtype == "bf16" else FP32_TOL


def relu_rounding_sets(cfg, states):
    """Per layer, the set of outputs whose ReLU decision rounding may legitimately flip when the
    layer is given the ORACLE's input (states[l]["X"], uploaded in the working type), computed
    from oracle quantities only (no GPU value enters): elements with |Z| <= bound,
        bound = (u_acc + u_store + u_in) * S
        S = (|A| |X| |W|) (+ |X[:n_dst]| |W_root|) + |b|     the magnitudes of all terms of Z summed
        u_acc   = 16 * 2^-24   fp32 accumulation of the terms (worst case n * 2^-24, typically sqrt(n) * 2^-24)
        u_store = 2^-9 in bf16: the one intermediate (X W or A X) the layer stores in bf16 between its
                  two kernels, rounded to nearest; 0 in fp32
        u_in    = 2^-24 in fp32: the fp64 oracle activations are rounded once when uploaded; 0 in bf16
                  (the oracle's activations are bf16 values already)
    Returns (sets, bounds): a boolean array per hidden (ReLU) layer, None for the last layer, and
    the element-wise bounds of every layer."""
    import oracle
    bf = cfg["dtype"] == "bf16"
    u = 16 * 2.0 ** -24 + (2.0 ** -9 if bf else 2.0 ** -24)
    L = len(states)
    sets, bounds = [], []
    for l in range(L):
        blk = cfg["blocks"][l]
        rp, ci, ns, nd = blk["rowptr"], blk["colidx"], blk["n_src"], blk["n_dst"]
        absX = np.abs(np.asarray(states[l]["X"], dtype=np.float64))
        S = oracle.combine(oracle.aggregate_fwd(rp, ci, ns, absX, cfg["reduce"], cfg.get("ew")),
                           np.abs(np.asarray(cfg["W"][l], dtype=np.float64)))
        if cfg["W_root"][l] is not None:
            S = S + oracle.combine(absX[:nd], np.abs(np.asarray(cfg["W_root"][l], dtype=np.float64)))
        S = S + np.abs(np.asarray(cfg["b"][l], dtype=np.float64))[None, :]
        bounds.append(u * S)
        sets.append((np.abs(states[l]["Z"]) <= u * S) if l < L - 1 else None)
    return sets, bounds
