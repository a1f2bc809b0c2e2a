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
