"""Seeded dense inputs: feature tables, Glorot weights, upstream gradients, bf16 payloads.

Only data generation and storage-format conversion; no aggregation / combination arithmetic.
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def normal(shape, seed: int, stream: int = 10) -> np.ndarray:
    """fp32 N(0,1) array."""
    return _rng(seed, stream).standard_normal(size=shape, dtype=np.float32)


def glorot(f_in: int, f_out: int, seed: int, stream: int = 20) -> np.ndarray:
    """Glorot-uniform weight [f_in, f_out], U(+-sqrt(6/(f_in+f_out))), fp32."""
    lim = np.sqrt(6.0 / (f_in + f_out))
    return _rng(seed, stream).uniform(-lim, lim, size=(f_in, f_out)).astype(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 payload (uint16), round-to-nearest-even; storage conversion for inputs."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 payload (uint16) -> the fp32 array holding exactly those values."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_values(x: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is representable in bf16 (inputs of the bf16 configs)."""
    return from_bf16_bits(to_bf16_bits(x))
