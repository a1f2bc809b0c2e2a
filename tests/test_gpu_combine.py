"""gt_combine against the oracle's triple loop.

Tolerance: fp32 MFMA accumulates K products in fp32; |gpu - ref| <= 1e-5 * (|A| |B| + |bias|)
element-wise (sequential-summation bound is K * 2^-24 per term, far looser in practice) and
max|gpu - ref| / max|ref| <= 1e-5.  bf16 inputs: products are exact in fp32, the fp32 sum is
rounded once to bf16 when C is bf16 (2^-8 relative, one step of slack against the oracle's
rounding); tensor-level <= 2e-2.
"""
import numpy as np
import pytest
import torch

import oracle
from gt_inputs import tensors
from gpu_util import announce, down, max_rel_err, tol_for, up_feat

pytestmark = pytest.mark.gpu

# (M, N, K): several tiles, ragged tails in every dimension, the skinny widths of the workloads
SHAPES = [(1, 1, 1), (300, 64, 64), (257, 16, 100), (515, 41, 128), (130, 47, 256), (260, 128, 602),
          (129, 256, 100), (70, 1024, 16), (200, 16, 1024), (33, 130, 37),
          # large enough for the fp32 path that runs on the bf16 matrix cores by three-way splitting
          (2100, 130, 1000), (1030, 602, 450),
          # few output tiles under a very wide feature row: the reduction is cut for every orientation
          (300, 64, 4353), (700, 2, 1100),
          # tall with a small weight matrix: the weight-stationary kernel (row blocks with a ragged end,
          # K and N off the chunk sizes, N beyond one column slice, K at both capacities)
          (9001, 41, 128), (8200, 128, 41), (8300, 256, 256), (10007, 47, 100), (8193, 1024, 16), (12000, 300, 37),
          (8192, 3, 5), (9000, 70, 250), (9000, 200, 100), (8500, 256, 128),
          # tall, wide fp32 rows onto at most 32 columns: the streaming form (16 and 32 weight rows kept, K a
          # multiple of the 128-column pass and off it, K off the 16-byte vector)
          (9000, 16, 1024), (8200, 29, 333), (20011, 7, 200), (8250, 32, 514),
          # the layers of a sampled batch: few rows, 64 x 64 tiles with a finely cut reduction; and a shape just
          # large enough to keep the big tiles
          (1024, 47, 256), (1100, 256, 47), (3000, 200, 300),
          # at most 64 output rows over a long reduction: 64 x 256 tiles of the split-bf16 kernel
          (48, 300, 20000),
          # at most 32 output rows: 32 x 256 tiles
          (16, 1024, 30000), (30, 260, 20000),
          # ... and at most 32 columns under many rows: 256 x 32 tiles
          (1024, 16, 30000), (300, 29, 20000),
          # weight-gradient shapes over a long reduction, split over workgroups (bf16: the transposing-load kernel)
          (256, 256, 20000), (100, 250, 12000), (200, 130, 11000)]


def _check(got, ref, absr, dtype, c_bf16, what):
    assert max_rel_err(got, ref) <= tol_for("bf16" if c_bf16 else dtype), (what, max_rel_err(got, ref))
    bound = 1e-5 * absr + 1e-30
    if c_bf16:
        bound = bound + 2.0 ** -7 * np.abs(ref)
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - ref).max()))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_combine_all_transposes(shape, dtype):
    from paper_2305_17469_amd import binding as B
    M, N, K = shape
    A = tensors.normal((M, K), seed=M + K)
    Bm = tensors.normal((K, N), seed=N + K + 1)
    bias = tensors.normal((N,), seed=5)
    if dtype == "bf16":
        A, Bm = tensors.bf16_values(A), tensors.bf16_values(Bm)
    ref_lin = oracle.combine(A, Bm)
    absr = oracle.combine(np.abs(A), np.abs(Bm))
    for tA in (False, True):
        for tB in (False, True):
            for padded in (False, True):
                announce("combine", dtype, shape, "tA", tA, "tB", tB, "padded", padded)
                a_host = A.T.copy() if tA else A
                b_host = Bm.T.copy() if tB else Bm
                v = 8 if dtype == "bf16" else 4
                lda = (a_host.shape[1] + v - 1) // v * v if padded else a_host.shape[1]
                ldb = (b_host.shape[1] + v - 1) // v * v if padded else b_host.shape[1]
                Ad, Bd = up_feat(a_host, dtype, lda), up_feat(b_host, dtype, ldb)
                C = B.gt_combine(Ad, Bd, transA=tA, transB=tB)
                ref = oracle.round_bf16(ref_lin) if dtype == "bf16" else ref_lin
                _check(down(C), ref, absr, dtype, dtype == "bf16", ("lin", tA, tB, padded))
                if not padded:
                    continue
                Cb = B.gt_combine(Ad, Bd, torch.from_numpy(bias).cuda(), relu=True, transA=tA, transB=tB)
                refb = oracle.combine(A, Bm, bias, relu=True)
                refb = oracle.round_bf16(refb) if dtype == "bf16" else refb
                _check(down(Cb), refb, absr + np.abs(bias)[None, :], dtype, dtype == "bf16", ("bias_relu", tA, tB))
                if dtype == "bf16":   # fp32 output from bf16 operands (the weight-gradient case)
                    C32 = B.gt_combine(Ad, Bd, transA=tA, transB=tB, out_dtype=torch.float32)
                    _check(down(C32), ref_lin, absr, dtype, False, ("f32out", tA, tB))


@pytest.mark.parametrize("shape", [(1500, 192, 1024), (9000, 96, 128), (8500, 100, 61)],
                         ids=["tiled", "weight_stationary", "weight_stationary_ragged"])
def test_split_bf16_path_keeps_fp32_accuracy_on_hard_inputs(shape):
    """Inputs with a wide dynamic range and no cancellation: the relative error of every output
    must stay at fp32 level (the three dropped cross products are below 2^-24 of each term).
    Both kernels that run fp32 data on the bf16 matrix cores: the tiled one and the tall,
    weight-stationary one."""
    from paper_2305_17469_amd import binding as B
    rng = np.random.default_rng(9)
    M, N, K = shape
    A = (np.abs(tensors.normal((M, K), seed=1)) * np.exp2(rng.integers(-20, 20, (M, 1)))).astype(np.float32)
    Bm = (np.abs(tensors.normal((K, N), seed=2)) * np.exp2(rng.integers(-20, 20, (1, N)))).astype(np.float32)
    announce("combine split-bf16 accuracy", (M, N, K))
    C = B.gt_combine(up_feat(A, "f32"), up_feat(Bm, "f32"))
    ref = oracle.combine(A, Bm)
    rel = np.abs(down(C) - ref) / ref          # all terms positive: ref is the sum of magnitudes
    assert rel.max() <= 1e-5, rel.max()   # fp32 accumulation of 1,024 positive terms: ~sqrt(K) * 2^-24


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_weight_gradient_shape_split_reduction(dtype):
    """op(A)^T op(B) with a long reduction (the node dimension): split over workgroups, summed in
    a fixed order; must be reproducible bit for bit."""
    from paper_2305_17469_amd import binding as B
    rows, fi, fo = (40_000, 100, 47) if dtype == "bf16" else (30_000, 130, 100)
    A = tensors.normal((rows, fi), seed=11)
    G = tensors.normal((rows, fo), seed=12)
    if dtype == "bf16":
        A, G = tensors.bf16_values(A), tensors.bf16_values(G)
    announce("combine weight gradient", dtype, rows, fi, fo)
    v = 8 if dtype == "bf16" else 4
    Ad = up_feat(A, dtype, (fi + v - 1) // v * v)
    Gd = up_feat(G, dtype, (fo + v - 1) // v * v)
    need = B.c_size_t()
    assert B.lib.gt_combine_ws_size(0, 1, 0, fi, fo, rows, B.byref(need)) == 0 and need.value > 0
    C1 = B.gt_combine(Ad, Gd, transA=True, out_dtype=torch.float32)
    C2 = B.gt_combine(Ad, Gd, transA=True, out_dtype=torch.float32)
    assert torch.equal(C1, C2)
    ref = oracle.combine(A, G, transA=True)
    absr = oracle.combine(np.abs(A), np.abs(G), transA=True)
    _check(down(C1), ref, absr, dtype, False, "dW")
    st = B.lib.gt_combine(0, 1, 0, fi, fo, rows, Ad.data_ptr(), Ad.stride(0), Gd.data_ptr(), Gd.stride(0), None, 0,
                          C1.data_ptr(), fo, 0, None, 0, None) if dtype == "f32" else 3
    assert st == 3   # the split reduction needs its workspace


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_combine_random_shapes_around_the_kernel_boundaries(seed):
    """Seeded random (M, N, K, transposes, padding, epilogue) drawn from the sizes at which the library
    changes kernel or tile: row lengths around the slice and capacity limits of the weight-stationary
    and streaming forms, widths around the 32 / 64 / 128 / 256-column tiles, tall outputs, long
    reductions (split over workgroups)."""
    from paper_2305_17469_amd import binding as B
    rng = np.random.default_rng(seed)
    Ks = [1, 5, 16, 17, 32, 33, 47, 64, 65, 100, 128, 129, 200, 256, 257, 333, 512, 514, 602, 1000, 1024, 1025]
    Ns = [1, 3, 7, 16, 17, 29, 32, 33, 41, 47, 64, 65, 100, 128, 129, 200, 256, 257, 300, 512, 1024]
    for it in range(60):
        kind = it % 3
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        if kind == 0:      # tall forward shapes
            M, N, K, tA = int(rng.choice([8192, 8193, 9000, 12345, 20011])), int(rng.choice(Ns)), int(rng.choice(Ks)), False
        elif kind == 1:    # weight-gradient shapes
            M, N, K, tA = int(rng.choice(Ns)), int(rng.choice(Ns)), int(rng.choice([8192, 9001, 20000, 30011])), True
        else:
            M, N, K, tA = int(rng.integers(1, 700)), int(rng.choice(Ns)), int(rng.choice(Ks)), bool(rng.integers(0, 2))
        tB, padded, extras = bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        if M * N * K > 2e9:
            continue
        A = tensors.normal((M, K), seed=1000 * seed + it * 3)
        Bm = tensors.normal((K, N), seed=1000 * seed + it * 3 + 1)
        bias = tensors.normal((N,), seed=1000 * seed + it * 3 + 2)
        if dtype == "bf16":
            A, Bm = tensors.bf16_values(A), tensors.bf16_values(Bm)
        a_host = A.T.copy() if tA else A
        b_host = Bm.T.copy() if tB else Bm
        v = 8 if dtype == "bf16" else 4
        lda = (a_host.shape[1] + v - 1) // v * v if padded else a_host.shape[1]
        ldb = (b_host.shape[1] + v - 1) // v * v if padded else b_host.shape[1]
        announce("combine random", seed, it, dtype, (M, N, K), "tA", tA, "tB", tB, "padded", padded, "extras", extras)
        Ad, Bd = up_feat(a_host, dtype, lda), up_feat(b_host, dtype, ldb)
        absr = oracle.combine(np.abs(A), np.abs(Bm))
        if extras:
            C = B.gt_combine(Ad, Bd, torch.from_numpy(bias).cuda(), relu=True, transA=tA, transB=tB)
            ref = oracle.combine(A, Bm, bias, relu=True)
            absr = absr + np.abs(bias)[None, :]
        else:
            C = B.gt_combine(Ad, Bd, transA=tA, transB=tB)
            ref = oracle.combine(A, Bm)
        ref = oracle.round_bf16(ref) if dtype == "bf16" else ref
        got = down(C)
        bound = 1e-5 * absr + 1e-30 + (2.0 ** -7 * np.abs(ref) if dtype == "bf16" else 0.0)
        bad = ~(np.abs(got - ref) <= bound)
        assert not bad.any(), ((M, N, K), dtype, tA, tB, padded, extras, int(bad.sum()), float(np.nanmax(np.abs(got - ref))))
