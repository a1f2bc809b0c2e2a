// Internal GEMM declarations shared by gt_combine.hip, gt_combine_x3.hip and the layer calls.
#pragma once
#include "gt_internal.h"

size_t gt_gemm_ws_bytes(int transA, int64_t M, int64_t N, int64_t K);

// C = act(rowscale .* (op(A) op(B)) + C_in + bias); C_in (same type and shape as C) may be null.
gt_status gt_gemm_run(const char *fn, gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, const void *B, int64_t ldb, const float *bias, const float *rowscale,
                      gt_act act, const void *Cin, int64_t ldcin, void *C, int64_t ldc, gt_dtype c_dtype, void *ws,
                      size_t ws_bytes, hipStream_t st);

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t gemm_bf16_t;

constexpr int GEMM_KT = 32;   // k-tile

__device__ inline uint32_t gemm_f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ inline float gemm_bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int VE = 4; static constexpr int PAD = 4; };
template <> struct Elem<gemm_bf16_t> { static constexpr int VE = 8; static constexpr int PAD = 8; };

struct GemmArgs {
    const void *A; int64_t lda;
    const void *B; int64_t ldb;
    void *C; int64_t ldc;          // output (type c_bf16 ? bf16 : f32), or fp32 partials when splits > 1
    const void *Cin; int64_t ldcin; // optional addend, same type as C
    const float *bias;
    const float *rowscale;         // optional per-row factor applied to the product before addend/bias
    int relu;
    int c_bf16;
    int64_t M, N, K;
    int64_t k_per_split;           // multiple of KT
    int vecA, vecB;                // 16-byte loads allowed
};


// Epilogue of a wavefront's TM x TN grid of 32x32 MFMA accumulators whose top-left element is
// (row0, col0).  Accumulator register r of lane (h, l32) holds row 8*(r/4) + 4*h + r%4, column l32.
template <int TM, int TN>
__device__ inline void gemm_epilogue(const GemmArgs &g, floatx16 (&acc)[TM][TN], int64_t row0, int64_t col0, int l32,
                                     int h) {
    const bool partial = gridDim.z > 1;
#pragma unroll
    for (int a = 0; a < TM; ++a) {
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int64_t col = col0 + b * 32 + l32;
            if (col >= g.N) continue;
            const float bia = (!partial && g.bias) ? g.bias[col] : 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = row0 + a * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (row >= g.M) continue;
                float v = acc[a][b][r];
                if (partial) {
                    static_cast<float *>(g.C)[((int64_t)blockIdx.z * g.M + row) * g.N + col] = v;
                    continue;
                }
                if (g.rowscale) v *= g.rowscale[row];
                if (g.Cin) {
                    v += g.c_bf16 ? gemm_bf16_to_f32(static_cast<const gemm_bf16_t *>(g.Cin)[row * g.ldcin + col])
                                  : static_cast<const float *>(g.Cin)[row * g.ldcin + col];
                }
                v += bia;
                if (g.relu) v = v > 0.0f ? v : 0.0f;
                if (g.c_bf16) static_cast<gemm_bf16_t *>(g.C)[row * g.ldc + col] = (gemm_bf16_t)gemm_f32_to_bf16(v);
                else static_cast<float *>(g.C)[row * g.ldc + col] = v;
            }
        }
    }
}

// fp32 GEMM through three-way bf16 splitting (gt_combine_x3.hip); 128 x 128 workgroup tiles.
gt_status gt_gemm_x3_launch(const GemmArgs &g, int transA, int transB, int splits, hipStream_t st);
