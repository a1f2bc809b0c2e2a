// Weight-stationary combination for tall, skinny products: C[M, N] = act(A[M, K] op(B) + ...)
// with M in the millions and K, N at most a few hundred (every layer of a GNN on a large graph).
//
// Such a product is bound by reading A and writing C once; the tiled kernel misses that bound
// because every 128-row workgroup fetches the weight tile again for every k-tile (half of all the
// bytes it moves through the L2) and its k-loop is a chain of workgroup barriers with one exposed
// load latency each.  Here the weight matrix is loaded into LDS ONCE per workgroup ([n][k],
// k contiguous, zero padded) and stays there; the workgroups are persistent and every wavefront
// works alone on 32-row blocks of A, with no workgroup barrier after the weights are in place:
//   * A is read in slices of 32 rows x 128 bytes, eight lanes per row, so every load instruction
//     covers whole 128-byte lines (loading MFMA fragments directly would touch 32 rows x 32 bytes
//     per instruction and fetch every line four times);
//   * a slice goes registers -> the wavefront's private LDS stage -> MFMA fragments; as soon as a
//     slice has left its registers, the same registers receive the loads of the NEXT block's
//     slice, so a whole block of loads is always in flight per wavefront;
//   * the MFMA operands are swapped (weights as the first operand, rows of A as the second), so
//     every lane ends up with four CONSECUTIVE columns of one output row per register group and
//     stores them directly, with no transposing pass through LDS.
//
// Operand mapping.  bf16 (v_mfma_f32_32x32x16_bf16): lane (l32, h) supplies row l32 and
// k = 16 s + 8 h .. + 7 of step s.  fp32 (v_mfma_f32_32x32x2f32) wants one k per lane half and
// step; a lane instead reads four consecutive k (16 bytes) and feeds them to four consecutive
// steps, i.e. step 4 c + j multiplies k = 8 c + 4 h + j; the weight fragment is read from LDS
// with the same assignment, so every k is used exactly once.
#include "gt_internal.h"
#include "gt_combine.h"

namespace {

typedef gemm_bf16_t bf16_t;

template <typename T> struct WsGeom;
// CK: k per MFMA chunk (both lane halves), HK: k per lane (16 bytes), SK: k per slice (128 bytes)
template <> struct WsGeom<float>  { static constexpr int CK = 8,  HK = 4, SK = 32, PAD = 4; };
template <> struct WsGeom<bf16_t> { static constexpr int CK = 16, HK = 8, SK = 64, PAD = 8; };

// zero the elements of a 16-byte chunk from element nv on
template <typename T>
__device__ inline uint4 ws_mask(uint4 v, int nv) {
    if constexpr (sizeof(T) == 4) {
        v.x = nv > 0 ? v.x : 0u; v.y = nv > 1 ? v.y : 0u; v.z = nv > 2 ? v.z : 0u; v.w = nv > 3 ? v.w : 0u;
    } else {
        v.x &= nv >= 2 ? 0xffffffffu : (nv == 1 ? 0x0000ffffu : 0u);
        v.y &= nv >= 4 ? 0xffffffffu : (nv == 3 ? 0x0000ffffu : 0u);
        v.z &= nv >= 6 ? 0xffffffffu : (nv == 5 ? 0x0000ffffu : 0u);
        v.w &= nv >= 8 ? 0xffffffffu : (nv == 7 ? 0x0000ffffu : 0u);
    }
    return v;
}

// two bf16 values of v, each kept where the bf16 value at the same place of m is > 0, else zeroed
__device__ inline uint32_t ws_mask_pair(uint32_t v, uint32_t m) {
    const uint32_t lo = __uint_as_float(m << 16) > 0.0f ? 0x0000ffffu : 0u;
    const uint32_t hi = __uint_as_float(m & 0xffff0000u) > 0.0f ? 0xffff0000u : 0u;
    return v & (lo | hi);
}

// One slice (32 rows x 128 bytes) of block rb: lane -> row lane/8 + 8 j (j = 0..3), chunk lane%8.
// Rows past M read the last row (never stored); chunks at or past K read the row's first chunk
// (always valid) and are zeroed when staged.
template <typename T>
__device__ inline void ws_load_slice(uint4 (&r)[4], const T *A, int64_t lda, int64_t rb, int s, int64_t M, int64_t K,
                                     int lane) {
    constexpr int HK = WsGeom<T>::HK, SK = WsGeom<T>::SK;
    const int64_t k = (int64_t)s * SK + (lane & 7) * HK;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int64_t row = rb * 32 + (lane >> 3) + 8 * j;
        if (row >= M) row = M - 1;
        r[j] = *reinterpret_cast<const uint4 *>(A + row * lda + (k < K ? k : 0));
    }
}

// The products are formed as (weights)^T x (rows)^T, so accumulator register r of lane (h, l32)
// holds output row l32 of the block and column 8 (r / 4) + 4 h + r % 4 of the 32-column group:
// four consecutive columns per register quadruple, stored straight from registers.  The bias is
// already in the accumulators (they start from it); only the activation is left to apply.
// CB: C is bf16;  EX: bias and / or ReLU present.
// FAST: every column group of the slice lies inside N and can be stored as one vector, so the
// epilogue is straight-line code.
template <bool CB, bool EX, bool FAST, int NB>
__device__ inline void ws_epilogue(const GemmArgs &g, floatx16 (&acc)[NB], int64_t row, int64_t n0, int h, bool vec) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t col = n0 + b * 32 + 8 * q + 4 * h;
            if (!FAST && col >= g.N) continue;
            const bool whole = FAST || (vec && col + 4 <= g.N);
            float v[4] = {acc[b][4 * q], acc[b][4 * q + 1], acc[b][4 * q + 2], acc[b][4 * q + 3]};
            if (EX) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = (g.relu && !(v[i] > 0.0f)) ? 0.0f : v[i];
                if (g.mask) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (!FAST && col + i >= g.N) continue;
                        const float mk = CB ? gemm_bf16_to_f32(static_cast<const gemm_bf16_t *>(g.mask)[row * g.ldmask + col + i])
                                            : static_cast<const float *>(g.mask)[row * g.ldmask + col + i];
                        v[i] = mk > 0.0f ? v[i] : 0.0f;
                    }
                }
            }
            if (CB) {
                gemm_bf16_t *p = static_cast<gemm_bf16_t *>(g.C) + row * g.ldc + col;
                if (whole) {
                    *reinterpret_cast<uint2 *>(p) = make_uint2(gt_pack_bf16(v[0], v[1]),
                                                               gt_pack_bf16(v[2], v[3]));
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (col + i < g.N) p[i] = (gemm_bf16_t)gemm_f32_to_bf16(v[i]);
                }
            } else {
                float *p = static_cast<float *>(g.C) + row * g.ldc + col;
                if (whole) {
                    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (col + i < g.N) p[i] = v[i];
                }
            }
        }
    }
}

// fp32 output, whole column groups, rows of C 16-byte aligned: each 32-column group of the block
// passes through the wavefront's private stage (free at this point: every fragment of the block has
// been read) and is written row-major, eight lanes per row, so a store instruction covers whole
// 128-byte lines of 8 rows instead of 32-byte pieces of 32 rows.  Rows past M hold the last row's
// values (their loads were clamped to it) and are written onto the last row.
// RAGGED: N need not fill the column slice (see ws_epilogue_rows_bf16).
template <bool EX, bool MK, bool RAGGED, int NB>
__device__ inline void ws_epilogue_rows_f32(const GemmArgs &g, floatx16 (&acc)[NB], int64_t row0, int64_t n0, int lane,
                                            float *stage) {
    constexpr int SSTR = 36;   // 32 columns + 4: the stage holds 32 x 36 floats
    const int l32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        __asm__ volatile("" ::: "memory");   // LDS operations of a wavefront run in program order; keep that order
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float4 v = make_float4(acc[b][4 * q], acc[b][4 * q + 1], acc[b][4 * q + 2], acc[b][4 * q + 3]);
            if (EX) {
                v.x = (g.relu && !(v.x > 0.0f)) ? 0.0f : v.x; v.y = (g.relu && !(v.y > 0.0f)) ? 0.0f : v.y;
                v.z = (g.relu && !(v.z > 0.0f)) ? 0.0f : v.z; v.w = (g.relu && !(v.w > 0.0f)) ? 0.0f : v.w;
            }
            *reinterpret_cast<float4 *>(stage + l32 * SSTR + 8 * q + 4 * h) = v;
        }
        __asm__ volatile("" ::: "memory");
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int rr = it * 8 + (lane >> 3), c4 = (lane & 7) * 4;
            float4 v = *reinterpret_cast<const float4 *>(stage + rr * SSTR + c4);
            int64_t row = row0 + rr;
            if (row >= g.M) row = g.M - 1;
            const int64_t c0 = n0 + b * 32 + c4;
            if constexpr (MK) {   // the host passes a mask here only when its rows allow 16-byte loads
                const float4 mk = *reinterpret_cast<const float4 *>(static_cast<const float *>(g.mask) + row * g.ldmask +
                                                                    ((!RAGGED || c0 < g.N) ? c0 : 0));
                v.x = mk.x > 0.0f ? v.x : 0.0f; v.y = mk.y > 0.0f ? v.y : 0.0f;
                v.z = mk.z > 0.0f ? v.z : 0.0f; v.w = mk.w > 0.0f ? v.w : 0.0f;
            }
            float *dst = static_cast<float *>(g.C) + row * g.ldc + c0;
            if constexpr (!RAGGED) {
                *reinterpret_cast<float4 *>(dst) = v;
            } else {
                const int64_t left = g.N - c0;
                if (left >= 4 || (g.pad_c && left > 0 && c0 + 4 <= g.ldc)) {   // (columns past N hold zeros)
                    *reinterpret_cast<float4 *>(dst) = v;
                } else if (left > 0) {
                    dst[0] = v.x;
                    if (left > 1) dst[1] = v.y;
                    if (left > 2) dst[2] = v.z;
                }
            }
        }
    }
    __asm__ volatile("" ::: "memory");
}

// The same for a bf16 C whose rows are 16-byte aligned: two 32-column groups at a time are rounded
// to bf16, staged as 32 rows x 64 columns (128 bytes + 16 of padding per row) and written eight lanes
// per row, 16 bytes per lane: whole 128-byte lines again.
// LATE: the mask vectors are requested when they are needed instead of before the round is staged (the
// instances with two wavefronts per SIMD have no 16 registers to hold them meanwhile).
// RAGGED: N need not fill the column slice: a lane whose eight columns straddle N stores the ones inside
// one by one, a lane past N stores nothing (config 3's 256 -> 47: storing from registers wrote every
// 96-byte row as twelve 8-byte pieces spread over six instructions).
template <bool EX, bool MK, bool LATE, bool RAGGED, int NB>
__device__ inline void ws_epilogue_rows_bf16(const GemmArgs &g, floatx16 (&acc)[NB], int64_t row0, int64_t n0, int lane,
                                             uint32_t *stage) {
    static_assert(NB % 2 == 0, "column groups are staged in pairs");
    constexpr int SSTR = 36;   // dwords per staged row: 64 bf16 + 16 bytes
    const int l32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int bp = 0; bp < NB / 2; ++bp) {
        uint4 mkv[4];
        if constexpr (MK && !LATE) {   // requested before the staging below, so that the round trip overlaps it
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                int64_t row = row0 + it * 8 + (lane >> 3);
                if (row >= g.M) row = g.M - 1;
                const int64_t cm = n0 + bp * 64 + (lane & 7) * 8;
                mkv[it] = *reinterpret_cast<const uint4 *>(static_cast<const gemm_bf16_t *>(g.mask) + row * g.ldmask +
                                                          ((!RAGGED || cm < g.N) ? cm : 0));
            }
        }
        __asm__ volatile("" ::: "memory");
#pragma unroll
        for (int bb = 0; bb < 2; ++bb) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v[4] = {acc[2 * bp + bb][4 * q], acc[2 * bp + bb][4 * q + 1], acc[2 * bp + bb][4 * q + 2],
                              acc[2 * bp + bb][4 * q + 3]};
                if (EX) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (g.relu && !(v[i] > 0.0f)) ? 0.0f : v[i];
                }
                *reinterpret_cast<uint2 *>(stage + l32 * SSTR + bb * 16 + 4 * q + 2 * h) =
                    make_uint2(gt_pack_bf16(v[0], v[1]),
                               gt_pack_bf16(v[2], v[3]));
            }
        }
        __asm__ volatile("" ::: "memory");
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int rr = it * 8 + (lane >> 3);
            uint4 v = *reinterpret_cast<const uint4 *>(stage + rr * SSTR + (lane & 7) * 4);
            int64_t row = row0 + rr;
            if (row >= g.M) row = g.M - 1;
            const int64_t c0 = n0 + bp * 64 + (lane & 7) * 8;
            if constexpr (MK) {
                const uint4 mk = LATE ? *reinterpret_cast<const uint4 *>(static_cast<const gemm_bf16_t *>(g.mask) + row * g.ldmask +
                                                                         ((!RAGGED || c0 < g.N) ? c0 : 0))
                                      : mkv[it];
                v.x = ws_mask_pair(v.x, mk.x); v.y = ws_mask_pair(v.y, mk.y);
                v.z = ws_mask_pair(v.z, mk.z); v.w = ws_mask_pair(v.w, mk.w);
            }
            gemm_bf16_t *dst = static_cast<gemm_bf16_t *>(g.C) + row * g.ldc + c0;
            if constexpr (!RAGGED) {
                *reinterpret_cast<uint4 *>(dst) = v;
            } else {
                const int64_t left = g.N - c0;
                if (left >= 8 || (g.pad_c && left > 0 && c0 + 8 <= g.ldc)) {   // (columns past N hold zeros)
                    *reinterpret_cast<uint4 *>(dst) = v;
                } else if (left > 0) {
                    // 1..7 columns as an 8-, a 4- and a 2-byte piece
                    if (left & 4) *reinterpret_cast<uint2 *>(dst) = make_uint2(v.x, v.y);
                    const uint32_t w2 = (left & 4) ? v.z : v.x, w3 = (left & 4) ? v.w : v.y;
                    gemm_bf16_t *d2 = dst + (left & 4);
                    if (left & 2) *reinterpret_cast<uint32_t *>(d2) = w2;
                    if (left & 1) d2[left & 2] = (gemm_bf16_t)(((left & 2) ? w3 : w2) & 0xffffu);
                }
            }
        }
    }
    __asm__ volatile("" ::: "memory");
}

// LDS bytes of an instance with NW wavefronts: the weight slice, one private A stage per wavefront, the
// bias of the column slice
template <typename T, int NB, int NS, int NW>
constexpr size_t ws_lds_bytes() {
    return (size_t)NB * 32 * (NS * WsGeom<T>::SK + WsGeom<T>::PAD) * sizeof(T) + (size_t)NW * GEMM_STAGE_FLOATS(1) * 4 +
           (size_t)NB * 32 * 4;
}
// Wavefronts per workgroup.  The kernel lives on memory operations in flight, so a CU should hold eight
// wavefronts: two workgroups of four where two weight slices fit its LDS (80 KB each), else one
// workgroup of eight, or of six where the weight slice leaves room for no more stages (256 x 256 bf16:
// 132 KB of weights; measured on MI355X over 2^21 rows, 4 -> 6 wavefronts 0.61 -> 0.50 ms, and 100 -> 256
// with 4 -> 8 wavefronts 0.49 -> 0.31 ms).
template <typename T, int NB, int NS>
constexpr int ws_waves() {
    if (ws_lds_bytes<T, NB, NS, 4>() <= 80 * 1024) return 4;
    if (ws_lds_bytes<T, NB, NS, 8>() <= 160 * 1024) return 8;
    if (ws_lds_bytes<T, NB, NS, 6>() <= 160 * 1024) return 6;
    return 4;
}
template <typename T, int NB, int NS>
constexpr int ws_per_cu() { return ws_lds_bytes<T, NB, NS, 4>() <= 80 * 1024 ? 2 : 1; }

// EX: bias and / or ReLU present.  C has the element type of A; products with a row scale or an
// addend stay on the tiled kernel.
// The slice loop is free of branches for every shape (loads past the end re-read the last block,
// slices and chunks at or past K re-read the row's first chunk and are staged as zeros, masks are
// always applied): with control flow in it the compiler waits for ALL outstanding memory
// operations before it touches a prefetched slice.
// FAST: N is a multiple of the slice width and C allows vector stores; then the epilogue is
// straight-line code as well (rows past M store the last row's values onto the last row), and the
// wait at the head of the row loop does not include the previous block's stores.
// HALF (one-slice instances): K is at most half a slice, the MFMA steps of the empty half are left out
// (2^20 x 16 -> 1024 fp32 spent 0.44 of its 1.0 ms multiplying zeros).
template <typename T, int NB, int NS, bool EX, bool FAST, bool MK, bool HALF, bool RG>
__global__ void __launch_bounds__((ws_waves<T, NB, NS>() * 64), (ws_per_cu<T, NB, NS>())) k_gemm_ws(const GemmArgs g, const int transB) {
    constexpr int NW = ws_waves<T, NB, NS>(), NT = NW * 64;
    static_assert(!HALF || NS == 1, "HALF is a form of the one-slice instances");
    constexpr int CK = WsGeom<T>::CK, HK = WsGeom<T>::HK, SK = WsGeom<T>::SK;
    constexpr int KP = NS * SK;                 // K capacity of this instance
    constexpr int WSTR = KP + WsGeom<T>::PAD;   // LDS row stride: 16 bytes past a multiple of 128
    constexpr int ASTR = SK + WsGeom<T>::PAD;   // stage row stride (144 bytes)
    constexpr int BN = NB * 32;
    static_assert(32 * ASTR * sizeof(T) <= GEMM_STAGE_FLOATS(1) * 4, "a slice must fit the wavefront's stage");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T *Ws = reinterpret_cast<T *>(smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    // this wavefront's private stage for A slices
    T *As = reinterpret_cast<T *>(smem + (size_t)BN * WSTR * sizeof(T) + (size_t)wave * GEMM_STAGE_FLOATS(1) * 4);
    float *bias_lds = reinterpret_cast<float *>(smem + (size_t)BN * WSTR * sizeof(T) + NW * (size_t)GEMM_STAGE_FLOATS(1) * 4);
    const T *A = static_cast<const T *>(g.A);
    const T *B = static_cast<const T *>(g.B);
    const int64_t n0 = (int64_t)blockIdx.y * BN;
    for (int n = threadIdx.x; n < BN; n += NT) bias_lds[n] = (g.bias && n0 + n < g.N) ? g.bias[n0 + n] : 0.0f;

    // the weight slice, once: Ws[n][k] = op(B)(k, n0 + n), zero outside (K, N).  16-byte loads,
    // several in flight per thread (the matrix is small, but one dependent load per element would
    // cost a load latency each).
    constexpr int VE = 16 / (int)sizeof(T);
    if (g.vecB && transB) {          // B[n][k]: vectors along k go straight to the LDS row
        constexpr int VPR = KP / VE, TOTAL = BN * VPR;
        for (int base = threadIdx.x; base < TOTAL; base += NT * 8) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {   // eight loads in flight, then eight stores
                const int idx = base + u * NT;
                const int n = idx / VPR, k = (idx % VPR) * VE;
                const bool ok = idx < TOTAL && n0 + n < g.N && k < g.K;
                v[u] = *reinterpret_cast<const uint4 *>(B + (ok ? (n0 + n) * g.ldb + k : 0));
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NT;
                const int n = idx / VPR, k = (idx % VPR) * VE;
                const bool ok = n0 + n < g.N && k < g.K;
                const int64_t left = g.K - k;
                if (idx < TOTAL)
                    *reinterpret_cast<uint4 *>(Ws + n * WSTR + k) = ws_mask<T>(v[u], ok ? (left < VE ? (int)left : VE) : 0);
            }
        }
    } else if (g.vecB) {             // B[k][n]: a vector holds VE columns of one k, scattered to VE rows
        constexpr int VPR = BN / VE, TOTAL = KP * VPR;
        for (int base = threadIdx.x; base < TOTAL; base += NT * 8) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NT;
                const int k = idx / VPR, n = (idx % VPR) * VE;
                const bool ok = idx < TOTAL && n0 + n < g.N && k < g.K;
                v[u] = *reinterpret_cast<const uint4 *>(B + (ok ? (int64_t)k * g.ldb + n0 + n : 0));
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NT;
                const int k = idx / VPR, n = (idx % VPR) * VE;
                const bool ok = n0 + n < g.N && k < g.K;
                const int64_t left = g.N - (n0 + n);
                const uint4 m = ws_mask<T>(v[u], ok ? (left < VE ? (int)left : VE) : 0);
                T e[VE];
                __builtin_memcpy(e, &m, 16);
                if (idx < TOTAL) {
#pragma unroll
                    for (int q = 0; q < VE; ++q) Ws[(n + q) * WSTR + k] = e[q];
                }
            }
        }
    } else if (transB) {
        for (int idx = threadIdx.x; idx < BN * KP; idx += NT) {
            const int n = idx / KP, k = idx % KP;
            const bool ok = n0 + n < g.N && k < g.K;
            const T v = B[ok ? (n0 + n) * g.ldb + k : 0];
            Ws[n * WSTR + k] = ok ? v : (T)0;
        }
    } else {
        for (int idx = threadIdx.x; idx < BN * KP; idx += NT) {
            const int k = idx / BN, n = idx % BN;
            const bool ok = n0 + n < g.N && k < g.K;
            const T v = B[ok ? (int64_t)k * g.ldb + n0 + n : 0];
            Ws[n * WSTR + k] = ok ? v : (T)0;
        }
    }
    __syncthreads();

    const bool out_vec = (g.ldc % 4 == 0) && (((uintptr_t)g.C & 15) == 0);   // 4-column groups of C are aligned
    const int64_t nrb = (g.M + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * NW;
    int64_t rb = (int64_t)blockIdx.x * NW + wave;
    if (rb >= nrb) return;   // no workgroup barrier below this point
    // PD slices of loads are in flight per wavefront: the whole next block where the registers allow
    // it; with two wavefronts per SIMD (256 registers each) and four slices, two slices ahead
    constexpr int PD = (NS == 4 && NW > 4) ? 2 : NS;
    uint4 R[PD][4];
#pragma unroll
    for (int s = 0; s < PD; ++s)
        ws_load_slice<T>(R[s], A, g.lda, rb, s, g.M, g.K, lane);
    for (; rb < nrb; rb += stride) {
        const bool more = rb + stride < nrb;
        const int64_t rb_next = more ? rb + stride : rb;
        // this lane's element offset inside a slice.  Where registers are tight it passes through an empty
        // asm statement once per block: otherwise the compiler computes the masks of all slices ahead of
        // the row loop, keeps them in registers and spills
        int kb = (lane & 7) * HK;
        if (NW > 4) __asm__ volatile("" : "+v"(kb));
        // accumulators start from the bias of their columns (register r of lane half h: column
        // 8 (r / 4) + 4 h + r % 4 of the group), so the epilogue has nothing to add
        floatx16 acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            // (also without a bias, whose LDS copy then holds zeros: with constant-zero accumulators the
            // compiler's register allocation of the wide instances spills inside the loop)
            if (EX || NW > 4) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 c = *reinterpret_cast<const float4 *>(bias_lds + b * 32 + 8 * q + 4 * h);
                    acc[b][4 * q] = c.x; acc[b][4 * q + 1] = c.y; acc[b][4 * q + 2] = c.z; acc[b][4 * q + 3] = c.w;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;
            }
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            // LDS operations of one wavefront execute in program order; the compiler must not move
            // this slice's stage writes above the previous slice's fragment reads
            __asm__ volatile("" ::: "memory");
            // registers -> stage (row-major, elements at or past K zeroed), then refill the registers
            const int left = (int)g.K - (s * SK + kb);
            const int nv = left >= HK ? HK : (left > 0 ? left : 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint4 v = ws_mask<T>(R[s % PD][j], nv);
                *reinterpret_cast<uint4 *>(As + ((lane >> 3) + 8 * j) * ASTR + (lane & 7) * HK) = v;
            }
            if (s + PD < NS) ws_load_slice<T>(R[s % PD], A, g.lda, rb, s + PD, g.M, g.K, lane);
            else ws_load_slice<T>(R[s % PD], A, g.lda, rb_next, s + PD - NS, g.M, g.K, lane);
#pragma unroll
            for (int c = 0; c < (HALF ? SK / CK / 2 : SK / CK); ++c) {
                const uint4 a = *reinterpret_cast<const uint4 *>(As + l32 * ASTR + c * CK + h * HK);
                const T *wrow = Ws + l32 * WSTR + s * SK + c * CK + h * HK;
                if constexpr (sizeof(T) == 4) {
                    const float a0 = __uint_as_float(a.x), a1 = __uint_as_float(a.y), a2 = __uint_as_float(a.z),
                                a3 = __uint_as_float(a.w);
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const float4 w = *reinterpret_cast<const float4 *>(wrow + b * 32 * WSTR);
                        floatx16 cc = acc[b];
                        cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.x, a0, cc, 0, 0, 0);
                        cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.y, a1, cc, 0, 0, 0);
                        cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.z, a2, cc, 0, 0, 0);
                        cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.w, a3, cc, 0, 0, 0);
                        acc[b] = cc;
                    }
                } else {
                    bf16x8 af;
                    __builtin_memcpy(&af, &a, 16);
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const bf16x8 w = *reinterpret_cast<const bf16x8 *>(wrow + b * 32 * WSTR);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, af, acc[b], 0, 0, 0);
                    }
                }
            }
        }
        const int64_t row = rb * 32 + l32;
        if constexpr (FAST && sizeof(T) == 4) ws_epilogue_rows_f32<EX, MK, RG, NB>(g, acc, rb * 32, n0, lane, reinterpret_cast<float *>(As));
        else if constexpr (FAST) ws_epilogue_rows_bf16<EX, MK, (NW > 4), RG, NB>(g, acc, rb * 32, n0, lane, reinterpret_cast<uint32_t *>(As));
        else if (row < g.M) ws_epilogue<sizeof(T) == 2, EX, false, NB>(g, acc, row, n0, h, out_vec);
    }
}

// ---------------------------------------------------------------------------------------------
// fp32 data on the bf16 matrix cores (three-way exact splitting, six products; see
// gt_combine_x3.hip for the arithmetic).  v_mfma_f32_32x32x2f32 makes the fp32 form of the kernel
// above matrix bound (128 x 64 weights: 8,192 MFMA cycles per 32-row block against 3,072 here), so
// where the three weight planes fit in LDS the fp32 products run here instead.  The weights are
// split once, while they are put into LDS ([plane][n][k] bf16, k contiguous); a lane reads its
// eight consecutive k of A from the stage as fp32 and splits them in registers.
// ---------------------------------------------------------------------------------------------
__device__ inline void ws_split3(float x, uint32_t &hi, uint32_t &mid, uint32_t &lo) {
    const uint32_t h = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(h);
    const uint32_t m = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(m);
    hi = h; mid = m; lo = __float_as_uint(r2);
}
// upper halves of two words as one word: (b & 0xffff0000) | (a >> 16)
__device__ inline uint32_t ws_pack_hi16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

template <int NB, int NS>
constexpr size_t ws_x3_lds_bytes() {
    return (size_t)3 * NB * 32 * (NS * 32 + 8) * 2 + 4 * GEMM_STAGE_FLOATS(1) * 4 + (size_t)NB * 32 * 4;
}
template <int NB, int NS>
constexpr int ws_x3_per_cu() { return ws_x3_lds_bytes<NB, NS>() <= 80 * 1024 ? 2 : 1; }

template <int NB, int NS, bool EX, bool FAST, bool MK, bool RG>
__global__ void __launch_bounds__(256, (ws_x3_per_cu<NB, NS>())) k_gemm_ws_x3(const GemmArgs g, const int transB) {
    constexpr int SK = 32;                      // k per slice (128 bytes of fp32)
    constexpr int KP = NS * SK;                 // K capacity of this instance
    constexpr int WSTR = KP + 8;                // plane row stride in bf16 elements (16 bytes past a multiple of 64)
    constexpr int ASTR = SK + 4;                // stage row stride in floats (144 bytes)
    constexpr int BN = NB * 32;
    constexpr int PLANE = BN * WSTR;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *Wp = reinterpret_cast<bf16_t *>(smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    float *As = reinterpret_cast<float *>(smem + (size_t)3 * PLANE * 2 + (size_t)wave * GEMM_STAGE_FLOATS(1) * 4);
    float *bias_lds = reinterpret_cast<float *>(smem + (size_t)3 * PLANE * 2 + 4 * (size_t)GEMM_STAGE_FLOATS(1) * 4);
    const float *A = static_cast<const float *>(g.A);
    const float *B = static_cast<const float *>(g.B);
    const int64_t n0 = (int64_t)blockIdx.y * BN;
    for (int n = threadIdx.x; n < BN; n += 256) bias_lds[n] = (g.bias && n0 + n < g.N) ? g.bias[n0 + n] : 0.0f;

    // the weight slice, once, as three planes: Wp[plane][n][k] = piece of op(B)(k, n0 + n), zero
    // outside (K, N).  A thread takes quads of four elements that are consecutive in memory, eight
    // quads in flight.
    {
        constexpr int TOTAL = BN * KP / 4;
        for (int base = threadIdx.x; base < TOTAL; base += 256 * 8) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * 256;
                int n, k;
                if (transB) { n = idx / (KP / 4); k = (idx % (KP / 4)) * 4; }     // B[n][k..k+3]
                else { k = idx / (BN / 4); n = (idx % (BN / 4)) * 4; }            // B[k][n..n+3]
                const bool ok = idx < TOTAL && n0 + n < g.N && k < g.K;
                const int64_t off = transB ? (n0 + n) * g.ldb + k : (int64_t)k * g.ldb + n0 + n;
                const int64_t lim = transB ? g.K - k : g.N - (n0 + n);            // elements of the quad inside
                if (g.vecB) {
                    v[u] = *reinterpret_cast<const float4 *>(B + (ok ? off : 0));
                } else {
                    v[u].x = B[ok ? off : 0];
                    v[u].y = B[ok && lim > 1 ? off + 1 : 0];
                    v[u].z = B[ok && lim > 2 ? off + 2 : 0];
                    v[u].w = B[ok && lim > 3 ? off + 3 : 0];
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * 256;
                if (idx >= TOTAL) continue;
                int n, k;
                if (transB) { n = idx / (KP / 4); k = (idx % (KP / 4)) * 4; }
                else { k = idx / (BN / 4); n = (idx % (BN / 4)) * 4; }
                const bool ok = n0 + n < g.N && k < g.K;
                const int64_t lim = transB ? g.K - k : g.N - (n0 + n);
                const float x[4] = {ok ? v[u].x : 0.0f, ok && lim > 1 ? v[u].y : 0.0f, ok && lim > 2 ? v[u].z : 0.0f,
                                    ok && lim > 3 ? v[u].w : 0.0f};
                uint32_t hi[4], mi[4], lo[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) ws_split3(x[q], hi[q], mi[q], lo[q]);
                if (transB) {    // four consecutive k of one row: one 8-byte run per plane
                    bf16_t *d = Wp + n * WSTR + k;
                    *reinterpret_cast<uint2 *>(d) = make_uint2(ws_pack_hi16(hi[0], hi[1]), ws_pack_hi16(hi[2], hi[3]));
                    *reinterpret_cast<uint2 *>(d + PLANE) = make_uint2(ws_pack_hi16(mi[0], mi[1]), ws_pack_hi16(mi[2], mi[3]));
                    *reinterpret_cast<uint2 *>(d + 2 * PLANE) = make_uint2(ws_pack_hi16(lo[0], lo[1]), ws_pack_hi16(lo[2], lo[3]));
                } else {         // four consecutive n at one k: one element in each of four rows
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        bf16_t *d = Wp + (n + q) * WSTR + k;
                        d[0] = (bf16_t)(hi[q] >> 16);
                        d[PLANE] = (bf16_t)(mi[q] >> 16);
                        d[2 * PLANE] = (bf16_t)(lo[q] >> 16);
                    }
                }
            }
        }
    }
    __syncthreads();

    const bool out_vec = (g.ldc % 4 == 0) && (((uintptr_t)g.C & 15) == 0);
    const int64_t nrb = (g.M + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * 4;
    int64_t rb = (int64_t)blockIdx.x * 4 + wave;
    if (rb >= nrb) return;   // no workgroup barrier below this point
    uint4 R[NS][4];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        ws_load_slice<float>(R[s], A, g.lda, rb, s, g.M, g.K, lane);
    for (; rb < nrb; rb += stride) {
        const bool more = rb + stride < nrb;
        const int64_t rb_next = more ? rb + stride : rb;
        floatx16 acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (EX) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 c = *reinterpret_cast<const float4 *>(bias_lds + b * 32 + 8 * q + 4 * h);
                    acc[b][4 * q] = c.x; acc[b][4 * q + 1] = c.y; acc[b][4 * q + 2] = c.z; acc[b][4 * q + 3] = c.w;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;
            }
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            __asm__ volatile("" ::: "memory");     // stage writes stay below the previous slice's fragment reads
            const int64_t left = g.K - ((int64_t)s * SK + (lane & 7) * 4);
            const int nv = left >= 4 ? 4 : (left > 0 ? (int)left : 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint4 v = ws_mask<float>(R[s][j], nv);
                *reinterpret_cast<uint4 *>(As + ((lane >> 3) + 8 * j) * ASTR + (lane & 7) * 4) = v;
            }
            ws_load_slice<float>(R[s], A, g.lda, rb_next, s, g.M, g.K, lane);
#pragma unroll
            for (int t = 0; t < SK / 16; ++t) {    // MFMA steps of 16 k: lane half h supplies k = 16 t + 8 h .. + 7
                const float *ap = As + l32 * ASTR + t * 16 + h * 8;
                const float4 a0 = *reinterpret_cast<const float4 *>(ap), a1 = *reinterpret_cast<const float4 *>(ap + 4);
                const float x[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                uint32_t hi[8], mi[8], lo[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) ws_split3(x[q], hi[q], mi[q], lo[q]);
                uint4 ph, pm, pl;
                ph = make_uint4(ws_pack_hi16(hi[0], hi[1]), ws_pack_hi16(hi[2], hi[3]), ws_pack_hi16(hi[4], hi[5]), ws_pack_hi16(hi[6], hi[7]));
                pm = make_uint4(ws_pack_hi16(mi[0], mi[1]), ws_pack_hi16(mi[2], mi[3]), ws_pack_hi16(mi[4], mi[5]), ws_pack_hi16(mi[6], mi[7]));
                pl = make_uint4(ws_pack_hi16(lo[0], lo[1]), ws_pack_hi16(lo[2], lo[3]), ws_pack_hi16(lo[4], lo[5]), ws_pack_hi16(lo[6], lo[7]));
                bf16x8 ah, am, al;
                __builtin_memcpy(&ah, &ph, 16);
                __builtin_memcpy(&am, &pm, 16);
                __builtin_memcpy(&al, &pl, 16);
                const bf16_t *wrow = Wp + l32 * WSTR + s * SK + t * 16 + h * 8;
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const bf16x8 wh = *reinterpret_cast<const bf16x8 *>(wrow + b * 32 * WSTR);
                    const bf16x8 wm = *reinterpret_cast<const bf16x8 *>(wrow + b * 32 * WSTR + PLANE);
                    const bf16x8 wl = *reinterpret_cast<const bf16x8 *>(wrow + b * 32 * WSTR + 2 * PLANE);
                    floatx16 cc = acc[b];
                    // smallest terms first: lo*hi, hi*lo, mid*mid, then mid*hi, hi*mid, then hi*hi
                    cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wl, ah, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh, al, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wm, am, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wm, ah, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh, am, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh, ah, cc, 0, 0, 0);
                    acc[b] = cc;
                }
            }
        }
        const int64_t row = rb * 32 + l32;
        if constexpr (FAST) ws_epilogue_rows_f32<EX, MK, RG, NB>(g, acc, rb * 32, n0, lane, As);
        else if (row < g.M) ws_epilogue<false, EX, false, NB>(g, acc, row, n0, h, out_vec);
    }
}

// ---------------------------------------------------------------------------------------------
// Wide fp32 rows onto a narrow output: C[M, N] = act(A[M, K] op(B) + bias) with N <= 32 and K from
// 129 to 1,024 (a first layer that shrinks a wide input).  The product is bound by reading A once.
// Same scheme as above (three bf16 weight planes resident in LDS, wavefronts working alone on 32-row
// blocks through a private stage), but a row no longer fits the registers, so a wavefront streams
// it in slices of 128 bytes with four slices (16 KB) of loads in flight, held in a ring of four
// register sets.  The slice loop is unrolled completely (NSP = 8, 16 or 32 slices, K rounded up; a
// padding slice re-reads the row's first chunk and is staged as zeros): with a run-time loop the
// compiler drains every outstanding load at the loop head, which leaves one slice of work to hide
// a memory latency.  One 32-column MFMA block; for N <= 16 only 16 weight rows are kept (lanes
// 16..31 of the weight operand re-read rows 0..15; their output columns are never stored), which
// is what lets K = 1,024 fit: 3 x 16 x 1032 x 2 bytes = 97 KB.
// KFULL: K = 32 NSP, so no slice needs masking or clamping.  NR: weight rows kept (16 or 32).
// ---------------------------------------------------------------------------------------------
constexpr int WS_STREAM_WAVES = 8, WS_STREAM_PD = 4;
static size_t ws_stream_lds_bytes(int NR, int64_t K) {
    const int64_t kr = (K + 31) / 32 * 32;
    return (size_t)3 * NR * (kr + 8) * 2 + (size_t)WS_STREAM_WAVES * GEMM_STAGE_FLOATS(1) * 4 + 32 * 4;
}

template <bool EX, bool KFULL, int NSP>
__global__ void __launch_bounds__(WS_STREAM_WAVES * 64, 1) k_gemm_ws_stream_x3(const GemmArgs g, const int transB, const int NR) {
    constexpr int SK = 32, ASTR = SK + 4, NW = WS_STREAM_WAVES, NT = NW * 64, PD = WS_STREAM_PD;
    const int KR = (int)((g.K + SK - 1) / SK) * SK, WSTR = KR + 8, PLANE = NR * WSTR;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *Wp = reinterpret_cast<bf16_t *>(smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    float *As = reinterpret_cast<float *>(smem + (size_t)3 * PLANE * 2 + (size_t)wave * GEMM_STAGE_FLOATS(1) * 4);
    float *bias_lds = reinterpret_cast<float *>(smem + (size_t)3 * PLANE * 2 + NW * (size_t)GEMM_STAGE_FLOATS(1) * 4);
    const float *A = static_cast<const float *>(g.A);
    const float *B = static_cast<const float *>(g.B);
    if (threadIdx.x < 32) bias_lds[threadIdx.x] = (g.bias && threadIdx.x < g.N) ? g.bias[threadIdx.x] : 0.0f;
    // the weights, once per workgroup, as three planes Wp[plane][n][k], zero outside (K, N)
    for (int idx = threadIdx.x; idx < NR * KR; idx += NT) {
        int n, k;
        if (transB) { n = idx / KR; k = idx % KR; } else { k = idx / NR; n = idx % NR; }
        const bool ok = n < g.N && k < g.K;
        const float x = ok ? B[transB ? (int64_t)n * g.ldb + k : (int64_t)k * g.ldb + n] : 0.0f;
        uint32_t hi, mi, lo;
        ws_split3(x, hi, mi, lo);
        bf16_t *d = Wp + n * WSTR + k;
        d[0] = (bf16_t)(hi >> 16);
        d[PLANE] = (bf16_t)(mi >> 16);
        d[2 * PLANE] = (bf16_t)(lo >> 16);
    }
    __syncthreads();

    const bool out_vec = (g.ldc % 4 == 0) && (((uintptr_t)g.C & 15) == 0);
    const int64_t nrb = (g.M + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * NW;
    int64_t rb = (int64_t)blockIdx.x * NW + wave;
    if (rb >= nrb) return;   // no workgroup barrier below this point
    // this lane's four rows of a block (lane / 8 + 8 i, clamped to the last row) at its 16-byte chunk of a slice
    auto row_ptrs = [&](const float *(&rp)[4], int64_t blk) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int64_t row = blk * 32 + (lane >> 3) + 8 * i;
            if (row >= g.M) row = g.M - 1;
            rp[i] = A + row * g.lda + (lane & 7) * 4;
        }
    };
    // kb: this lane's element offset inside a slice, (lane & 7) * 4.  The loop below passes it through an empty
    // asm statement once per block: otherwise the compiler computes the masks of all NSP slices once, ahead of
    // the block loop, and keeps them in registers (spilling them when NSP = 32)
    auto load_slice = [&](uint4 (&r)[4], const float *const (&rp)[4], int s, int kb) {
        int k = s * SK;
        if (!KFULL && k + kb >= g.K) k = -kb;   // chunks at or past K re-read the row's first chunk
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = *reinterpret_cast<const uint4 *>(rp[i] + k);
    };
    const float *rp[4], *rpn[4];
    row_ptrs(rp, rb);
    uint4 R[PD][4];
#pragma unroll
    for (int j = 0; j < PD; ++j) load_slice(R[j], rp, j, (lane & 7) * 4);
    const bf16_t *wlane = Wp + (l32 & (NR - 1)) * WSTR + h * 8;
    for (; rb < nrb; rb += stride) {
        const int64_t rb_next = rb + stride < nrb ? rb + stride : rb;
        row_ptrs(rpn, rb_next);
        int kb = (lane & 7) * 4;
        if (!KFULL) __asm__ volatile("" : "+v"(kb));
        floatx16 acc[1];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 c = *reinterpret_cast<const float4 *>(bias_lds + 8 * q + 4 * h);
            acc[0][4 * q] = c.x; acc[0][4 * q + 1] = c.y; acc[0][4 * q + 2] = c.z; acc[0][4 * q + 3] = c.w;
        }
#pragma unroll
        for (int s = 0; s < NSP; ++s) {
            const int j = s % PD;
            __asm__ volatile("" ::: "memory");     // stage writes stay below the previous slice's fragment reads
            const int left = (int)g.K - (s * SK + kb);
            const int nv = left >= 4 ? 4 : (left > 0 ? left : 0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<uint4 *>(As + ((lane >> 3) + 8 * i) * ASTR + (lane & 7) * 4) =
                    KFULL ? R[j][i] : ws_mask<float>(R[j][i], nv);
            // refill: four slices ahead, which is the next block's row once this one's slices are all requested
            if (s + PD < NSP) load_slice(R[j], rp, s + PD, kb);
            else load_slice(R[j], rpn, s + PD - NSP, kb);
            // a padding slice (all zeros in the stage) multiplies the last real slice's weights
            const int ks = KFULL ? s * SK : (s * SK < KR ? s * SK : KR - SK);
#pragma unroll
            for (int t = 0; t < SK / 16; ++t) {    // MFMA steps of 16 k: lane half h supplies k = 16 t + 8 h .. + 7
                const float *ap = As + l32 * ASTR + t * 16 + h * 8;
                const float4 a0 = *reinterpret_cast<const float4 *>(ap), a1 = *reinterpret_cast<const float4 *>(ap + 4);
                const float x[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                uint32_t hi[8], mi[8], lo[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) ws_split3(x[q], hi[q], mi[q], lo[q]);
                uint4 ph, pm, pl;
                ph = make_uint4(ws_pack_hi16(hi[0], hi[1]), ws_pack_hi16(hi[2], hi[3]), ws_pack_hi16(hi[4], hi[5]), ws_pack_hi16(hi[6], hi[7]));
                pm = make_uint4(ws_pack_hi16(mi[0], mi[1]), ws_pack_hi16(mi[2], mi[3]), ws_pack_hi16(mi[4], mi[5]), ws_pack_hi16(mi[6], mi[7]));
                pl = make_uint4(ws_pack_hi16(lo[0], lo[1]), ws_pack_hi16(lo[2], lo[3]), ws_pack_hi16(lo[4], lo[5]), ws_pack_hi16(lo[6], lo[7]));
                bf16x8 ah, am, al;
                __builtin_memcpy(&ah, &ph, 16);
                __builtin_memcpy(&am, &pm, 16);
                __builtin_memcpy(&al, &pl, 16);
                const bf16_t *wrow = wlane + ks + t * 16;
                const bf16x8 wh = *reinterpret_cast<const bf16x8 *>(wrow);
                const bf16x8 wm = *reinterpret_cast<const bf16x8 *>(wrow + PLANE);
                const bf16x8 wl = *reinterpret_cast<const bf16x8 *>(wrow + 2 * PLANE);
                floatx16 cc = acc[0];
                // smallest terms first: lo*hi, hi*lo, mid*mid, then mid*hi, hi*mid, then hi*hi
                cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wl, ah, cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh, al, cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wm, am, cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wm, ah, cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh, am, cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh, ah, cc, 0, 0, 0);
                acc[0] = cc;
            }
        }
        const int64_t row = rb * 32 + l32;
        if (row < g.M) ws_epilogue<false, EX, false, 1>(g, acc, row, 0, h, out_vec);
#pragma unroll
        for (int i = 0; i < 4; ++i) rp[i] = rpn[i];
    }
}

// shapes of the streaming kernel: fp32, N <= 32, rows longer than the register-resident kernels take,
// at most 1,024 elements, and short enough for the three weight planes to fit in LDS beside the stages
static bool ws_stream_shape(gt_dtype dtype, int64_t N, int64_t K, int *NR, int *nsp) {
    if (dtype != GT_F32 || N > 32 || K <= 4 * WsGeom<float>::SK || K > 1024) return false;
    const int nr = N <= 16 ? 16 : 32;
    if (ws_stream_lds_bytes(nr, K) > 160 * 1024) return false;
    *NR = nr; *nsp = K <= 256 ? 8 : (K <= 512 ? 16 : 32);
    return true;
}

template <int NSP>
static gt_status ws_stream_launch_n(const GemmArgs &g, int transB, int NR, hipStream_t st) {
    const size_t lds = ws_stream_lds_bytes(NR, g.K);
    const bool extras = g.bias || g.relu || g.mask;
    const int64_t nrb = (g.M + 31) / 32;
    int64_t gx = (nrb + WS_STREAM_WAVES - 1) / WS_STREAM_WAVES;
    if (gx > 256) gx = 256;
    const bool kfull = g.K == 32 * NSP;
#define GT_WS_STREAM(EX_, KF_)                                                                                       \
    do {                                                                                                             \
        GT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_ws_stream_x3<EX_, KF_, NSP>),              \
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                           \
        k_gemm_ws_stream_x3<EX_, KF_, NSP><<<(unsigned)gx, WS_STREAM_WAVES * 64, lds, st>>>(g, transB, NR);          \
    } while (0)
    if (extras && kfull) GT_WS_STREAM(true, true);
    else if (extras) GT_WS_STREAM(true, false);
    else if (kfull) GT_WS_STREAM(false, true);
    else GT_WS_STREAM(false, false);
#undef GT_WS_STREAM
    GT_LAUNCH_CHECK("k_gemm_ws_stream_x3");
    return GT_OK;
}

static gt_status ws_stream_launch(const GemmArgs &g, int transB, hipStream_t st) {
    int NR = 0, nsp = 0;
    if (!ws_stream_shape(GT_F32, g.N, g.K, &NR, &nsp)) return gt_fail(GT_ERR_INTERNAL, "ws_stream_launch: shape not supported");
    if (nsp == 8) return ws_stream_launch_n<8>(g, transB, NR, st);
    if (nsp == 16) return ws_stream_launch_n<16>(g, transB, NR, st);
    return ws_stream_launch_n<32>(g, transB, NR, st);
}

template <int NB, int NS, bool EX, bool FAST, bool MK = false, bool RG = false>
gt_status ws_x3_launch_ex(const GemmArgs &g, int transB, hipStream_t st) {
    constexpr size_t lds = ws_x3_lds_bytes<NB, NS>();
    if (lds > 64 * 1024) {
        GT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_ws_x3<NB, NS, EX, FAST, MK, RG>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    }
    const int64_t nrb = (g.M + 31) / 32;
    const int per_cu = ws_x3_per_cu<NB, NS>();
    int64_t gx = (nrb + 3) / 4;
    if (gx > 256 * per_cu) gx = 256 * per_cu;
    dim3 grid((unsigned)gx, (unsigned)((g.N + NB * 32 - 1) / (NB * 32)), 1);
    k_gemm_ws_x3<NB, NS, EX, FAST, MK, RG><<<grid, 256, lds, st>>>(g, transB);
    GT_LAUNCH_CHECK("k_gemm_ws_x3");
    return GT_OK;
}

template <int NB, int NS>
gt_status ws_x3_launch(const GemmArgs &g, int transB, hipStream_t st) {
    const bool extras = g.bias || g.relu || g.mask;
    if constexpr (NB >= 4) {
        const bool fast = g.N % (NB * 32) == 0 && g.ldc % 4 == 0 && (((uintptr_t)g.C & 15) == 0) &&
                          (!g.mask || (g.ldmask % 8 == 0 && ((uintptr_t)g.mask & 15) == 0));
        if (fast)
            return g.mask ? ws_x3_launch_ex<NB, NS, true, true, true>(g, transB, st)
                 : extras ? ws_x3_launch_ex<NB, NS, true, true>(g, transB, st)
                          : ws_x3_launch_ex<NB, NS, false, true>(g, transB, st);
    }
    if constexpr (NB == 2) {   // at most 64 fp32 columns, any N: the staged, row-major epilogue with a ragged end
        const bool rows = g.ldc % 4 == 0 && (((uintptr_t)g.C & 15) == 0) &&
                          (!g.mask || (g.ldmask % 8 == 0 && ((uintptr_t)g.mask & 15) == 0));
        if (rows)
            return g.mask ? ws_x3_launch_ex<NB, NS, true, true, true, true>(g, transB, st)
                 : extras ? ws_x3_launch_ex<NB, NS, true, true, false, true>(g, transB, st)
                          : ws_x3_launch_ex<NB, NS, false, true, false, true>(g, transB, st);
    }
    return extras ? ws_x3_launch_ex<NB, NS, true, false>(g, transB, st)
                  : ws_x3_launch_ex<NB, NS, false, false>(g, transB, st);
}

template <typename T, int NB, int NS, bool EX, bool FAST, bool MK = false, bool HALF = false, bool RG = false>
gt_status ws_launch_ex(const GemmArgs &g, int transB, hipStream_t st) {
    constexpr int NW = ws_waves<T, NB, NS>();
    constexpr size_t lds = ws_lds_bytes<T, NB, NS, NW>();
    // More than 64 KB of dynamic LDS has to be allowed per kernel.  Done on every launch that needs
    // it (a host-side setting, no stream operation), so the first launch of an instance behaves
    // like any other, also under stream capture.
    if (lds > 64 * 1024) {
        GT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_ws<T, NB, NS, EX, FAST, MK, HALF, RG>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    }
    const int64_t nrb = (g.M + 31) / 32;
    const int per_cu = ws_per_cu<T, NB, NS>();
    int64_t gx = (nrb + NW - 1) / NW;
    if (gx > 256 * per_cu) gx = 256 * per_cu;
    dim3 grid((unsigned)gx, (unsigned)((g.N + NB * 32 - 1) / (NB * 32)), 1);
    k_gemm_ws<T, NB, NS, EX, FAST, MK, HALF, RG><<<grid, NW * 64, lds, st>>>(g, transB);
    GT_LAUNCH_CHECK("k_gemm_ws");
    return GT_OK;
}

template <typename T, int NB, int NS>
gt_status ws_launch(const GemmArgs &g, int transB, hipStream_t st) {
    const bool extras = g.bias || g.relu || g.mask;
    if constexpr (NB >= 4) {   // the branch-free form exists for the wide slices, where the stores dominate
        // (a bf16 C is written 16 bytes, eight columns, per lane)
        const bool fast = g.N % (NB * 32) == 0 && g.ldc % (sizeof(T) == 2 ? 8 : 4) == 0 && (((uintptr_t)g.C & 15) == 0) &&
                          (!g.mask || (g.ldmask % 8 == 0 && ((uintptr_t)g.mask & 15) == 0));
        if constexpr (NS == 1) {
            if (fast && g.K <= WsGeom<T>::SK / 2)
                return g.mask ? ws_launch_ex<T, NB, NS, true, true, true, true>(g, transB, st)
                     : extras ? ws_launch_ex<T, NB, NS, true, true, false, true>(g, transB, st)
                              : ws_launch_ex<T, NB, NS, false, true, false, true>(g, transB, st);
        }
        if (fast)
            return g.mask ? ws_launch_ex<T, NB, NS, true, true, true>(g, transB, st)
                 : extras ? ws_launch_ex<T, NB, NS, true, true>(g, transB, st)
                          : ws_launch_ex<T, NB, NS, false, true>(g, transB, st);
    }
    if constexpr (NB == 2 && sizeof(T) == 2) {   // at most 64 bf16 columns, any N: the staged, row-major epilogue with a ragged end
        const bool rows = g.ldc % 8 == 0 && (((uintptr_t)g.C & 15) == 0) &&
                          (!g.mask || (g.ldmask % 8 == 0 && ((uintptr_t)g.mask & 15) == 0));
        if (rows)
            return g.mask ? ws_launch_ex<T, NB, NS, true, true, true, false, true>(g, transB, st)
                 : extras ? ws_launch_ex<T, NB, NS, true, true, false, false, true>(g, transB, st)
                          : ws_launch_ex<T, NB, NS, false, true, false, false, true>(g, transB, st);
    }
    return extras ? ws_launch_ex<T, NB, NS, true, false>(g, transB, st)
                  : ws_launch_ex<T, NB, NS, false, false>(g, transB, st);
}

template <typename T, int NB>
gt_status ws_pick_ns(const GemmArgs &g, int transB, hipStream_t st) {
    const int64_t slices = (g.K + WsGeom<T>::SK - 1) / WsGeom<T>::SK;
    if constexpr (sizeof(T) == 4 && NB <= 4) {
        // fp32 on the bf16 matrix cores for outputs of up to 128 columns (measured on MI355X, 2^18 rows:
        // 128 -> 41 0.074 -> 0.052 ms, 41 -> 128 0.067 -> 0.053 ms); wider outputs are bound by their
        // stores and ran slower this way (2^20 rows, 16 -> 1024: 1.15 -> 1.30 ms), they keep the fp32 MFMA
        if (slices <= 1) return ws_x3_launch<NB, 1>(g, transB, st);
        if (slices <= 2) return ws_x3_launch<NB, 2>(g, transB, st);
        return ws_x3_launch<NB, 4>(g, transB, st);
    } else {
        if (slices <= 1) return ws_launch<T, NB, 1>(g, transB, st);
        if (slices <= 2) return ws_launch<T, NB, 2>(g, transB, st);
        return ws_launch<T, NB, 4>(g, transB, st);
    }
}

template <typename T>
gt_status ws_pick(const GemmArgs &g, int transB, hipStream_t st) {
    if (g.N <= 64) return ws_pick_ns<T, 2>(g, transB, st);
    if (g.N <= 128) return ws_pick_ns<T, 4>(g, transB, st);
    return ws_pick_ns<T, 8>(g, transB, st);
}

}  // namespace

// (the caller also requires C to have A's element type and no row scale or addend)
bool gt_gemm_ws_applicable(gt_dtype dtype, int transA, int64_t M, int64_t N, int64_t K, int vecA) {
    const int64_t kcap = dtype == GT_BF16 ? 4 * WsGeom<bf16_t>::SK : 4 * WsGeom<float>::SK;   // 256 / 128
    int nr, nsp;
    return !transA && vecA && K >= 1 && (K <= kcap || ws_stream_shape(dtype, N, K, &nr, &nsp)) && N >= 1 && M >= 8192;
}

gt_status gt_gemm_ws_launch(const GemmArgs &g, gt_dtype dtype, int transB, hipStream_t st) {
    if (dtype == GT_F32 && g.K > 4 * WsGeom<float>::SK) return ws_stream_launch(g, transB, st);
    return dtype == GT_BF16 ? ws_pick<bf16_t>(g, transB, st) : ws_pick<float>(g, transB, st);
}
