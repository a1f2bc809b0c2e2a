// Internal GEMM declarations shared by gt_combine.hip, gt_combine_x3.hip and the layer calls.
#pragma once
#include "gt_internal.h"

size_t gt_gemm_ws_bytes(int transA, int64_t M, int64_t N, int64_t K);

// C = act(rowscale .* (op(A) op(B)) + C_in + bias); C_in (same type and shape as C) may be null.
gt_status gt_gemm_run(const char *fn, gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, const void *B, int64_t ldb, const float *bias, const float *rowscale,
                      gt_act act, const void *Cin, int64_t ldcin, void *C, int64_t ldc, gt_dtype c_dtype, void *ws,
                      size_t ws_bytes, hipStream_t st, const void *mask = nullptr, int64_t ldmask = 0,
                      float *colsum_b = nullptr, bool pad_c = false);
// colsum_b (transA products with !transB only): also writes the N column sums of op(B) there, a
// by-product of streaming B (the bias gradient when B is dZ); sums have a fixed order.

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t gemm_bf16_t;

constexpr int GEMM_KT = 32;   // k-tile

__device__ inline uint32_t gemm_f32_to_bf16(float f) { return gt_to_bf16(f); }
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
    const void *mask; int64_t ldmask; // optional, type and shape of C: outputs are zeroed where mask <= 0
    float *colsum;                 // optional [splits][N]: column sums of op(B) over each split's k-range (!transB),
                                   // written by the workgroups of row tile 0
    int relu;
    int c_bf16;
    int64_t M, N, K;
    int64_t k_per_split;           // multiple of KT
    int vecA, vecB;                // 16-byte loads allowed
    int ntm, ntn;                  // output tiles along M and N (host side; see gemm_tile_of_block)
    int split_xcd;                 // splits % 8 == 0: the output tiles of one k-range run on one XCD
    int pad_c;                     // rows of C are padded and the padding may be written (zeros): a row's last
                                   // 16 bytes go out whole instead of in pieces (honoured by the staged epilogues)
};

// Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own L2.  The
// 1-D grid is therefore read as (xcd, sequence number within the xcd): an XCD walks one row tile
// at a time through all of its column tiles, so the row tile of op(A) that those column tiles
// share is fetched into one L2 once.  Returns false for the padding workgroups of a ragged grid.
// Used only when there are many row tiles; with few (the weight-gradient shape) the plain order
// keeps all XCDs busy.
//
// A reduction cut into k-ranges (gridDim.z > 1) with a few output tiles: the tiles of one k-range read
// the same k-slab of the operand they share (the weight gradient's 5 row tiles of config 2 all read
// the whole of dZ).  In grid order they would land on different XCDs and the slab would cross the
// fabric once per tile; with split_xcd the linear workgroup id is read as (xcd, sequence number) and
// an XCD works through whole k-ranges, all tiles of a range back to back, so the re-reads hit its L2.
#define GEMM_SWIZZLE_MIN_ROW_TILES 64
__device__ inline bool gemm_tile_of_block(const GemmArgs &g, int &tile_m, int &tile_n, int &split) {
    if (g.split_xcd) {
        const int tiles = g.ntm * g.ntn;
        const int L = blockIdx.z * gridDim.x + blockIdx.x;
        const int xcd = L & 7, seq = L >> 3;
        const int t = seq % tiles;
        split = (seq / tiles) * 8 + xcd;
        tile_n = t % g.ntn;
        tile_m = t / g.ntn;
        return true;
    }
    split = blockIdx.z;
    const int L = blockIdx.x;
    if (g.ntm < GEMM_SWIZZLE_MIN_ROW_TILES) {
        tile_n = L % g.ntn;
        tile_m = L / g.ntn;
        return true;
    }
    const int xcd = L & 7, i = L >> 3;
    tile_n = i % g.ntn;
    tile_m = (i / g.ntn) * 8 + xcd;
    return tile_m < g.ntm;
}
static inline int gemm_split_xcd(int ntm, int ntn, int splits) {
    return ntm < GEMM_SWIZZLE_MIN_ROW_TILES && ntm * ntn > 1 && splits >= 16 && splits % 8 == 0;
}
static inline unsigned gemm_grid_x(int ntm, int ntn) {
    return (unsigned)((ntm < GEMM_SWIZZLE_MIN_ROW_TILES ? ntm : (ntm + 7) / 8 * 8) * ntn);
}


// Epilogue of a wavefront's TM x TN grid of 32x32 MFMA accumulators whose top-left element is
// (row0, col0).  Accumulator register r of lane (h, l32) holds row 8*(r/4) + 4*h + r%4, column l32,
// i.e. a lane owns single columns: storing from registers would write 4-byte pieces.  The tile is
// therefore passed through a per-wavefront LDS stage (32 rows at a time) and written row-major,
// four consecutive columns per lane, so every store instruction covers whole 128-byte lines.
// `stage` is this wavefront's private region of GEMM_STAGE_FLOATS(TN) floats; the caller has
// already put a workgroup barrier between the last operand read and this call.
#define GEMM_STAGE_STRIDE(TN) ((TN) * 32 + 4)
#define GEMM_STAGE_FLOATS(TN) (32 * GEMM_STAGE_STRIDE(TN))

template <int TM, int TN>
__device__ inline void gemm_epilogue(const GemmArgs &g, floatx16 (&acc)[TM][TN], int64_t row0, int64_t col0, int l32,
                                     int h, float *stage, int split) {
    constexpr int STRIDE = GEMM_STAGE_STRIDE(TN);
    constexpr int LPR = TN * 8;            // lanes per row: 4 columns each
    constexpr int RPI = 64 / LPR;          // rows per store instruction
    const bool partial = gridDim.z > 1;
    const int lane = h * 32 + l32;
    const int c4 = (lane % LPR) * 4;
    const int64_t col = col0 + c4;
    float *out_f = static_cast<float *>(g.C);
    gemm_bf16_t *out_h = static_cast<gemm_bf16_t *>(g.C);
    const int64_t ldc = partial ? g.N : g.ldc;
    if (partial) out_f += (int64_t)split * g.M * g.N;
    const bool as_bf16 = !partial && g.c_bf16;
    // whole vectors: inside N, or (padded rows whose padding may be written) the row's last one, zeros past N
    const bool vec_ok = (ldc % 4 == 0) && (((uintptr_t)g.C & 15) == 0) &&
                        (col + 4 <= g.N || (g.pad_c && !partial && col < g.N && col + 4 <= ldc));
    float bia[4] = {0.f, 0.f, 0.f, 0.f};
    if (!partial && g.bias) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (col + i < g.N) bia[i] = g.bias[col + i];
    }
#pragma unroll
    for (int a = 0; a < TM; ++a) {
        // registers -> stage: lanes write consecutive columns of one row (conflict free)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                stage[(8 * (r / 4) + 4 * h + (r % 4)) * STRIDE + b * 32 + l32] = acc[a][b][r];
        // stage -> memory, row-major (same wavefront wrote and reads: no workgroup barrier needed,
        // LDS operations of one wavefront complete in order)
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int rr = it * RPI + lane / LPR;
            const int64_t row = row0 + a * 32 + rr;
            const float4 v4 = *reinterpret_cast<const float4 *>(&stage[rr * STRIDE + c4]);
            if (row >= g.M || col >= g.N) continue;
            float v[4] = {v4.x, v4.y, v4.z, v4.w};
            if (!partial) {
                const float rs = g.rowscale ? g.rowscale[row] : 1.0f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float x = v[i];
                    if (g.rowscale) x *= rs;
                    if (g.Cin && col + i < g.N)
                        x += g.c_bf16 ? gemm_bf16_to_f32(static_cast<const gemm_bf16_t *>(g.Cin)[row * g.ldcin + col + i])
                                      : static_cast<const float *>(g.Cin)[row * g.ldcin + col + i];
                    x += bia[i];
                    if (g.relu) x = x > 0.0f ? x : 0.0f;
                    if (g.mask && col + i < g.N) {
                        const float mk = g.c_bf16 ? gemm_bf16_to_f32(static_cast<const gemm_bf16_t *>(g.mask)[row * g.ldmask + col + i])
                                                  : static_cast<const float *>(g.mask)[row * g.ldmask + col + i];
                        x = mk > 0.0f ? x : 0.0f;
                    }
                    v[i] = (col + i < g.N) ? x : 0.0f;
                }
            }
            if (as_bf16) {
                gemm_bf16_t *p = out_h + row * ldc + col;
                if (vec_ok) {
                    *reinterpret_cast<uint2 *>(p) = make_uint2(gt_pack_bf16(v[0], v[1]),
                                                               gt_pack_bf16(v[2], v[3]));
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (col + i < g.N) p[i] = (gemm_bf16_t)gemm_f32_to_bf16(v[i]);
                }
            } else {
                float *p = out_f + row * ldc + col;
                if (vec_ok) {
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

// fp32 GEMM through three-way bf16 splitting (gt_combine_x3.hip); 128 x 128 workgroup tiles.
gt_status gt_gemm_x3_launch(const GemmArgs &g, int transA, int transB, int splits, hipStream_t st);
void gt_gemm_x3_tile(int64_t M, int64_t N, int64_t *bm, int64_t *bn);

// Weight-stationary kernel for tall products with small K and N (gt_combine_ws.hip).
bool gt_gemm_ws_applicable(gt_dtype dtype, int transA, int64_t M, int64_t N, int64_t K, int vecA);
gt_status gt_gemm_ws_launch(const GemmArgs &g, gt_dtype dtype, int transB, hipStream_t st);
