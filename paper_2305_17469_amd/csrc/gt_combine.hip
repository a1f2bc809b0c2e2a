// Combination (the paper's Apply primitive: linear transform, bias, non-linearity) and its
// derivatives, as one LDS-tiled MFMA GEMM family:  C = act(op(A) op(B) + C_in + bias).
//
// The paper delegates this step to a vendor GEMM (Frontend section, Apply); here it is written
// for CDNA4: 64-lane wavefronts own 64x64 accumulator tiles built from 32x32 MFMA blocks
// (fp32 MFMA for fp32 data so fp32 accuracy is kept, bf16 MFMA with fp32 accumulation for bf16
// data), operands are staged through LDS in whichever layout their global layout gives without
// a transposing store, the next k-tile is prefetched into registers while the current one is
// multiplied, and the weight-gradient shape (reduction over the node dimension) is split over
// workgroups and summed in a fixed order, so results are reproducible.
#include "gt_internal.h"
#include "gt_combine.h"
#include "gt_trace.h"

namespace {

typedef gemm_bf16_t bf16_t;
constexpr int KT = 64;   // granularity of the split-k ranges: a multiple of every kernel's k-tile
__device__ inline uint32_t f32_to_bf16(float f) { return gemm_f32_to_bf16(f); }
__device__ inline float bf16_to_f32(uint32_t h) { return gemm_bf16_to_f32(h); }

// Global -> registers for a ROWS x COLS tile whose COLS direction is contiguous in memory.
// Element (r, c) sits at p[(r0 + r) * ld + c0 + c]; anything at or beyond (rlim, clim) reads 0.
template <typename T, int ROWS, int COLS>
struct TileLoader {
    static constexpr int VE = Elem<T>::VE;
    static constexpr int VPR = COLS / VE;                 // vectors per tile row
    static constexpr int TOTAL = ROWS * VPR;
    static constexpr int NV = (TOTAL + 255) / 256;        // vectors per thread
    uint4 reg[NV];
    int nvalid[NV];   // elements of reg[it] that lie inside the matrix; the rest is zeroed when the
                      // vector is stored to LDS (masking at load time would consume the data and
                      // stall the prefetch)

    // Branch free: an out-of-range vector reads the (always valid) start of the matrix instead and
    // is masked to zero afterwards, so all loads of a tile are issued back to back and stay in
    // flight together.  `vec` is uniform over the grid.
    __device__ inline void load(const T *p, int64_t ld, int64_t r0, int64_t c0, int64_t rlim, int64_t clim, int vec) {
        if (vec) {
#pragma unroll
            for (int it = 0; it < NV; ++it) {
                const int q = threadIdx.x + 256 * it;
                const int r = q / VPR, c = (q % VPR) * VE;
                const int64_t gr = r0 + r, gc = c0 + c;
                const bool ok = (TOTAL % 256 == 0 || q < TOTAL) && gr < rlim && gc < clim;
                reg[it] = *reinterpret_cast<const uint4 *>(p + (ok ? gr * ld + gc : 0));
                nvalid[it] = ok ? (int)((clim - gc) < VE ? (clim - gc) : VE) : 0;
            }
        } else {
#pragma unroll
            for (int it = 0; it < NV; ++it) {
                const int q = threadIdx.x + 256 * it;
                const int r = q / VPR, c = (q % VPR) * VE;
                const int64_t gr = r0 + r, gc = c0 + c;
                const bool rok = (TOTAL % 256 == 0 || q < TOTAL) && gr < rlim;
                T tmp[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    const bool ok = rok && gc + e < clim;
                    const T x = p[ok ? gr * ld + gc + e : 0];
                    tmp[e] = ok ? x : (T)0;
                }
                reg[it] = *reinterpret_cast<const uint4 *>(tmp);
                nvalid[it] = VE;
            }
        }
    }
    // adds this thread's (masked) elements to cs: the VE columns a thread loads are the same for all of
    // its vectors when 256 is a multiple of VPR
    __device__ inline void add_to(float (&cs)[VE]) const {
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int nv = nvalid[it];
            const uint32_t w[4] = {reg[it].x, reg[it].y, reg[it].z, reg[it].w};
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                float x;
                if constexpr (sizeof(T) == 4) x = __uint_as_float(w[e]);
                else x = __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
                cs[e] += e < nv ? x : 0.0f;
            }
        }
    }
    template <int STR>
    __device__ inline void store(T *lds) const {
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int q = threadIdx.x + 256 * it;
            const int r = q / VPR, c = (q % VPR) * VE;
            uint4 v = reg[it];
            const int nv = nvalid[it];
            if constexpr (sizeof(T) == 4) {
                v.x = nv > 0 ? v.x : 0u; v.y = nv > 1 ? v.y : 0u; v.z = nv > 2 ? v.z : 0u; v.w = nv > 3 ? v.w : 0u;
            } else {
                v.x &= nv >= 2 ? 0xffffffffu : (nv == 1 ? 0x0000ffffu : 0u);
                v.y &= nv >= 4 ? 0xffffffffu : (nv == 3 ? 0x0000ffffu : 0u);
                v.z &= nv >= 6 ? 0xffffffffu : (nv == 5 ? 0x0000ffffu : 0u);
                v.w &= nv >= 8 ? 0xffffffffu : (nv == 7 ? 0x0000ffffu : 0u);
            }
            if (TOTAL % 256 == 0 || q < TOTAL) *reinterpret_cast<uint4 *>(lds + r * STR + c) = v;
        }
    }
};

// op(A)(i,k): TA ? A[k*lda+i] : A[i*lda+k];   op(B)(k,j): TB ? B[j*ldb+k] : B[k*ldb+j]
// VA / VB: the operand allows 16-byte loads (aligned base, row stride a multiple of 16 bytes)
template <typename T, bool TA, bool TB, int WGM, int WGN, int TM, int TN, bool VA, bool VB>
__global__ void __launch_bounds__(256) k_gemm(const GemmArgs g) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    constexpr int PAD = Elem<T>::PAD;
    // k-tile of 32 for both types (64 was measured for bf16: fewer barrier rounds, but the extra
    // staging registers cost a wavefront of occupancy and the memory-bound shapes got slower)
    constexpr int KT = 32;
    constexpr int ASTR = TA ? BM + PAD : KT + PAD;
    constexpr int BSTR = TB ? KT + PAD : BN + PAD;
    constexpr int A_ELEMS = TA ? KT * ASTR : BM * ASTR;
    constexpr int B_ELEMS = TB ? BN * BSTR : KT * BSTR;
    // one LDS buffer: operand tiles during the k-loop, the per-wavefront output stages afterwards
    constexpr int TILE_BYTES = (A_ELEMS + B_ELEMS) * (int)sizeof(T);
    constexpr int STAGE_BYTES = 4 * GEMM_STAGE_FLOATS(TN) * 4;
    constexpr int SMEM_BYTES = TILE_BYTES > STAGE_BYTES ? TILE_BYTES : STAGE_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
    T *As = reinterpret_cast<T *>(smem);
    T *Bs = As + A_ELEMS;
    static_assert((A_ELEMS * sizeof(T)) % 16 == 0, "B tile must stay 16-byte aligned");
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int wm = wave / WGN, wn = wave % WGN;
    int tile_m, tile_n;
    int split;
    if (!gemm_tile_of_block(g, tile_m, tile_n, split)) return;   // whole workgroup leaves before any barrier
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int64_t kbeg = (int64_t)split * g.k_per_split;
    const int64_t kend = (kbeg + g.k_per_split < g.K) ? kbeg + g.k_per_split : g.K;
    const T *A = static_cast<const T *>(g.A);
    const T *B = static_cast<const T *>(g.B);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
    // column sums of op(B) over this workgroup's k-range, a by-product of loading B (row tile 0 only)
    constexpr int VEB = Elem<T>::VE;
    const bool do_cs = !TB && g.colsum && tile_m == 0;
    float cs[VEB];
#pragma unroll
    for (int e = 0; e < VEB; ++e) cs[e] = 0.0f;

    typedef TileLoader<T, TA ? KT : BM, TA ? BM : KT> LoadA;
    typedef TileLoader<T, TB ? BN : KT, TB ? KT : BN> LoadB;
    // Register stages: the loads of k-tile t + STAGES are issued while tile t is multiplied.
    constexpr int STAGES = 1;
    LoadA la[STAGES];
    LoadB lb[STAGES];
    auto fetch = [&](LoadA &sa, LoadB &sb, int64_t k0) {
        if (TA) sa.load(A, g.lda, k0, m0, kend, g.M, VA); else sa.load(A, g.lda, m0, k0, g.M, kend, VA);
        if (TB) sb.load(B, g.ldb, n0, k0, g.N, kend, VB); else sb.load(B, g.ldb, k0, n0, kend, g.N, VB);
    };
#pragma unroll
    for (int st = 0; st < STAGES; ++st)
        if (kbeg + st * KT < kend) fetch(la[st], lb[st], kbeg + st * KT);

    for (int64_t kb = kbeg; kb < kend; kb += STAGES * KT) {
#pragma unroll
      for (int st = 0; st < STAGES; ++st) {     // unrolled: every stage is addressed statically
        const int64_t k0 = kb + st * KT;
        if (k0 >= kend) break;
        __syncthreads();                      // previous tile fully consumed
        la[st].template store<ASTR>(As);
        lb[st].template store<BSTR>(Bs);
        if constexpr (!TB) {
            if (do_cs) lb[st].add_to(cs);
        }
        __syncthreads();
        if (k0 + STAGES * KT < kend) fetch(la[st], lb[st], k0 + STAGES * KT);

        if constexpr (sizeof(T) == 4) {
            // fp32: v_mfma_f32_32x32x2f32.  Lane half h owns k = h*16 + t of the tile at step t;
            // both operands use the same assignment, so the sum over the tile is complete.
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float af[TM][8], bf[TN][8];
                const int kk = h * 16 + half * 8;
#pragma unroll
                for (int a = 0; a < TM; ++a) {
                    const int i = (wm * TM + a) * 32 + l32;
                    if constexpr (!TA) {
                        const float4 x = *reinterpret_cast<const float4 *>(&As[i * ASTR + kk]);
                        const float4 y = *reinterpret_cast<const float4 *>(&As[i * ASTR + kk + 4]);
                        af[a][0] = x.x; af[a][1] = x.y; af[a][2] = x.z; af[a][3] = x.w;
                        af[a][4] = y.x; af[a][5] = y.y; af[a][6] = y.z; af[a][7] = y.w;
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q) af[a][q] = As[(kk + q) * ASTR + i];
                    }
                }
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    const int j = (wn * TN + b) * 32 + l32;
                    if constexpr (TB) {
                        const float4 x = *reinterpret_cast<const float4 *>(&Bs[j * BSTR + kk]);
                        const float4 y = *reinterpret_cast<const float4 *>(&Bs[j * BSTR + kk + 4]);
                        bf[b][0] = x.x; bf[b][1] = x.y; bf[b][2] = x.z; bf[b][3] = x.w;
                        bf[b][4] = y.x; bf[b][5] = y.y; bf[b][6] = y.z; bf[b][7] = y.w;
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q) bf[b][q] = Bs[(kk + q) * BSTR + j];
                    }
                }
#pragma unroll
                for (int q = 0; q < 8; ++q)
#pragma unroll
                    for (int a = 0; a < TM; ++a)
#pragma unroll
                        for (int b = 0; b < TN; ++b)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a][q], bf[b][q], acc[a][b], 0, 0, 0);
            }
        } else {
            // bf16: v_mfma_f32_32x32x16_bf16.  Lane half h supplies k = s*16 + h*8 .. +7.
#pragma unroll
            for (int s = 0; s < KT / 16; ++s) {
                bf16x8 af[TM], bf[TN];
                const int kk = s * 16 + h * 8;
#pragma unroll
                for (int a = 0; a < TM; ++a) {
                    const int i = (wm * TM + a) * 32 + l32;
                    if constexpr (!TA) {
                        af[a] = *reinterpret_cast<const bf16x8 *>(&As[i * ASTR + kk]);
                    } else {
                        bf16_t tmp[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) tmp[q] = As[(kk + q) * ASTR + i];
                        af[a] = *reinterpret_cast<const bf16x8 *>(tmp);
                    }
                }
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    const int j = (wn * TN + b) * 32 + l32;
                    if constexpr (TB) {
                        bf[b] = *reinterpret_cast<const bf16x8 *>(&Bs[j * BSTR + kk]);
                    } else {
                        bf16_t tmp[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) tmp[q] = Bs[(kk + q) * BSTR + j];
                        bf[b] = *reinterpret_cast<const bf16x8 *>(tmp);
                    }
                }
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
            }
        }
      }
    }

    __syncthreads();   // every wavefront is done reading the operand tiles
    if constexpr (!TB) {
        if (do_cs) {   // uniform over the workgroup
            // thread t holds columns (t % VPR) * VE ..; the 256 / VPR threads that share them are added in
            // thread order
            constexpr int VPR = BN / VEB;
            static_assert(256 % VPR == 0 && 256 * VEB * 4 <= SMEM_BYTES, "column-sum staging");
            float *red = reinterpret_cast<float *>(smem);
#pragma unroll
            for (int e = 0; e < VEB; ++e) red[threadIdx.x * VEB + e] = cs[e];
            __syncthreads();
            if (threadIdx.x < BN) {
                const int cv = threadIdx.x / VEB, e = threadIdx.x % VEB;
                float t = 0.0f;
                for (int o = 0; o < 256 / VPR; ++o) t += red[(cv + VPR * o) * VEB + e];
                if (n0 + threadIdx.x < g.N) g.colsum[(int64_t)split * g.N + n0 + threadIdx.x] = t;
            }
            __syncthreads();
        }
    }
    gemm_epilogue<TM, TN>(g, acc, m0 + wm * TM * 32, n0 + wn * TN * 32, l32, h,
                          reinterpret_cast<float *>(smem) + wave * GEMM_STAGE_FLOATS(TN), split);
}

// bf16 weight gradient  C[M, N] (+)= A^T B  with A stored [K][lda] (m contiguous) and B stored [K][ldb]
// (n contiguous): both operands are k-major in memory, while an MFMA fragment wants eight consecutive
// k of one row.  The general kernel above leaves the tiles k-major in LDS and builds every fragment
// from eight 2-byte LDS reads; here a thread loads a 4 (k) x 8 (row) patch (four 16-byte loads),
// transposes it in registers and writes eight 8-byte k-runs, so the tiles sit in LDS as [row][k] and a
// fragment is one 16-byte read (a quarter of the LDS instructions).  The first half of the threads loads
// the A tile, the second half the B tile.  Split over k like k_gemm (partials in g.C when gridDim.z > 1),
// same epilogue, same column-sum by-product.
__device__ inline uint32_t tn_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }   // lo16(a) | lo16(b) << 16
__device__ inline uint32_t tn_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }   // hi16(a) | hi16(b) << 16

// BIG = false: 128 x 128 tile, 4 wavefronts of 64 x 64, k-tile 32.  BIG = true: ONE 256 x 256 tile per
// workgroup, i.e. the whole output of a layer of up to 256 x 256 weights, one workgroup per k-range: every
// element of A and B is then read from memory exactly once (with 128 x 128 tiles each is read by two
// workgroups, on different XCDs, and the product is bound by those reads).  That form runs 16 wavefronts
// of 64 x 64 with a k-tile of 64: the bytes a CU has in flight are the loads its threads hold in
// registers, and 1,024 threads x 64 bytes are what it takes to cover the memory latency (with 8
// wavefronts of 64 x 128 and a k-tile of 32, half as many, the product ran at 4.1 TB/s).
template <bool BIG>
__global__ void __launch_bounds__(BIG ? 1024 : 256) k_gemm_tn_bf16(const GemmArgs g) {
    constexpr int KT = BIG ? 64 : 32, KQ = KT / 4, STR = KT + 8, BM = BIG ? 256 : 128, BN = BM, NT = BIG ? 1024 : 256, HALF = NT / 2;
    constexpr int WN = 2, WGN = BIG ? 4 : 2;                         // 32-column MFMA blocks per wavefront; wavefronts along n
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // max(tiles, output stages): see tn_lds_bytes
    bf16_t *As = reinterpret_cast<bf16_t *>(smem);
    bf16_t *Bs = As + BM * STR;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int wm = wave / WGN, wn = wave % WGN;
    int tile_m, tile_n;
    int split;
    if (!gemm_tile_of_block(g, tile_m, tile_n, split)) return;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int64_t kbeg = (int64_t)split * g.k_per_split;
    const int64_t kend = (kbeg + g.k_per_split < g.K) ? kbeg + g.k_per_split : g.K;

    // this thread's patch: operand (first half of the threads: A, second half: B), k-group (4 k), row
    // group (8 rows of the tile)
    const bool isB = threadIdx.x >= HALF;
    const int t = threadIdx.x & (HALF - 1), kq = t % KQ, rq = t / KQ;
    const bf16_t *P = static_cast<const bf16_t *>(isB ? g.B : g.A);
    const int64_t ld = isB ? g.ldb : g.lda;
    const int64_t c0 = (isB ? n0 : m0) + rq * 8;              // first row (column of the stored matrix) of the patch
    const int64_t clim = isB ? g.N : g.M;
    const int nv = c0 >= clim ? 0 : (int)((clim - c0) < 8 ? (clim - c0) : 8);
    bf16_t *dst = (isB ? Bs : As) + rq * 8 * STR + kq * 4;

    floatx16 acc[2][WN];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < WN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
    const bool do_cs = g.colsum && tile_m == 0 && isB;
    float cs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[e] = 0.0f;

    // One register stage: the loads of the next k-tile are in flight while a tile is multiplied.
    uint4 r[1][4];
    bool rok[1][4];
    const bf16_t *src = P + (kbeg + kq * 4) * ld + c0;   // this thread's patch of the tile at k0; only read where ok
    auto fetch = [&](uint4 (&rr)[4], bool (&ok)[4], int64_t k0) {
#pragma unroll
        for (int dk = 0; dk < 4; ++dk) {
            ok[dk] = k0 + kq * 4 + dk < kend && nv > 0;
            rr[dk] = *reinterpret_cast<const uint4 *>(ok[dk] ? src + dk * ld : P);   // branch free: masked at the store
        }
        src += KT * ld;
    };
    auto consume = [&](const uint4 (&rr)[4], const bool (&ok)[4]) {   // registers -> LDS, transposed
        uint32_t w[4][4];
#pragma unroll
        for (int dk = 0; dk < 4; ++dk) {
            uint4 v = rr[dk];
            const int n = ok[dk] ? nv : 0;
            v.x &= n >= 2 ? 0xffffffffu : (n == 1 ? 0x0000ffffu : 0u);
            v.y &= n >= 4 ? 0xffffffffu : (n == 3 ? 0x0000ffffu : 0u);
            v.z &= n >= 6 ? 0xffffffffu : (n == 5 ? 0x0000ffffu : 0u);
            v.w &= n >= 8 ? 0xffffffffu : (n == 7 ? 0x0000ffffu : 0u);
            w[dk][0] = v.x; w[dk][1] = v.y; w[dk][2] = v.z; w[dk][3] = v.w;
        }
        if (do_cs) {
#pragma unroll
            for (int dk = 0; dk < 4; ++dk)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    cs[2 * c] += __uint_as_float(w[dk][c] << 16);
                    cs[2 * c + 1] += __uint_as_float(w[dk][c] & 0xffff0000u);
                }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {   // rows 2c and 2c + 1 of the patch: their four k as one 8-byte run each
            *reinterpret_cast<uint2 *>(dst + (2 * c) * STR) = make_uint2(tn_lo(w[0][c], w[1][c]), tn_lo(w[2][c], w[3][c]));
            *reinterpret_cast<uint2 *>(dst + (2 * c + 1) * STR) = make_uint2(tn_hi(w[0][c], w[1][c]), tn_hi(w[2][c], w[3][c]));
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int s = 0; s < KT / 16; ++s) {
            const int kk = s * 16 + h * 8;   // lane half h supplies k = kk .. kk + 7 of this step
            bf16x8 af[2], bfr[WN];
#pragma unroll
            for (int a = 0; a < 2; ++a) af[a] = *reinterpret_cast<const bf16x8 *>(&As[((wm * 2 + a) * 32 + l32) * STR + kk]);
#pragma unroll
            for (int b = 0; b < WN; ++b) bfr[b] = *reinterpret_cast<const bf16x8 *>(&Bs[((wn * WN + b) * 32 + l32) * STR + kk]);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < WN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    };
    if (kbeg < kend) fetch(r[0], rok[0], kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += KT) {
        __syncthreads();   // previous tile fully consumed
        consume(r[0], rok[0]);
        __syncthreads();
        if (k0 + KT < kend) fetch(r[0], rok[0], k0 + KT);
        multiply();
    }
    __syncthreads();   // every wavefront is done reading the operand tiles
    if (g.colsum && tile_m == 0) {   // uniform over the workgroup
        // B thread (rq, kq) holds columns 8 rq .. + 7; the KQ k-groups that share them are added in order
        float *red = reinterpret_cast<float *>(smem);
        if (isB) {
#pragma unroll
            for (int e = 0; e < 8; ++e) red[t * 8 + e] = cs[e];
        }
        __syncthreads();
        if (threadIdx.x < BN) {
            const int q = threadIdx.x >> 3, e = threadIdx.x & 7;
            float sum = 0.0f;
            for (int k = 0; k < KQ; ++k) sum += red[(q * KQ + k) * 8 + e];
            if (n0 + threadIdx.x < g.N) g.colsum[(int64_t)split * g.N + n0 + threadIdx.x] = sum;
        }
        __syncthreads();
    }
    float *stage = reinterpret_cast<float *>(smem) + wave * GEMM_STAGE_FLOATS(2);
    gemm_epilogue<2, 2>(g, acc, m0 + wm * 64, n0 + wn * 64, l32, h, stage, split);
}
template <bool BIG>
constexpr size_t tn_lds_bytes() {
    constexpr size_t tiles = (size_t)(BIG ? 512 * 72 : 256 * 40) * 2, stages = (size_t)(BIG ? 16 : 4) * GEMM_STAGE_FLOATS(2) * 4;
    return tiles > stages ? tiles : stages;
}

// C = act(sum_z P[z] + C_in + bias), partials added in z order
__global__ void __launch_bounds__(256) k_splitk_reduce(const float *P, int splits, int64_t M, int64_t N, void *C,
                                                       int64_t ldc, const void *Cin, int64_t ldcin, const float *bias,
                                                       const float *rowscale, int relu, int c_bf16) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t row = idx / N, col = idx % N;
    float v = 0.0f;
    const int64_t stride = M * N;
    int z = 0;
    for (; z + 8 <= splits; z += 8) {   // eight independent loads in flight, added in z order
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = P[(int64_t)(z + u) * stride + idx];
#pragma unroll
        for (int u = 0; u < 8; ++u) v += t[u];
    }
    for (; z < splits; ++z) v += P[(int64_t)z * stride + idx];
    if (rowscale) v *= rowscale[row];
    if (Cin) v += c_bf16 ? bf16_to_f32(static_cast<const bf16_t *>(Cin)[row * ldcin + col])
                         : static_cast<const float *>(Cin)[row * ldcin + col];
    if (bias) v += bias[col];
    if (relu) v = v > 0.0f ? v : 0.0f;
    if (c_bf16) static_cast<bf16_t *>(C)[row * ldc + col] = (bf16_t)f32_to_bf16(v);
    else static_cast<float *>(C)[row * ldc + col] = v;
}

// The same for many splits: eight lanes per output element, lane l adds the partials l, l + 8, ... (four
// loads in flight), the eight sums are then added in lane order.  A fixed order again, and the chain of
// dependent additions is an eighth as long (256 splits of a 64 x 64 output: one thread per element
// walked 32 rounds of loads one after the other).
__global__ void __launch_bounds__(256) k_splitk_reduce8(const float *P, int splits, int64_t M, int64_t N, void *C,
                                                        int64_t ldc, const void *Cin, int64_t ldcin, const float *bias,
                                                        const float *rowscale, int relu, int c_bf16) {
    const int l = threadIdx.x & 7;
    const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 3;
    const bool live = idx < M * N;
    const int64_t stride = M * N;
    float v = 0.0f;
    if (live) {
        int z = l;
        for (; z + 24 < splits; z += 32) {
            float t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = P[(int64_t)(z + 8 * u) * stride + idx];
#pragma unroll
            for (int u = 0; u < 4; ++u) v += t[u];
        }
        for (; z < splits; z += 8) v += P[(int64_t)z * stride + idx];
    }
    float tot = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) tot += __shfl(v, k, 8);
    if (!live || l != 0) return;
    const int64_t row = idx / N, col = idx % N;
    v = tot;
    if (rowscale) v *= rowscale[row];
    if (Cin) v += c_bf16 ? bf16_to_f32(static_cast<const bf16_t *>(Cin)[row * ldcin + col])
                         : static_cast<const float *>(Cin)[row * ldcin + col];
    if (bias) v += bias[col];
    if (relu) v = v > 0.0f ? v : 0.0f;
    if (c_bf16) static_cast<bf16_t *>(C)[row * ldc + col] = (bf16_t)f32_to_bf16(v);
    else static_cast<float *>(C)[row * ldc + col] = v;
}

// Workgroup tile.  Products with little work and so few 256- or 128-row tiles that most compute
// units would idle (the layers of a sampled batch: a thousand rows, a 256 x 47 weight gradient) use
// 64 x 64 tiles, one MFMA block per wavefront, and cut the reduction finer; they are bound by the
// latency of one workgroup's k-loop, not by bytes or flops.
struct TileShape { int64_t bm, bn; bool small; };

TileShape pick_tile(int64_t M, int64_t N, int64_t K) {
    const int64_t bn = N <= 32 ? 32 : (N <= 64 ? 64 : 128);
    const int64_t bm = bn == 128 ? 128 : 256;
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    const bool little = (double)M * (double)N * (double)K < 268435456.0;
    if (little && tiles < 32) return TileShape{64, 64, true};
    return TileShape{bm, bn, false};
}

// fp32 products with enough work to be bound by matrix throughput go through the split-bf16 kernel
// (3/8 of the fp32 MFMA cost at fp32-level accuracy): 128 x 128 tiles in general, 256 x 64 tiles for
// outputs of 33..64 columns (a sampled block's 91 K x 602 -> 64 product: 111 -> 80 us; the plain kernel's
// 357 tiles of slow fp32 MFMA, four wavefronts each, passed over the 1,024 SIMDs twice), 64 x 256 tiles
// for outputs of at most 64 rows (32 x 256 for at most 32).  Narrower outputs keep the plain fp32 MFMA
// (256 x 32 tiles), except weight gradients: a small one (at most 256 x 64 outputs over a long reduction),
// where the plain kernel's tile is mostly padding and the slow fp32 MFMA makes that padding the bottleneck
// (config 2, 128 x 41: 0.093 -> 0.06 ms), and one of at most 32 columns under at least 256 rows over a
// long reduction (256 x 32 split-bf16 tiles; 1024 x 16 over 2^20 rows: 0.87 -> 0.85 ms).
bool use_x3(gt_dtype dtype, int transA, int64_t M, int64_t N, int64_t K) {
    const bool big = (double)M * (double)N * (double)K >= 268435456.0;
    return dtype == GT_F32 && K >= 64 && big && (N > 32 || (transA && N >= 32 && M <= 256) || (transA && M >= 256 && K >= 8192));
}

struct SplitPlan { int splits; int64_t k_per_split; };

// bf16 weight gradients of up to 256 x 256 outputs over a long reduction: one 256 x 256 tile per workgroup
// (k_gemm_tn_bf16<true>), one workgroup per CU
bool tn256_shape(int transA, int transB, int64_t M, int64_t N, int64_t K) {
    return transA && !transB && M > 64 && M <= 256 && N > 64 && N <= 256 && K >= 8192 &&
           (double)M * (double)N * (double)K >= 268435456.0;
}

SplitPlan plan_split(int transA, int64_t M, int64_t N, int64_t K, bool x3, bool tn256 = false) {
    TileShape t = pick_tile(M, N, K);
    if (x3) { gt_gemm_x3_tile(M, N, &t.bm, &t.bn); t.small = false; }
    if (tn256) {
        SplitPlan p{1, (K + KT - 1) / KT * KT};
        int64_t want = 256, max_by_len = K / (4 * KT);
        if (want > max_by_len) want = max_by_len;
        if (want < 1) want = 1;
        const int64_t kps = ((K + want - 1) / want + KT - 1) / KT * KT;
        p.splits = (int)((K + kps - 1) / kps);
        p.k_per_split = kps;
        return p;
    }
    const int64_t tiles = ((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
    SplitPlan p{1, (K + KT - 1) / KT * KT};
    if (K <= 0) { p.k_per_split = KT; return p; }
    int64_t want, max_by_len;
    if (t.small) {
        if (tiles >= 128 || K < 2 * KT) return p;
        want = 256 / tiles;                                   // about one workgroup per CU, all resident at once
        max_by_len = K / KT;                                  // at least one 64-wide k-range per split
    } else {
        // The reduction is cut when the output has too few tiles to fill the chip: the weight-gradient
        // shape (very long K), and a tall product over a very wide feature row with few rows
        if (tiles >= 256 || K < 8 * KT) return p;
        if (!transA && (tiles >= 128 || K < 1024)) return p;
        // two workgroups per CU, and never more blocks than those 512 places: the blocks of a split
        // reduction all run equally long, so a few left over once the places are full double the kernel's
        // time (5 tiles x 103 ranges = 515 blocks took 0.31 ms, 5 x 102 = 510 take 0.17 ms)
        // (three per CU for the 128 x 64 tile of the split-bf16 kernel: 46 KB of LDS, 134 registers)
        want = ((x3 && t.bm == 128 && t.bn == 64) ? 768 : 512) / tiles;
        max_by_len = K / (4 * KT);                            // at least 4 k-tiles per split
    }
    if (want > max_by_len) want = max_by_len;
    if (want < 1) want = 1;
    if (tiles > 1 && want >= 16) want = want / 8 * 8;        // whole k-ranges per XCD (gemm_split_xcd)
    int64_t kps = ((K + want - 1) / want + KT - 1) / KT * KT;
    p.splits = (int)((K + kps - 1) / kps);
    p.k_per_split = kps;
    return p;
}

template <typename T, bool TA, bool TB>
gt_status launch_gemm(GemmArgs g, int splits, hipStream_t st) {
    const TileShape t = pick_tile(g.M, g.N, g.K);
    const int64_t bn = t.bn, bm = t.bm;
    g.ntn = (int)((g.N + bn - 1) / bn);
    g.ntm = (int)((g.M + bm - 1) / bm);
    dim3 grid(gemm_grid_x(g.ntm, g.ntn), 1, (unsigned)splits);
    g.split_xcd = gemm_split_xcd(g.ntm, g.ntn, splits);
    if constexpr (sizeof(T) == 2 && TA && !TB) {
        // the weight-gradient shape in bf16 with 128 x 128 tiles: transposing loads (see k_gemm_tn_bf16)
        if (!t.small && bn == 128 && g.vecA && g.vecB) {
            k_gemm_tn_bf16<false><<<grid, 256, tn_lds_bytes<false>(), st>>>(g);
            GT_LAUNCH_CHECK("k_gemm_tn_bf16");
            return GT_OK;
        }
    }
#define GT_GEMM_CFG(VA_, VB_)                                                                         \
    do {                                                                                             \
        if (t.small) k_gemm<T, TA, TB, 2, 2, 1, 1, VA_, VB_><<<grid, 256, 0, st>>>(g);               \
        else if (bn == 128) k_gemm<T, TA, TB, 2, 2, 2, 2, VA_, VB_><<<grid, 256, 0, st>>>(g);        \
        else if (bn == 64) k_gemm<T, TA, TB, 4, 1, 2, 2, VA_, VB_><<<grid, 256, 0, st>>>(g);         \
        else k_gemm<T, TA, TB, 4, 1, 2, 1, VA_, VB_><<<grid, 256, 0, st>>>(g);                       \
    } while (0)
    if (g.vecA && g.vecB) GT_GEMM_CFG(true, true);
    else if (g.vecA) GT_GEMM_CFG(true, false);
    else if (g.vecB) GT_GEMM_CFG(false, true);
    else GT_GEMM_CFG(false, false);
#undef GT_GEMM_CFG
    GT_LAUNCH_CHECK("k_gemm");
    return GT_OK;
}

gt_status launch_tn256(GemmArgs g, int splits, hipStream_t st) {
    g.ntm = 1; g.ntn = 1;
    constexpr size_t lds = tn_lds_bytes<true>();
    GT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_tn_bf16<true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    k_gemm_tn_bf16<true><<<dim3(1, 1, (unsigned)splits), 1024, lds, st>>>(g);
    GT_LAUNCH_CHECK("k_gemm_tn_bf16");
    return GT_OK;
}

template <typename T>
gt_status launch_gemm_t(const GemmArgs &g, int transA, int transB, int splits, hipStream_t st) {
    if (!transA && !transB) return launch_gemm<T, false, false>(g, splits, st);
    if (!transA && transB) return launch_gemm<T, false, true>(g, splits, st);
    if (transA && !transB) return launch_gemm<T, true, false>(g, splits, st);
    return launch_gemm<T, true, true>(g, splits, st);
}

}  // namespace

// the data type is not known here: the larger of the two plans
size_t gt_gemm_ws_bytes(int transA, int64_t M, int64_t N, int64_t K) {
    const SplitPlan p = plan_split(transA, M, N, K, false);
    const SplitPlan q = plan_split(transA, M, N, K, use_x3(GT_F32, transA, M, N, K));
    int splits = p.splits > q.splits ? p.splits : q.splits;
    if (tn256_shape(transA, 0, M, N, K)) {
        const SplitPlan r = plan_split(transA, M, N, K, false, true);
        if (r.splits > splits) splits = r.splits;
    }
    // partial tiles of a split reduction, plus (weight-gradient shape) room for the column sums of B per split
    return (splits > 1 ? gt_align_up((size_t)splits * (size_t)M * (size_t)N * 4) : 0) +
           (transA ? gt_align_up((size_t)splits * (size_t)N * 4) : 0);
}

// out[c] = sum over the splits' column sums: 4 columns per workgroup, 64 lanes per column stride over
// the splits, the lanes' sums are added in lane order (fixed order; a single thread per column walking
// a few hundred splits one after the other took 0.1 ms)
__global__ void __launch_bounds__(256) k_colsum_splits(const float *partial, int splits, int64_t cols, float *out) {
    __shared__ float red[256];
    const int cl = threadIdx.x & 3, rl = threadIdx.x >> 2;
    const int64_t c = (int64_t)blockIdx.x * 4 + cl;
    float s = 0.0f;
    if (c < cols)
        for (int z = rl; z < splits; z += 64) s += partial[(int64_t)z * cols + c];
    red[threadIdx.x] = s;
    __syncthreads();
    if (rl == 0 && c < cols) {
        float t = 0.0f;
        for (int k = 0; k < 64; ++k) t += red[k * 4 + cl];
        out[c] = t;
    }
}

gt_status gt_gemm_run(const char *fn, gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, const void *B, int64_t ldb, const float *bias, const float *rowscale,
                      gt_act act, const void *Cin, int64_t ldcin, void *C, int64_t ldc, gt_dtype c_dtype, void *ws,
                      size_t ws_bytes, hipStream_t st, const void *mask, int64_t ldmask, float *colsum_b, bool pad_c) {
    if (dtype != GT_F32 && dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown dtype", fn);
    if (mask && ldmask < N) return gt_fail(GT_ERR_INVALID_ARG, "%s: mask leading dimension too small", fn);
    if (c_dtype != GT_F32 && c_dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown c_dtype", fn);
    if (M < 0 || N < 0 || K < 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: negative size", fn);
    if (M == 0 || N == 0) return GT_OK;
    if (!C) return gt_fail(GT_ERR_INVALID_ARG, "%s: C is null", fn);
    if (K > 0 && (!A || !B)) return gt_fail(GT_ERR_INVALID_ARG, "%s: A or B is null", fn);
    if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N || (Cin && ldcin < N))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension too small", fn);
    const size_t es = gt_dtype_size(dtype), cs = gt_dtype_size(c_dtype);
    if (((uintptr_t)A % es) || ((uintptr_t)B % es) || ((uintptr_t)C % cs) || ((uintptr_t)Cin % cs))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: pointer misaligned for dtype", fn);
    const bool x3 = use_x3(dtype, transA, M, N, K);
    const int ve0 = dtype == GT_BF16 ? 8 : 4;
    const bool tn256 = dtype == GT_BF16 && tn256_shape(transA, transB, M, N, K) && ((uintptr_t)A & 15) == 0 &&
                       ((uintptr_t)B & 15) == 0 && lda % ve0 == 0 && ldb % ve0 == 0;
    const SplitPlan p = plan_split(transA, M, N, K, x3, tn256);
    if (colsum_b && (!transA || transB)) return gt_fail(GT_ERR_INTERNAL, "%s: column sums of B need the A^T B shape", fn);
    const size_t need_part = p.splits > 1 ? gt_align_up((size_t)p.splits * (size_t)M * (size_t)N * 4) : 0;
    const size_t need = need_part + (colsum_b ? gt_align_up((size_t)p.splits * (size_t)N * 4) : 0);
    if (need) {
        if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: ws null or not 256-byte aligned", fn);
        if (ws_bytes < need) return gt_fail(GT_ERR_WORKSPACE, "%s: ws_bytes %zu < required %zu", fn, ws_bytes, need);
    }
    const int ve = dtype == GT_BF16 ? 8 : 4;
    GemmArgs g{};
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb;
    g.M = M; g.N = N; g.K = K;
    g.k_per_split = p.k_per_split;
    g.vecA = (((uintptr_t)A & 15) == 0 && lda % ve == 0);
    g.vecB = (((uintptr_t)B & 15) == 0 && ldb % ve == 0);
    g.bias = bias; g.rowscale = rowscale; g.relu = (act == GT_ACT_RELU); g.c_bf16 = (c_dtype == GT_BF16);
    g.Cin = Cin; g.ldcin = ldcin;
    g.mask = mask; g.ldmask = ldmask;
    g.pad_c = pad_c ? 1 : 0;
    g.colsum = colsum_b ? reinterpret_cast<float *>(static_cast<char *>(ws) + need_part) : nullptr;
    if (mask && p.splits > 1) return gt_fail(GT_ERR_INTERNAL, "%s: an output mask on a split reduction", fn);
    if (p.splits > 1) { g.C = ws; g.ldc = N; } else { g.C = C; g.ldc = ldc; }
    const int tr = gt_trace_open(GT_TRACE_COMBINE, N, M, M * N * K, st);
    // tall products with a small weight matrix are bound by streaming A and C once: the
    // weight-stationary kernel does exactly that
    const bool ws_path = p.splits == 1 && c_dtype == dtype && !Cin && !rowscale &&
                         gt_gemm_ws_applicable(dtype, transA, M, N, K, g.vecA);
    gt_status s = ws_path ? gt_gemm_ws_launch(g, dtype, transB, st)
                  : tn256 ? launch_tn256(g, p.splits, st)
                  : x3 ? gt_gemm_x3_launch(g, transA, transB, p.splits, st)
                       : (dtype == GT_F32) ? launch_gemm_t<float>(g, transA, transB, p.splits, st)
                                           : launch_gemm_t<bf16_t>(g, transA, transB, p.splits, st);
    gt_trace_close(tr, st);
    if (s != GT_OK) return s;
    if (p.splits > 1) {
        const int64_t n = M * N;
        if (p.splits >= 64)
            k_splitk_reduce8<<<(unsigned)((n * 8 + 255) / 256), 256, 0, st>>>(static_cast<const float *>(ws), p.splits, M, N,
                                                                            C, ldc, Cin, ldcin, bias, rowscale, g.relu,
                                                                            g.c_bf16);
        else
            k_splitk_reduce<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(static_cast<const float *>(ws), p.splits, M, N, C,
                                                                         ldc, Cin, ldcin, bias, rowscale, g.relu, g.c_bf16);
        GT_LAUNCH_CHECK("k_splitk_reduce");
    }
    if (colsum_b) {
        k_colsum_splits<<<(unsigned)((N + 3) / 4), 256, 0, st>>>(g.colsum, p.splits, N, colsum_b);
        GT_LAUNCH_CHECK("k_colsum_splits");
    }
    return GT_OK;
}

extern "C" gt_status gt_combine_ws_size(gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                                        size_t *ws_bytes) {
    (void)dtype; (void)transB;
    if (!ws_bytes) return gt_fail(GT_ERR_INVALID_ARG, "gt_combine_ws_size: ws_bytes is null");
    if (M < 0 || N < 0 || K < 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_combine_ws_size: negative size");
    *ws_bytes = gt_gemm_ws_bytes(transA, M, N, K);
    return GT_OK;
}

extern "C" gt_status gt_combine(gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K, const void *A,
                                int64_t lda, const void *B, int64_t ldb, const float *bias, gt_act act, void *C,
                                int64_t ldc, gt_dtype c_dtype, void *ws, size_t ws_bytes, void *stream) {
    if (act != GT_ACT_NONE && act != GT_ACT_RELU) return gt_fail(GT_ERR_INVALID_ARG, "gt_combine: unknown activation");
    return gt_gemm_run("gt_combine", dtype, transA != 0, transB != 0, M, N, K, A, lda, B, ldb, bias, nullptr, act,
                       nullptr, 0, C, ldc, c_dtype, ws, ws_bytes, (hipStream_t)stream);
}
