// fp32 combination on the bf16 matrix cores by exact three-way splitting.
//
// Every fp32 operand element x is cut into three bf16 pieces by truncation, x = hi + mid + lo
// exactly (8 + 8 + 8 significand bits; the residuals x - hi and x - hi - mid are exact in fp32).
// A product a*b is then the sum of nine bf16 x bf16 products, each exact in fp32; the six
// largest (hi*hi, hi*mid, mid*hi, hi*lo, lo*hi, mid*mid) are accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16 and the three dropped ones are below 2^-24 of |a*b|, i.e. at the
// level of fp32 rounding itself.  On CDNA4 the bf16 MFMA rate is 16x the fp32 MFMA rate, so six
// bf16 instructions per product block cost 3/8 of the fp32 instruction they replace.  Used for
// the shapes of the combination that are bound by matrix throughput (wide K and N); the skinny,
// memory-bound shapes stay on the plain fp32 MFMA kernel.
//
// Layout: 4 wavefronts, in general 64 x 64 accumulators each on a 128 x 128 workgroup tile (other
// tiles: see x3_lds_bytes), k-tile 32.  Both
// operands are converted and split while they are stored to LDS, k-contiguous per row
// ([row][k], three planes), so every MFMA fragment is one ds_read_b128.  Operands whose global
// layout is k-major (the weight matrix, both operands of the weight gradient) are transposed on
// the way in registers: a thread loads a 4(k) x 4(row) patch and writes four 8-byte k-runs.
#include <type_traits>

#include "gt_internal.h"
#include "gt_combine.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int KT = GEMM_KT;          // 32
constexpr int STR = KT + 8;          // LDS row stride in bf16 elements (80 bytes: 16-byte aligned, bank friendly)

// Three truncated bf16 pieces of x: x == hi + mid + lo exactly (barring underflow).  The pieces are
// returned as fp32 bit patterns whose upper halves are the bf16 values (the lower halves of `hi`
// and `lo` are not cleared: only the upper halves are ever used).
__device__ inline void split3(float x, uint32_t &hi, uint32_t &mid, uint32_t &lo) {
    const uint32_t h = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(h);
    const uint32_t m = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(m);
    hi = h; mid = m; lo = __float_as_uint(r2);
}

// upper halves of two words as one word: (b & 0xffff0000) | (a >> 16), one v_perm_b32
__device__ inline uint32_t pack_hi16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// four consecutive-k values -> three 8-byte k-runs (one per plane) at lds[plane][row][k]
template <int PLANE>
__device__ inline void store_run4(gemm_bf16_t *lds, int row, int k, float x0, float x1, float x2, float x3) {
    uint32_t h[4], m[4], l[4];
    split3(x0, h[0], m[0], l[0]);
    split3(x1, h[1], m[1], l[1]);
    split3(x2, h[2], m[2], l[2]);
    split3(x3, h[3], m[3], l[3]);
    gemm_bf16_t *p = lds + row * STR + k;
    *reinterpret_cast<uint2 *>(p) = make_uint2(pack_hi16(h[0], h[1]), pack_hi16(h[2], h[3]));
    *reinterpret_cast<uint2 *>(p + PLANE) = make_uint2(pack_hi16(m[0], m[1]), pack_hi16(m[2], m[3]));
    *reinterpret_cast<uint2 *>(p + 2 * PLANE) = make_uint2(pack_hi16(l[0], l[1]), pack_hi16(l[2], l[3]));
}

// Four consecutive elements at p[off..off+3] (position c of a row that ends at clim).  Branch
// free: an out-of-range request reads the (always valid) start of the matrix; `nv` receives the
// number of elements that are real, and mask4 zeroes the rest when the data is consumed (masking at
// load time would wait for the data and stall the prefetch).  `vec` is grid-uniform.
__device__ inline float4 load4(const float *p, int64_t off, int64_t c, int64_t clim, bool row_ok, int vec, int &nv) {
    const bool ok = row_ok && c < clim;
    nv = ok ? (int)((clim - c) < 4 ? (clim - c) : 4) : 0;
    float4 v;
    if (vec) {
        v = *reinterpret_cast<const float4 *>(p + (ok ? off : 0));
    } else {
        v.x = p[nv > 0 ? off : 0];
        v.y = p[nv > 1 ? off + 1 : 0];
        v.z = p[nv > 2 ? off + 2 : 0];
        v.w = p[nv > 3 ? off + 3 : 0];
    }
    return v;
}
__device__ inline float4 mask4(float4 v, int nv) {
    v.x = nv > 0 ? v.x : 0.0f;
    v.y = nv > 1 ? v.y : 0.0f;
    v.z = nv > 2 ? v.z : 0.0f;
    v.w = nv > 3 ? v.w : 0.0f;
    return v;
}

// ROWS rows x 32 k of an operand whose k direction is contiguous in memory: element (i, k) at
// p[(i0 + i) * ld + k0 + k].  ROWS / 32 float4 per thread, lanes run along k first.
template <int ROWS>
struct LoadKC {
    static constexpr int NV = ROWS / 32;
    static constexpr int PLANE = ROWS * STR;
    float4 r[NV];
    int nv[NV];
    __device__ inline void load(const float *p, int64_t ld, int64_t i0, int64_t k0, int64_t ilim, int64_t klim, int vec) {
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int u = threadIdx.x + 256 * it;
            const int i = u >> 3, kq = u & 7;
            const int64_t gi = i0 + i, gk = k0 + kq * 4;
            r[it] = load4(p, gi * ld + gk, gk, klim, gi < ilim, vec, nv[it]);
        }
    }
    __device__ inline void store(gemm_bf16_t *lds) const {
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int u = threadIdx.x + 256 * it;
            const float4 v = mask4(r[it], nv[it]);
            store_run4<PLANE>(lds, u >> 3, (u & 7) * 4, v.x, v.y, v.z, v.w);
        }
    }
};

// 32 k x ROWS rows of an operand whose row direction is contiguous in memory: element (i, k) at
// p[(k0 + k) * ld + i0 + i].  4(k) x 4(i) patches, transposed in registers: one patch per thread
// covers 128 rows (ROWS = 256: two patches; ROWS = 64: the upper half of the threads has none).
template <int ROWS>
struct LoadKM {
    static constexpr int NPATCH = ROWS > 128 ? ROWS / 128 : 1;
    static constexpr int PLANE = ROWS * STR;
    float4 r[NPATCH][4];   // r[q][dk] = rows i..i+3 at k + dk
    int nv[NPATCH][4];
    __device__ inline void load(const float *p, int64_t ld, int64_t i0, int64_t k0, int64_t ilim, int64_t klim, int vec) {
        const int kq = threadIdx.x & 7;
#pragma unroll
        for (int q = 0; q < NPATCH; ++q) {
            const int iq = (threadIdx.x >> 3) + 32 * q;
            const bool mine = iq * 4 < ROWS;
#pragma unroll
            for (int dk = 0; dk < 4; ++dk) {
                const int64_t gk = k0 + kq * 4 + dk, gi = i0 + iq * 4;
                r[q][dk] = load4(p, gk * ld + gi, gi, ilim, mine && gk < klim, vec, nv[q][dk]);
            }
        }
    }
    // adds this thread's (masked) elements to cs[q][0..3]: rows 4 iq .. + 3 of patch q, summed over its four k
    __device__ inline void add_to(float (&cs)[NPATCH][4]) const {
#pragma unroll
        for (int q = 0; q < NPATCH; ++q)
#pragma unroll
            for (int dk = 0; dk < 4; ++dk) {
                const float4 v = mask4(r[q][dk], nv[q][dk]);
                cs[q][0] += v.x; cs[q][1] += v.y; cs[q][2] += v.z; cs[q][3] += v.w;
            }
    }
    __device__ inline void store(gemm_bf16_t *lds) const {
        const int kq = threadIdx.x & 7;
#pragma unroll
        for (int q = 0; q < NPATCH; ++q) {
            const int iq = (threadIdx.x >> 3) + 32 * q;
            if (iq * 4 >= ROWS) continue;
            const float4 a = mask4(r[q][0], nv[q][0]), b = mask4(r[q][1], nv[q][1]), c = mask4(r[q][2], nv[q][2]),
                         d = mask4(r[q][3], nv[q][3]);
            store_run4<PLANE>(lds, iq * 4 + 0, kq * 4, a.x, b.x, c.x, d.x);
            store_run4<PLANE>(lds, iq * 4 + 1, kq * 4, a.y, b.y, c.y, d.y);
            store_run4<PLANE>(lds, iq * 4 + 2, kq * 4, a.z, b.z, c.z, d.z);
            store_run4<PLANE>(lds, iq * 4 + 3, kq * 4, a.w, b.w, c.w, d.w);
        }
    }
};

// Workgroup tile: WGM x WGN wavefronts of 64 x 64 accumulators each: 128 x 128 (2 x 2) in general,
// 256 x 64 (4 x 1) for outputs of at most 64 columns, where half of a 128-wide tile would be padding.
// A wavefront holds TMW x TNW blocks of 32 x 32 (2 x 2 in those shapes); 32 x 256 (1 x 4 wavefronts of 1 x 2
// blocks) serves weight gradients with at most 32 rows, whose 64-row tile was three quarters padding.
template <int WGM, int WGN, int TMW, int TNW>
constexpr size_t x3_lds_bytes() {
    constexpr size_t planes = (size_t)3 * (WGM * TMW + WGN * TNW) * 32 * STR * 2, stages = (size_t)4 * GEMM_STAGE_FLOATS(TNW) * 4;
    return planes > stages ? planes : stages;
}

template <bool TA, bool TB, bool VA, bool VB, int WGM, int WGN, int TMW, int TNW>
__global__ void __launch_bounds__(256) k_gemm_x3(const GemmArgs g) {
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int BM = WGM * TMW * 32, BN = WGN * TNW * 32;
    constexpr int PLANE_A = BM * STR, PLANE_B = BN * STR;
    // one LDS buffer: operand planes during the k-loop, the per-wavefront output stages afterwards
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    gemm_bf16_t *smem = reinterpret_cast<gemm_bf16_t *>(smem_raw);
    static_assert(x3_lds_bytes<WGM, WGN, TMW, TNW>() >= 4 * GEMM_STAGE_FLOATS(TNW) * 4, "output stages must fit");
    gemm_bf16_t *As = smem, *Bs = smem + 3 * PLANE_A;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int wm = wave / WGN, wn = wave % WGN;
    int tile_m, tile_n;
    int split;
    if (!gemm_tile_of_block(g, tile_m, tile_n, split)) return;   // whole workgroup leaves before any barrier
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int64_t kbeg = (int64_t)split * g.k_per_split;
    const int64_t kend = (kbeg + g.k_per_split < g.K) ? kbeg + g.k_per_split : g.K;
    const float *A = static_cast<const float *>(g.A);
    const float *B = static_cast<const float *>(g.B);

    floatx16 acc[TMW][TNW];
#pragma unroll
    for (int a = 0; a < TMW; ++a)
#pragma unroll
        for (int b = 0; b < TNW; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    // op(A)(i,k) = TA ? A[k*lda + i] : A[i*lda + k];  op(B)(k,j) = TB ? B[j*ldb + k] : B[k*ldb + j]
    typename std::conditional<TA, LoadKM<BM>, LoadKC<BM>>::type la;
    typename std::conditional<TB, LoadKC<BN>, LoadKM<BN>>::type lb;
    // column sums of op(B) over this workgroup's k-range, a by-product of loading B (row tile 0 only)
    constexpr int NPB = BN > 128 ? BN / 128 : 1;
    const bool do_cs = !TB && g.colsum && tile_m == 0;
    float cs[NPB][4];
#pragma unroll
    for (int q = 0; q < NPB; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[q][e] = 0.0f;
    if (kbeg < kend) {
        la.load(A, g.lda, m0, kbeg, g.M, kend, VA);
        lb.load(B, g.ldb, n0, kbeg, g.N, kend, VB);
    }
    // One register stage: the loads of k-tile t+1 are in flight while tile t is multiplied.  (Two
    // stages were measured slower on MI355X: the extra registers halve the occupancy.)
    for (int64_t k0 = kbeg; k0 < kend; k0 += KT) {
        __syncthreads();
        la.store(As);
        lb.store(Bs);
        if constexpr (!TB) {
            if (do_cs) lb.add_to(cs);
        }
        __syncthreads();
        if (k0 + KT < kend) {
            la.load(A, g.lda, m0, k0 + KT, g.M, kend, VA);
            lb.load(B, g.ldb, n0, k0 + KT, g.N, kend, VB);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int kk = s * 16 + h * 8;   // lane half h supplies k = kk .. kk+7 of this step
            bf16x8 af[TMW][3], bf[TNW][3];
#pragma unroll
            for (int a = 0; a < TMW; ++a) {
                const int i = (wm * TMW + a) * 32 + l32;
#pragma unroll
                for (int p = 0; p < 3; ++p)
                    af[a][p] = *reinterpret_cast<const bf16x8 *>(&As[p * PLANE_A + i * STR + kk]);
            }
#pragma unroll
            for (int b = 0; b < TNW; ++b) {
                const int j = (wn * TNW + b) * 32 + l32;
#pragma unroll
                for (int p = 0; p < 3; ++p)
                    bf[b][p] = *reinterpret_cast<const bf16x8 *>(&Bs[p * PLANE_B + j * STR + kk]);
            }
#pragma unroll
            for (int a = 0; a < TMW; ++a)
#pragma unroll
                for (int b = 0; b < TNW; ++b) {
                    floatx16 c = acc[a][b];
                    // smallest terms first: lo*hi, hi*lo, mid*mid, then mid*hi, hi*mid, then hi*hi
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a][2], bf[b][0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a][0], bf[b][2], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a][1], bf[b][1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a][1], bf[b][0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a][0], bf[b][1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a][0], bf[b][0], c, 0, 0, 0);
                    acc[a][b] = c;
                }
        }
    }
    __syncthreads();   // every wavefront is done reading the operand planes
    if constexpr (!TB) {
        if (do_cs) {   // uniform over the workgroup
            // thread t holds, per patch q, columns 4 ((t >> 3) + 32 q) ..; the eight threads t & 7 that share
            // them (they loaded different k) are added in thread order
            static_assert((size_t)256 * NPB * 4 * 4 <= x3_lds_bytes<WGM, WGN, TMW, TNW>(), "column-sum staging");
            float *red = reinterpret_cast<float *>(smem_raw);
#pragma unroll
            for (int q = 0; q < NPB; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) red[(threadIdx.x * NPB + q) * 4 + e] = cs[q][e];
            __syncthreads();
            for (int j = threadIdx.x; j < BN; j += 256) {
                const int iq = j >> 2, e = j & 3, q = iq >> 5, base = (iq & 31) * 8;
                float t = 0.0f;
                for (int kq = 0; kq < 8; ++kq) t += red[((base + kq) * NPB + q) * 4 + e];
                if (n0 + j < g.N) g.colsum[(int64_t)split * g.N + n0 + j] = t;
            }
            __syncthreads();
        }
    }
    gemm_epilogue<TMW, TNW>(g, acc, m0 + wm * TMW * 32, n0 + wn * TNW * 32, l32, h,
                            reinterpret_cast<float *>(smem_raw) + wave * GEMM_STAGE_FLOATS(TNW), split);
}


template <bool TA, bool TB, bool VA, bool VB, int WGM, int WGN, int TMW, int TNW>
gt_status x3_launch_one(const GemmArgs &g, dim3 grid, hipStream_t st) {
    constexpr size_t lds = x3_lds_bytes<WGM, WGN, TMW, TNW>();
    if (lds > 64 * 1024) {   // host-side setting, no stream operation (also fine under stream capture)
        GT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_x3<TA, TB, VA, VB, WGM, WGN, TMW, TNW>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    }
    k_gemm_x3<TA, TB, VA, VB, WGM, WGN, TMW, TNW><<<grid, 256, lds, st>>>(g);
    GT_LAUNCH_CHECK("k_gemm_x3");
    return GT_OK;
}

template <int WGM, int WGN, int TMW = 2, int TNW = 2>
gt_status x3_launch_shape(const GemmArgs &g_in, int transA, int transB, int splits, hipStream_t st) {
    GemmArgs g = g_in;
    constexpr int BM = WGM * TMW * 32, BN = WGN * TNW * 32;
    g.ntn = (int)((g.N + BN - 1) / BN);
    g.ntm = (int)((g.M + BM - 1) / BM);
    dim3 grid(gemm_grid_x(g.ntm, g.ntn), 1, (unsigned)splits);
    g.split_xcd = gemm_split_xcd(g.ntm, g.ntn, splits);
#define GT_X3(TA_, TB_)                                                                                   \
    do {                                                                                                  \
        if (g.vecA && g.vecB) return x3_launch_one<TA_, TB_, true, true, WGM, WGN, TMW, TNW>(g, grid, st);          \
        else if (g.vecA) return x3_launch_one<TA_, TB_, true, false, WGM, WGN, TMW, TNW>(g, grid, st);              \
        else if (g.vecB) return x3_launch_one<TA_, TB_, false, true, WGM, WGN, TMW, TNW>(g, grid, st);              \
        else return x3_launch_one<TA_, TB_, false, false, WGM, WGN, TMW, TNW>(g, grid, st);                         \
    } while (0)
    if (!transA && !transB) GT_X3(false, false);
    else if (!transA && transB) GT_X3(false, true);
    else if (transA && !transB) GT_X3(true, false);
    else GT_X3(true, true);
#undef GT_X3
}

}  // namespace

// Tile of the split-bf16 kernel for an M x N output: 256 x 64 for at most 64 columns, 64 x 256 for at
// most 64 rows (the weight gradient of a layer with a narrow input: a 128-row tile would be mostly
// padding, and the padding is multiplied like everything else), 128 x 128 otherwise.
// up to this many rows a 256 x 64 tiling leaves the CUs unevenly loaded (fewer than two rounds of tiles)
#define X3_SHORT_ROWS 196608
void gt_gemm_x3_tile(int64_t M, int64_t N, int64_t *bm, int64_t *bn) {
    if (N <= 32) { *bm = 256; *bn = 32; }
    else if (N <= 64 && M <= X3_SHORT_ROWS) { *bm = 128; *bn = 64; }
    else if (N <= 64) { *bm = 256; *bn = 64; }
    else if (M <= 32) { *bm = 32; *bn = 256; }
    else if (M <= 64) { *bm = 64; *bn = 256; }
    else { *bm = 128; *bn = 128; }
}

gt_status gt_gemm_x3_launch(const GemmArgs &g, int transA, int transB, int splits, hipStream_t st) {
    if (g.N <= 32) return x3_launch_shape<4, 1, 2, 1>(g, transA, transB, splits, st);
    if (g.N <= 64 && g.M <= X3_SHORT_ROWS) return x3_launch_shape<4, 1, 1, 2>(g, transA, transB, splits, st);
    if (g.N <= 64) return x3_launch_shape<4, 1>(g, transA, transB, splits, st);
    if (g.M <= 32) return x3_launch_shape<1, 4, 1, 2>(g, transA, transB, splits, st);
    if (g.M <= 64) return x3_launch_shape<1, 4>(g, transA, transB, splits, st);
    return x3_launch_shape<2, 2>(g, transA, transB, splits, st);
}
