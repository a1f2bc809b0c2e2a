// Fused aggregation-first forward:  Y = act( (A X) W + b )  in one kernel.
//
// The paper's Pull keeps the aggregated row of a destination on chip until it is complete
// (Frontend section: the running sum lives in the SM and is written once); here the finished
// row is not written to memory at all: it goes from the gathering lanes' registers into a
// wavefront-private LDS tile, and that tile is the row operand of the combination's MFMA
// (Apply), whose weight matrix sits in LDS for the life of the persistent workgroup.  What is
// saved against the two-kernel path is the write of A X and the combination's read of it; that
// only helps when A X is not needed afterwards (inference: the weight gradient of training reads
// it), and it costs occupancy (one workgroup per CU holds the weights), so the layer call uses it
// only where it measured faster.
//
// Structure (weights and staging as in the weight-stationary combination kernel): persistent
// workgroups of NW wavefronts; the weight matrix is put into LDS once ([n][k], k contiguous,
// zero padded).  Every wavefront then works alone on blocks of 32 work-list entries:
//   gather   G = 8 * NS lanes per entry cover the KP = NS * 128 bytes of a row, 16 bytes per lane,
//            64 / G entries at a time; an entry is a whole-row work item of the plan (its
//            neighbours are gathered and summed in fp32 exactly as the aggregation kernel does) or,
//            after the item list, a split long row (its partial rows, written beforehand by the
//            aggregation kernel over the chunk items, are added in chunk order);
//   stage    the finished row is scaled (mean), rounded to the working type and written to row
//            r of the wavefront's LDS tile [32][KP];
//   multiply the tile times the weights: v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2f32 with the
//            operands swapped (weights first), so a lane ends up with four consecutive output
//            columns per register quadruple;
//   store    bias is the accumulators' start value, ReLU is applied on the way out; rows go to the
//            output rows the entries name (the work list is ordered by row length, not by row).
#include "gt_aggregate_kernel.h"
#include "gt_combine.h"

namespace {

template <typename T> struct FusedGeom;
// V: elements per 16-byte lane load, CK: k per MFMA chunk, HK: k per lane and chunk, SK: k per 128-byte slice
template <> struct FusedGeom<float>  { static constexpr int V = 4, CK = 8,  HK = 4, SK = 32, PAD = 4; };
template <> struct FusedGeom<bf16_t> { static constexpr int V = 8, CK = 16, HK = 8, SK = 64, PAD = 8; };

struct FusedArgs {
    const void *W;       // [K][N] row-major, row stride ldw
    int64_t ldw;
    const float *bias;   // [N] or null
    int relu;
    int64_t N;           // output columns
    int64_t n_entries;   // work items followed by split rows
};

template <typename T, int NB, int NS, int NW>
constexpr size_t fused_lds_bytes() {
    constexpr int KP = NS * FusedGeom<T>::SK, STR = KP + FusedGeom<T>::PAD;
    return (size_t)NB * 32 * STR * sizeof(T) + (size_t)NW * 32 * STR * sizeof(T) + (size_t)NB * 32 * 4 + (size_t)NW * 32 * 4;
}

__device__ inline uint4 pack_row(const float (&v)[8]) {   // fp32 -> bf16 (nearest even), 8 values
    return make_uint4(gt_pack_bf16(v[0], v[1]), gt_pack_bf16(v[2], v[3]),
                      gt_pack_bf16(v[4], v[5]), gt_pack_bf16(v[6], v[7]));
}
__device__ inline uint4 pack_row(const float (&v)[4]) {
    return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
}

// FASTOUT: N is a multiple of the staged width (64 bf16 / 32 fp32 columns) and rows of Y are 16-byte
// aligned: output rows leave through the LDS tile, eight lanes per row, whole 128-byte lines.
template <typename T, int NB, int NS, int NW, bool FASTOUT>
__global__ void __launch_bounds__(NW * 64) k_fused_agg_combine(const AggArgs a, const FusedArgs f) {
    typedef FusedGeom<T> GE;
    constexpr int V = GE::V, CK = GE::CK, HK = GE::HK, SK = GE::SK;
    constexpr int KP = NS * SK, STR = KP + GE::PAD, BN = NB * 32;
    constexpr int G = NS * 8, NG = 64 / G, U = 8;
    typedef typename Raw<T, V>::type raw_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T *Ws = reinterpret_cast<T *>(smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    T *As = reinterpret_cast<T *>(smem + (size_t)BN * STR * sizeof(T)) + (size_t)wave * 32 * STR;
    float *bias_lds = reinterpret_cast<float *>(smem + (size_t)(BN + NW * 32) * STR * sizeof(T));
    int *rowid = reinterpret_cast<int *>(bias_lds + BN) + wave * 32;
    const T *X = static_cast<const T *>(a.X);
    const T *W = static_cast<const T *>(f.W);
    const int64_t K = a.F;

    for (int n = threadIdx.x; n < BN; n += NW * 64) bias_lds[n] = (f.bias && n < f.N) ? f.bias[n] : 0.0f;
    // the weights, once: Ws[n][k] = W[k][n], zero outside (K, N); consecutive threads read consecutive n
    for (int base = threadIdx.x; base < BN * KP; base += NW * 64 * 8) {
        T v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = base + u * NW * 64;
            const int k = idx / BN, n = idx % BN;
            const bool ok = idx < BN * KP && n < f.N && k < K;
            v[u] = W[ok ? (int64_t)k * f.ldw + n : 0];
            if (!ok) v[u] = (T)0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = base + u * NW * 64;
            if (idx < BN * KP) Ws[(idx % BN) * STR + idx / BN] = v[u];
        }
    }
    __syncthreads();   // the only workgroup barrier: wavefronts are on their own from here

    const int gl = lane & (G - 1), grp = lane / G;
    const int64_t col = (int64_t)gl * V;          // this lane's columns of a gathered row
    const bool col_live = col < K;
    const int64_t nblk = (f.n_entries + 31) / 32;
    for (int64_t blk = (int64_t)blockIdx.x * NW + wave; blk < nblk; blk += (int64_t)gridDim.x * NW) {
        __asm__ volatile("" ::: "memory");   // this block's tile writes stay below the previous block's tile reads
        // ---- gather: 32 entries, NG at a time, into the LDS tile
        for (int r = 0; r < 32 / NG; ++r) {
            const int trow = r * NG + grp;
            const int64_t e = blk * 32 + trow;
            float acc[V];
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = 0.0f;
            int out_row = -1;
            if (e < a.n_items) {
                const int4 it = reinterpret_cast<const int4 *>(a.items)[e];
                if (it.w < 0) {          // a whole row (chunk items of split rows were run beforehand)
                    out_row = it.x;
                    const int e0 = it.y, e1 = it.z;
                    // the group fetches G neighbour ids and coefficients at a time with one coalesced
                    // load, the next G being requested before these are used (as the aggregation kernel)
                    int idx_next = 0;
                    float c_next = 0.0f;
                    if (e0 + gl < e1) {
                        idx_next = a.nbr[e0 + gl];
                        c_next = a.coef ? a.coef[e0 + gl] : 1.0f;
                    }
                    for (int base = e0; base < e1; base += G) {
                        const int idx = idx_next;
                        const float c = c_next;
                        const int en = base + G + gl;
                        idx_next = 0;
                        c_next = 0.0f;
                        if (en < e1) {
                            idx_next = a.nbr[en];
                            c_next = a.coef ? a.coef[en] : 1.0f;
                        }
                        const int cnt = (e1 - base) < G ? (e1 - base) : G;
                        for (int j = 0; j < cnt; j += U) {
                            raw_t v[U];
                            float cj[U];
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                const int jj = j + u;
                                const int src = __shfl(idx, jj & (G - 1), G);
                                cj[u] = __shfl(c, jj & (G - 1), G);
                                const bool live = jj < cnt;
                                if (!live) cj[u] = 0.0f;
                                v[u] = raw_t{};
                                if (live && col_live) v[u] = load_raw<T, V>(X + (int64_t)src * a.ldx + col);
                            }
#pragma unroll
                            for (int u = 0; u < U; ++u) fma_raw(acc, cj[u], v[u]);
                        }
                    }
                }
            } else if (e < f.n_entries) {   // a split row: its partial rows in chunk order
                const gt_split s = a.splits[e - a.n_items];
                out_row = s.row;
                for (int k = 0; k < s.count; ++k) {
                    const float *P = a.partials + (int64_t)(s.first + k) * a.ldp + col;
                    if (col_live) {
#pragma unroll
                        for (int q = 0; q < V / 4; ++q) {
                            const float4 x = *reinterpret_cast<const float4 *>(P + 4 * q);
                            acc[4 * q] += x.x; acc[4 * q + 1] += x.y; acc[4 * q + 2] += x.z; acc[4 * q + 3] += x.w;
                        }
                    }
                }
            }
            if (out_row >= 0 && a.post_mode == 2) {   // mean: divide by the row's entry count
                const int d = a.rowptr[out_row + 1] - a.rowptr[out_row];
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = d > 0 ? acc[i] / (float)d : 0.0f;
            }
            // columns at or past K must be exact zeros in the tile (a 16-byte load may have brought in
            // row padding of X or of a partial row, whatever that holds)
#pragma unroll
            for (int i = 0; i < V; ++i)
                if (col + i >= K) acc[i] = 0.0f;
            *reinterpret_cast<uint4 *>(As + trow * STR + col) = pack_row(acc);
            if (gl == 0) rowid[trow] = out_row;
        }
        __asm__ volatile("" ::: "memory");   // LDS operations of a wavefront run in program order
        // ---- multiply the tile by the weights
        floatx16 cacc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 c = *reinterpret_cast<const float4 *>(bias_lds + b * 32 + 8 * q + 4 * h);
                cacc[b][4 * q] = c.x; cacc[b][4 * q + 1] = c.y; cacc[b][4 * q + 2] = c.z; cacc[b][4 * q + 3] = c.w;
            }
        }
#pragma unroll
        for (int kc = 0; kc < KP / CK; ++kc) {
            if ((int64_t)kc * CK >= K) continue;   // uniform: nothing left
            const uint4 av = *reinterpret_cast<const uint4 *>(As + l32 * STR + kc * CK + h * HK);
            const T *wrow = Ws + l32 * STR + kc * CK + h * HK;
            if constexpr (sizeof(T) == 4) {
                const float a0 = __uint_as_float(av.x), a1 = __uint_as_float(av.y), a2 = __uint_as_float(av.z),
                            a3 = __uint_as_float(av.w);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const float4 w = *reinterpret_cast<const float4 *>(wrow + b * 32 * STR);
                    floatx16 cc = cacc[b];
                    cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.x, a0, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.y, a1, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.z, a2, cc, 0, 0, 0);
                    cc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.w, a3, cc, 0, 0, 0);
                    cacc[b] = cc;
                }
            } else {
                bf16x8 af;
                __builtin_memcpy(&af, &av, 16);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const bf16x8 w = *reinterpret_cast<const bf16x8 *>(wrow + b * 32 * STR);
                    cacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, af, cacc[b], 0, 0, 0);
                }
            }
        }
        __asm__ volatile("" ::: "memory");
        // ---- store: register r of lane (h, l32) holds tile row l32, column 8 (r / 4) + 4 h + r % 4 of
        // each 32-column group
        T *Y = static_cast<T *>(a.Y);
        if constexpr (FASTOUT) {
            uint32_t *stage = reinterpret_cast<uint32_t *>(As);   // the tile has been read: 32 x 36 dwords are free
            constexpr int SSTR = 36;
            constexpr int GPS = sizeof(T) == 2 ? 2 : 1;           // 32-column groups per staging round
#pragma unroll
            for (int bp = 0; bp < NB / GPS; ++bp) {
                __asm__ volatile("" ::: "memory");
#pragma unroll
                for (int bb = 0; bb < GPS; ++bb) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float v[4] = {cacc[GPS * bp + bb][4 * q], cacc[GPS * bp + bb][4 * q + 1], cacc[GPS * bp + bb][4 * q + 2],
                                      cacc[GPS * bp + bb][4 * q + 3]};
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = (f.relu && !(v[i] > 0.0f)) ? 0.0f : v[i];
                        if constexpr (sizeof(T) == 2) {
                            *reinterpret_cast<uint2 *>(stage + l32 * SSTR + bb * 16 + 4 * q + 2 * h) =
                                make_uint2(gt_pack_bf16(v[0], v[1]), gt_pack_bf16(v[2], v[3]));
                        } else {
                            *reinterpret_cast<float4 *>(stage + l32 * SSTR + 8 * q + 4 * h) = make_float4(v[0], v[1], v[2], v[3]);
                        }
                    }
                }
                __asm__ volatile("" ::: "memory");
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int rr = it * 8 + (lane >> 3);
                    const uint4 v = *reinterpret_cast<const uint4 *>(stage + rr * SSTR + (lane & 7) * 4);
                    const int row = rowid[rr];
                    if (row >= 0)
                        *reinterpret_cast<uint4 *>(Y + (int64_t)row * a.ldy + bp * (GPS * 32) + (lane & 7) * V) = v;
                }
            }
        } else {
            const int row = rowid[l32];
            if (row >= 0) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int64_t c0 = b * 32 + 8 * q + 4 * h;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            float v = cacc[b][4 * q + i];
                            v = (f.relu && !(v > 0.0f)) ? 0.0f : v;
                            if (c0 + i < f.N) {
                                if constexpr (sizeof(T) == 2) Y[(int64_t)row * a.ldy + c0 + i] = (T)f32_to_bf16(v);
                                else Y[(int64_t)row * a.ldy + c0 + i] = v;
                            }
                        }
                    }
                }
            }
        }
    }
}

template <typename T, int NB, int NS, int NW>
gt_status fused_launch(const AggArgs &a, const FusedArgs &f, hipStream_t st) {
    constexpr size_t lds = fused_lds_bytes<T, NB, NS, NW>();
    constexpr int OW = sizeof(T) == 2 ? 64 : 32;    // columns per staging round of the row-major store
    const int ve = 16 / (int)sizeof(T);
    const bool fast = f.N % OW == 0 && f.N == NB * 32 && a.ldy % ve == 0 && (((uintptr_t)a.Y & 15) == 0);
    const int64_t nblk = (f.n_entries + 31) / 32;
    int64_t gx = (nblk + NW - 1) / NW;
    const int per_cu = lds <= 80 * 1024 ? 2 : 1;
    if (gx > 256 * per_cu) gx = 256 * per_cu;
    if (gx < 1) gx = 1;
#define GT_FUSED_GO(FAST_)                                                                                            \
    do {                                                                                                              \
        if (lds > 64 * 1024)                                                                                          \
            GT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_fused_agg_combine<T, NB, NS, NW, FAST_>),    \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                        \
        k_fused_agg_combine<T, NB, NS, NW, FAST_><<<(unsigned)gx, NW * 64, lds, st>>>(a, f);                          \
    } while (0)
    if (fast) GT_FUSED_GO(true);
    else GT_FUSED_GO(false);
#undef GT_FUSED_GO
    GT_LAUNCH_CHECK("k_fused_agg_combine");
    return GT_OK;
}

// NB from the output width, NS from the input width, NW = 8 wavefronts where the tiles fit, else 4
template <typename T, int NB>
gt_status fused_pick_ns(const AggArgs &a, const FusedArgs &f, hipStream_t st) {
    const int64_t slices = (a.F + FusedGeom<T>::SK - 1) / FusedGeom<T>::SK;
    constexpr size_t cap = 160 * 1024;
#define GT_FUSED_NS(NS_)                                                                          \
    do {                                                                                          \
        if constexpr (fused_lds_bytes<T, NB, NS_, 8>() <= cap) return fused_launch<T, NB, NS_, 8>(a, f, st); \
        else if constexpr (fused_lds_bytes<T, NB, NS_, 4>() <= cap) return fused_launch<T, NB, NS_, 4>(a, f, st); \
        else return gt_fail(GT_ERR_UNSUPPORTED, "gt_aggregate_combine_fwd: weights and tiles exceed the LDS"); \
    } while (0)
    if (slices <= 1) GT_FUSED_NS(1);
    if (slices <= 2) GT_FUSED_NS(2);
    GT_FUSED_NS(4);
#undef GT_FUSED_NS
}

template <typename T>
gt_status fused_pick(const AggArgs &a, const FusedArgs &f, hipStream_t st) {
    if (f.N <= 64) return fused_pick_ns<T, 2>(a, f, st);
    if (f.N <= 128) return fused_pick_ns<T, 4>(a, f, st);
    return fused_pick_ns<T, 8>(a, f, st);
}

size_t fused_lds_for(gt_dtype t, int64_t fi, int64_t fo, int nw) {
    const int es = t == GT_BF16 ? 2 : 4, sk = 128 / es, pad = 16 / es;
    const int64_t slices = (fi + sk - 1) / sk;
    const int ns = slices <= 1 ? 1 : slices <= 2 ? 2 : 4;
    const int nb = fo <= 64 ? 2 : fo <= 128 ? 4 : 8;
    const size_t str = (size_t)ns * sk + pad;
    return (size_t)nb * 32 * str * es + (size_t)nw * 32 * str * es + (size_t)nb * 32 * 4 + (size_t)nw * 32 * 4;
}

}  // namespace

// Shapes the fused kernel takes: input rows of at most four 128-byte slices, at most 256 output
// columns, weights plus at least four row tiles within the 160 KB of LDS, vectorisable rows of X.
bool gt_fused_applicable(gt_dtype dtype, int64_t in_dim, int64_t out_dim) {
    const int64_t kcap = dtype == GT_BF16 ? 256 : 128;
    if (in_dim < 1 || in_dim > kcap || out_dim < 1 || out_dim > 256) return false;
    return fused_lds_for(dtype, in_dim, out_dim, 4) <= 160 * 1024;
}

gt_status gt_fused_run(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t fi, int64_t fo, const void *X, int64_t ldx,
                       const void *W, int64_t ldw, const float *bias, gt_act act, void *Y, int64_t ldy, void *ws,
                       size_t ws_bytes, hipStream_t st) {
    const char *fn = "gt_aggregate_combine_fwd";
    if (!g) return gt_fail(GT_ERR_INVALID_ARG, "%s: g is null", fn);
    if (dtype != GT_F32 && dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown dtype", fn);
    if (reduce != GT_SUM && reduce != GT_MEAN && reduce != GT_SYMNORM) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown reduce", fn);
    if (act != GT_ACT_NONE && act != GT_ACT_RELU) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown activation", fn);
    if (fi <= 0 || fo <= 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: in_dim and out_dim must be positive", fn);
    if (reduce == GT_SYMNORM && g->n_dst != g->n_src) return gt_fail(GT_ERR_UNSUPPORTED, "%s: GT_SYMNORM needs a square graph", fn);
    if (!gt_fused_applicable(dtype, fi, fo))
        return gt_fail(GT_ERR_UNSUPPORTED, "%s: in_dim %lld / out_dim %lld outside what fits on chip", fn, (long long)fi, (long long)fo);
    if (g->n_dst == 0) return GT_OK;
    if (!X || !W || !Y) return gt_fail(GT_ERR_INVALID_ARG, "%s: X, W or Y is null", fn);
    if (ldx < fi || ldy < fo || ldw < fo) return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension too small", fn);
    const size_t es = gt_dtype_size(dtype);
    const int ve = 16 / (int)es;
    if (((uintptr_t)X & 15) || ldx % ve) return gt_fail(GT_ERR_UNSUPPORTED, "%s: rows of X must be 16-byte aligned", fn);
    if (((uintptr_t)W % es) || ((uintptr_t)Y % es)) return gt_fail(GT_ERR_INVALID_ARG, "%s: pointer misaligned for dtype", fn);
    {
        const char *xb = (const char *)X, *xe = xb + (size_t)g->n_src * ldx * es;
        const char *yb = (const char *)Y, *ye = yb + (size_t)g->n_dst * ldy * es;
        if (xb < ye && yb < xe) return gt_fail(GT_ERR_INVALID_ARG, "%s: X and Y overlap", fn);
    }
    const gt_sched &sc = g->fwd;
    const size_t need = sc.n_partials > 0 ? gt_aggregate_ws_bytes(g, fi) : 0;
    if (need > 0) {
        if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: ws null or not 256-byte aligned", fn);
        if (ws_bytes < need) return gt_fail(GT_ERR_WORKSPACE, "%s: ws_bytes %zu < required %zu", fn, ws_bytes, need);
    }
    AggArgs a{};
    a.items = sc.items; a.n_items = sc.n_items;
    a.rowptr = sc.rowptr; a.nbr = sc.nbr;
    a.coef = sc.wt; a.post_mode = 0;
    if (reduce == GT_MEAN) a.post_mode = 2;
    else if (reduce == GT_SYMNORM) a.coef = sc.coef_sym;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy; a.F = fi;
    a.partials = static_cast<float *>(ws); a.ldp = (fi + 7) / 8 * 8;
    a.splits = sc.splits; a.n_splits = sc.n_splits;
    a.table_bytes = g->n_src * ldx * (int64_t)es;
    a.trace_kind = -1;
    a.n_rows = g->n_dst; a.n_edges = g->n_edges;
    if (sc.n_splits > 0) {
        // chunk items of the split rows first: partial rows only (no post-scaling; the fused kernel
        // adds them and scales), whole-row items skipped
        AggArgs c = a;
        c.post_mode = 0;
        c.only_split = 1;   // whole-row items are skipped ...
        c.no_reduce = 1;    // ... and the partial rows are left for the fused kernel to add
        c.Y = nullptr;
        const gt_status s = dtype == GT_F32 ? dispatch<float, 4>(c, st) : dispatch<bf16_t, 8>(c, st);
        if (s != GT_OK) return s;
    }
    FusedArgs f{};
    f.W = W; f.ldw = ldw; f.bias = bias; f.relu = act == GT_ACT_RELU; f.N = fo;
    f.n_entries = sc.n_items + sc.n_splits;
    const int tr = gt_trace_open(GT_TRACE_FUSED, fi, g->n_dst, g->n_edges, st);
    const gt_status s = dtype == GT_F32 ? fused_pick<float>(a, f, st) : fused_pick<bf16_t>(a, f, st);
    gt_trace_close(tr, st);
    return s;
}

extern "C" gt_status gt_aggregate_combine_supported(gt_dtype dtype, int64_t in_dim, int64_t out_dim, int *yes) {
    if (!yes) return gt_fail(GT_ERR_INVALID_ARG, "gt_aggregate_combine_supported: null");
    if (dtype != GT_F32 && dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "gt_aggregate_combine_supported: unknown dtype");
    *yes = gt_fused_applicable(dtype, in_dim, out_dim) ? 1 : 0;
    return GT_OK;
}

extern "C" gt_status gt_aggregate_combine_fwd(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t in_dim,
                                              int64_t out_dim, const void *X, int64_t ldx, const void *W, const float *b,
                                              gt_act act, void *Y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
    return gt_fused_run(g, reduce, dtype, in_dim, out_dim, X, ldx, W, out_dim, b, act, Y, ldy, ws, ws_bytes,
                        (hipStream_t)stream);
}
