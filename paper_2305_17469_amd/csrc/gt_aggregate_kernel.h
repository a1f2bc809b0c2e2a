// Kernel templates of the neighbour aggregation (included by gt_aggregate.hip and gt_edge.hip).
//
// Neighbour aggregation (the paper's Pull primitive) and its derivative, as one gather-reduce
// kernel family over a work list.
//
// Prior art kept from the paper (Frontend section, "GNN graph aware scheduling" and the Pull
// description): traversal is destination-centric, all features of one output row are handled by
// one group of lanes spread over the feature columns, the running sum stays in registers and the
// row is written once, so no atomics or locks are needed.  What differs for CDNA4 and for full
// power-law graphs: a "group" is G = 4..64 lanes of a 64-wide wavefront, each lane moving
// 16 bytes per gathered row, so narrow rows still issue full-width memory instructions; rows
// longer than 1.5 chunks (a chunk is 512 entries, fewer on small graphs) are cut into chunk-sized work items whose fp32 partial rows
// are added by a second kernel in chunk order (deterministic, no floating-point atomics); work
// items are ordered longest first so the groups of a wavefront see similar trip counts.
//
// The same kernels serve the backward pass on the transposed structure: the derivative of the
// aggregation is an aggregation whose outputs are the source vertices (paper, "Training for
// GNNs").
#pragma once
#include "gt_internal.h"
#include "gt_trace.h"

namespace {

struct AggArgs {
    const gt_item *items;
    int64_t n_items;
    const int32_t *rowptr;   // of the output rows (for the mean's divisor)
    const int32_t *nbr;
    const float *coef;       // per-entry coefficient (edge weight x normalisation) or null (= 1)
    const int32_t *eidx;     // entry -> position in coef / VW (the transposed structure's perm), or null (= entry)
    const float *coef2;      // second per-entry factor, indexed by the entry itself, or null (= 1)
    const void *VW;          // per-entry vector weights [E][ldvw] (type T) for the VWM modes, or null
    int64_t ldvw;
    int post_mode;           // 0 none, 2 divide by the row's entry count (mean, forward)
    const float *bias;       // per-column bias added after scaling, or null
    int relu;
    const void *mask;        // [n_rows][ldmask] of type T or null: outputs are zeroed where mask <= 0 (the
    int64_t ldmask;          // derivative of the ReLU that produced `mask`, applied as the row is written)
    int pad_out;             // a row's last vector may be stored whole, with zeros past F, where it fits below ldy:
                             // a row end written in 2-byte pieces leaves a hole in its 32-byte sector, and memory
                             // has to read the sector back to merge it (2^21 rows of 47 bf16: 0.977 -> 0.918 ms)
    const void *X;
    int64_t ldx;
    void *Y;
    int64_t ldy;
    int64_t F;
    float *partials;         // [n_partials][ldp]
    int64_t ldp;
    const gt_split *splits;
    int64_t n_splits;
    int64_t table_bytes;     // host-side: size of the gathered table (picks the unroll)
    int xcd_run;             // item blocks per XCD run (0 or 1: plain order)
    int only_split;          // run only the chunk items of split rows (the whole-row items are someone else's)
    int no_reduce;           // host-side: do not launch the kernel that adds the partial rows
    int trace_kind;          // host-side bookkeeping of the optional kernel timing
    int64_t n_rows, n_edges;
};

typedef uint16_t bf16_t;

__device__ inline float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ inline uint32_t f32_to_bf16(float f) { return gt_to_bf16(f); }   // round to nearest even; NaN stays NaN

// Raw (unconverted) V consecutive elements, as they travel from memory: 16 bytes when V > 1.
template <typename T, int V> struct Raw;
template <> struct Raw<float, 4> { typedef float4 type; };
template <> struct Raw<float, 1> { typedef float type; };
template <> struct Raw<bf16_t, 8> { typedef uint4 type; };
template <> struct Raw<bf16_t, 1> { typedef bf16_t type; };

template <typename T, int V>
__device__ inline typename Raw<T, V>::type load_raw(const T *p) {
    return *reinterpret_cast<const typename Raw<T, V>::type *>(p);
}

// acc += c * raw  (fp32 accumulation)
__device__ inline void fma_raw(float (&acc)[4], float c, const float4 &v) {
    acc[0] = fmaf(c, v.x, acc[0]); acc[1] = fmaf(c, v.y, acc[1]);
    acc[2] = fmaf(c, v.z, acc[2]); acc[3] = fmaf(c, v.w, acc[3]);
}
__device__ inline void fma_raw(float (&acc)[1], float c, const float &v) { acc[0] = fmaf(c, v, acc[0]); }
__device__ inline void fma_raw(float (&acc)[8], float c, const uint4 &v) {
    acc[0] = fmaf(c, __uint_as_float(v.x << 16), acc[0]); acc[1] = fmaf(c, __uint_as_float(v.x & 0xffff0000u), acc[1]);
    acc[2] = fmaf(c, __uint_as_float(v.y << 16), acc[2]); acc[3] = fmaf(c, __uint_as_float(v.y & 0xffff0000u), acc[3]);
    acc[4] = fmaf(c, __uint_as_float(v.z << 16), acc[4]); acc[5] = fmaf(c, __uint_as_float(v.z & 0xffff0000u), acc[5]);
    acc[6] = fmaf(c, __uint_as_float(v.w << 16), acc[6]); acc[7] = fmaf(c, __uint_as_float(v.w & 0xffff0000u), acc[7]);
}
__device__ inline void fma_raw(float (&acc)[1], float c, const bf16_t &v) {
    acc[0] = fmaf(c, __uint_as_float((uint32_t)v << 16), acc[0]);
}

// raw -> fp32 values
__device__ inline void unpack_raw(const float4 &v, float (&o)[4]) { o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
__device__ inline void unpack_raw(const float &v, float (&o)[1]) { o[0] = v; }
__device__ inline void unpack_raw(const uint4 &v, float (&o)[8]) {
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
}
__device__ inline void unpack_raw(const bf16_t &v, float (&o)[1]) { o[0] = __uint_as_float((uint32_t)v << 16); }

// Vector-weight modes of the gather (paper: the function h that transforms the source embedding
// with the edge weight before the aggregation): 1: acc += c * (x + w),  2: acc += c * (x * w)
enum { VWM_NONE = 0, VWM_ADD = 1, VWM_MUL = 2 };
template <int VWM, int V, typename RawT>
__device__ inline void fma_vw(float (&acc)[V], float c, const RawT &x, const RawT &w) {
    float xf[V], wf[V];
    unpack_raw(x, xf);
    unpack_raw(w, wf);
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const float t = (VWM == VWM_ADD) ? xf[i] + wf[i] : xf[i] * wf[i];
        acc[i] = fmaf(c, t, acc[i]);
    }
}

// V consecutive elements starting at p (p is 16-byte aligned when V > 1) -> fp32
template <typename T, int V>
__device__ inline void load_vec(const T *p, float (&out)[V]);

template <>
__device__ inline void load_vec<float, 4>(const float *p, float (&out)[4]) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <>
__device__ inline void load_vec<float, 1>(const float *p, float (&out)[1]) { out[0] = *p; }
template <>
__device__ inline void load_vec<bf16_t, 8>(const bf16_t *p, float (&out)[8]) {
    const uint4 v = *reinterpret_cast<const uint4 *>(p);
    out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
    out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
    out[4] = __uint_as_float(v.z << 16); out[5] = __uint_as_float(v.z & 0xffff0000u);
    out[6] = __uint_as_float(v.w << 16); out[7] = __uint_as_float(v.w & 0xffff0000u);
}
template <>
__device__ inline void load_vec<bf16_t, 1>(const bf16_t *p, float (&out)[1]) { out[0] = bf16_to_f32(*p); }

// store the first `n` (<= V) of V values; full vectors go out as 16-byte stores
template <typename T, int V>
__device__ inline void store_vec(T *p, const float (&v)[V], int n);

template <>
__device__ inline void store_vec<float, 4>(float *p, const float (&v)[4], int n) {
    if (n >= 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        for (int i = 0; i < n; ++i) p[i] = v[i];
    }
}
template <>
__device__ inline void store_vec<float, 1>(float *p, const float (&v)[1], int n) { if (n > 0) p[0] = v[0]; }
template <>
__device__ inline void store_vec<bf16_t, 8>(bf16_t *p, const float (&v)[8], int n) {
    if (n >= 8) {
        uint4 o;
        o.x = gt_pack_bf16(v[0], v[1]);
        o.y = gt_pack_bf16(v[2], v[3]);
        o.z = gt_pack_bf16(v[4], v[5]);
        o.w = gt_pack_bf16(v[6], v[7]);
        *reinterpret_cast<uint4 *>(p) = o;
    } else {
        for (int i = 0; i < n; ++i) p[i] = (bf16_t)f32_to_bf16(v[i]);
    }
}
template <>
__device__ inline void store_vec<bf16_t, 1>(bf16_t *p, const float (&v)[1], int n) {
    if (n > 0) p[0] = (bf16_t)f32_to_bf16(v[0]);
}

// scale, bias, activation and store of one finished output row segment
// the mask values of this lane's segments of output row `row` (16-byte loads where the segment is whole);
// issued early by the callers so that the load is not a dependent round trip at the end of the item
template <typename T, int V, int G, int NP>
__device__ inline void load_mask_row(const AggArgs &a, int row, int gl, int64_t col0, float (&m)[NP][V]) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int64_t col = col0 + (int64_t)(p * G + gl) * V;
#pragma unroll
        for (int i = 0; i < V; ++i) m[p][i] = 1.0f;
        if (col >= a.F) continue;
        const int n = (int)((a.F - col) < V ? (a.F - col) : V);
        const T *mp = static_cast<const T *>(a.mask) + (int64_t)row * a.ldmask + col;
        if (n >= V) {
            load_vec<T, V>(mp, m[p]);
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) {
                float one[1] = {1.0f};
                if (i < n) load_vec<T, 1>(mp + i, one);
                m[p][i] = one[0];
            }
        }
    }
}

template <typename T, int V, int G, int NP>
__device__ inline void finish_row(const AggArgs &a, int row, int gl, int64_t col0, float (&acc)[NP][V],
                                  const float (&msk)[NP][V]) {
    bool zero = false;
    float div = 1.0f;
    if (a.post_mode == 2) {
        const int d = a.rowptr[row + 1] - a.rowptr[row];
        zero = d <= 0;
        div = (float)(d > 0 ? d : 1);
    }
    T *y = static_cast<T *>(a.Y) + (int64_t)row * a.ldy;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int64_t col = col0 + (int64_t)(p * G + gl) * V;
        if (col >= a.F) continue;
        const int n = (int)((a.F - col) < V ? (a.F - col) : V);
        float o[V];
#pragma unroll
        for (int i = 0; i < V; ++i) {
            float x = acc[p][i];
            if (a.post_mode == 2) x = zero ? 0.0f : x / div;
            if (a.bias && i < n) x += a.bias[col + i];
            if (a.relu) x = x > 0.0f ? x : 0.0f;
            if (a.mask) x = msk[p][i] > 0.0f ? x : 0.0f;
            o[i] = x;
        }
        int nst = n;
        if (V > 1 && a.pad_out && n < V && col + V <= a.ldy) {
#pragma unroll
            for (int i = 0; i < V; ++i) o[i] = i < n ? o[i] : 0.0f;
            nst = V;
        }
        store_vec<T, V>(y + col, o, nst);
    }
}

// Item block of this workgroup under the XCD-run order (run <= 1: plain order).  The remapping is
// a bijection on the blocks of every complete group of 8 * run blocks; the ragged end of the grid
// keeps the plain order.
__device__ inline int64_t agg_item_block(int run) {
    int64_t bx = blockIdx.x;
    if (gridDim.y == 1 && run > 1) {
        const int64_t super = 8 * (int64_t)run;
        const int64_t full = (int64_t)gridDim.x / super * super;
        if (bx < full) {
            const int64_t w = bx % super;
            bx = bx - w + (w & 7) * run + (w >> 3);
        }
    }
    return bx;
}

// Run length for a grid of gx item blocks: as long as possible for L2 reuse, but at least 64 turns
// over the 8 XCDs so that the longest-first order stays balanced (measured on MI355X: 2^18-vertex
// graph, 512-byte rows, 0.58 -> 0.50 ms at 64; narrow rows and small grids prefer 16-32; 256 was
// slower than 64 on a 2^21-vertex graph).
static inline int agg_xcd_run(int64_t gx) {
    int run = 1;
    while (run < 64 && (int64_t)run * 2 * 512 <= gx) run *= 2;
    return run;
}

// One group of G lanes per work item; 64/G items per wavefront; 4 wavefronts per workgroup.
// blockIdx.y selects a column tile of G*V*NP columns.
// MK: an output mask is present (its values are fetched when the item starts; a separate instance so
// that the registers they occupy during the gather cost the unmasked kernel nothing)
template <typename T, int V, int G, int NP, int U, int VWM = VWM_NONE, bool MK = false>
__global__ void __launch_bounds__(256) k_aggregate(const AggArgs a) {
    constexpr int NG = 64 / G;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int gl = lane & (G - 1);
    const int grp = lane / G;
    // Workgroups go to the 8 XCDs round-robin by index, and every XCD has its own L2.  Items are
    // sorted so that neighbours in the list gather from the same slice of the table; runs of
    // xcd_run consecutive item blocks are therefore handed to ONE XCD (the runs themselves still
    // rotate over the XCDs, which keeps the longest-first order balanced).
    const int64_t bx = agg_item_block(a.xcd_run);
    const int64_t item_id = (bx * 4 + wave) * NG + grp;
    if (item_id >= a.n_items) return;   // whole groups leave together; no barriers are used below
    const int4 raw = reinterpret_cast<const int4 *>(a.items)[item_id];
    int row = raw.x, e0 = raw.y, e1 = raw.z, slot = raw.w;
    if (a.only_split && slot < 0) return;   // uniform within the group
    if constexpr (G == 64) {   // one item per wavefront: keep its bounds in scalar registers
        row = __builtin_amdgcn_readfirstlane(row);
        e0 = __builtin_amdgcn_readfirstlane(e0);
        e1 = __builtin_amdgcn_readfirstlane(e1);
        slot = __builtin_amdgcn_readfirstlane(slot);
    }
    const int64_t col0 = (int64_t)blockIdx.y * (G * V * NP);
    const T *X = static_cast<const T *>(a.X);

    float acc[NP][V];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[p][i] = 0.0f;
    float msk[NP][V];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int i = 0; i < V; ++i) msk[p][i] = 1.0f;
    if constexpr (MK) {
        if (slot < 0) load_mask_row<T, V, G, NP>(a, row, gl, col0, msk);   // needed only when the row is finished here
    }

    typedef typename Raw<T, V>::type raw_t;
    // The group fetches G neighbour ids and coefficients with one coalesced load and walks them;
    // the next G are requested before the current ones are used, so the id fetch of the next
    // batch overlaps the row gathers of this one.
    int idx_next = 0, ei_next = 0;
    float c_next = 0.0f;
    auto fetch_entry = [&](int e) {
        idx_next = a.nbr[e];
        ei_next = a.eidx ? a.eidx[e] : e;
        c_next = a.coef ? a.coef[ei_next] : 1.0f;
        if (a.coef2) c_next *= a.coef2[e];
    };
    if (e0 + gl < e1) fetch_entry(e0 + gl);
    const T *VWp = static_cast<const T *>(a.VW);
    for (int base = e0; base < e1; base += G) {
        const int idx = idx_next;
        const int ei = ei_next;
        const float c = c_next;
        const int en = base + G + gl;
        idx_next = 0;
        ei_next = 0;
        c_next = 0.0f;
        if (en < e1) fetch_entry(en);
        const int cnt = (e1 - base) < G ? (e1 - base) : G;
        for (int j = 0; j < cnt; j += U) {
            raw_t v[U][NP];
            raw_t w[VWM == VWM_NONE ? 1 : U][VWM == VWM_NONE ? 1 : NP];
            float cj[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int jj = j + u;
                int src, we = 0;
                if constexpr (G == 64) {   // wave-uniform: scalar broadcast, scalar row base
                    src = __builtin_amdgcn_readlane(idx, jj & 63);
                    cj[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c), jj & 63));
                    if constexpr (VWM != VWM_NONE) we = __builtin_amdgcn_readlane(ei, jj & 63);
                } else {
                    src = __shfl(idx, jj & (G - 1), G);
                    cj[u] = __shfl(c, jj & (G - 1), G);
                    if constexpr (VWM != VWM_NONE) we = __shfl(ei, jj & (G - 1), G);
                }
                const bool live = jj < cnt;
                if (!live) cj[u] = 0.0f;
                const T *xr = X + (int64_t)src * a.ldx;
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const int64_t col = col0 + (int64_t)(p * G + gl) * V;
                    v[u][p] = raw_t{};
                    if (live && col < a.F) v[u][p] = load_raw<T, V>(xr + col);
                    if constexpr (VWM != VWM_NONE) {
                        w[u][p] = raw_t{};
                        if (live && col < a.F) w[u][p] = load_raw<T, V>(VWp + (int64_t)we * a.ldvw + col);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    if constexpr (VWM == VWM_NONE) fma_raw(acc[p], cj[u], v[u][p]);
                    else fma_vw<VWM, V>(acc[p], cj[u], v[u][p], w[u][p]);
                }
        }
    }

    if (slot >= 0) {
        float *P = a.partials + (int64_t)slot * a.ldp;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int64_t col = col0 + (int64_t)(p * G + gl) * V;
            if (col >= a.F) continue;
#pragma unroll
            for (int i = 0; i < V; ++i)
                if (col + i < a.F) P[col + i] = acc[p][i];
        }
    } else {
        finish_row<T, V, G, NP>(a, row, gl, col0, acc, msk);
    }
}

// Second pass for split rows: add the row's partial rows in chunk order.
template <typename T, int V, int G, int NP>
__global__ void __launch_bounds__(256) k_reduce_partials(const AggArgs a) {
    constexpr int NG = 64 / G;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int gl = lane & (G - 1);
    const int grp = lane / G;
    const int64_t sid = ((int64_t)blockIdx.x * 4 + wave) * NG + grp;
    if (sid >= a.n_splits) return;
    const gt_split s = a.splits[sid];
    const int64_t col0 = (int64_t)blockIdx.y * (G * V * NP);
    float acc[NP][V];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[p][i] = 0.0f;
    float msk[NP][V];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int i = 0; i < V; ++i) msk[p][i] = 1.0f;
    if (a.mask) load_mask_row<T, V, G, NP>(a, s.row, gl, col0, msk);
    // UR partial rows are requested at a time (branch free: a request past the end re-reads the
    // last row and is discarded) and added in chunk order.  Partial rows are padded to a multiple
    // of 8 floats, so whole vectors can be read; padding lanes are never stored.  The kernel runs as
    // long as its longest row (a hub of 86 K entries has 170 partial rows), one memory round trip
    // per UR rows: sixteen at a time where the registers allow it.
    constexpr int UR = NP * V <= 8 ? 16 : (NP * V <= 16 ? 8 : 4);
    for (int k = 0; k < s.count; k += UR) {
        float t[UR][NP][V];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int kk = (k + u < s.count) ? k + u : s.count - 1;
            const float *P = a.partials + (int64_t)(s.first + kk) * a.ldp;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int64_t col = col0 + (int64_t)(p * G + gl) * V;
                const int64_t c = col < a.F ? col : 0;
                if constexpr (V == 1) {
                    t[u][p][0] = P[c];
                } else {
#pragma unroll
                    for (int q = 0; q < V / 4; ++q) {
                        const float4 x = *reinterpret_cast<const float4 *>(P + c + 4 * q);
                        t[u][p][4 * q + 0] = x.x; t[u][p][4 * q + 1] = x.y;
                        t[u][p][4 * q + 2] = x.z; t[u][p][4 * q + 3] = x.w;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const bool live = k + u < s.count;
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int i = 0; i < V; ++i) acc[p][i] += live ? t[u][p][i] : 0.0f;
        }
    }
    finish_row<T, V, G, NP>(a, s.row, gl, col0, acc, msk);
}

template <typename T, int V, int G, int NP, int U, int VWM = VWM_NONE>
gt_status launch(const AggArgs &a, hipStream_t st) {
    constexpr int NG = 64 / G;
    const int64_t tile = (int64_t)G * V * NP;
    const unsigned gy = (unsigned)((a.F + tile - 1) / tile);
    if (a.n_items > 0) {
        const int64_t gx = (a.n_items + 4 * NG - 1) / (4 * NG);
        AggArgs b = a;
        b.xcd_run = agg_xcd_run(gx);
        const int tr = gt_trace_open(a.trace_kind, a.F, a.n_rows, a.n_edges, st);
        gt_trace_variant(tr, V, G, NP, U, VWM == VWM_NONE && a.mask != nullptr);
        if constexpr (VWM == VWM_NONE) {
            if (b.mask) k_aggregate<T, V, G, NP, U, VWM, true><<<dim3((unsigned)gx, gy), 256, 0, st>>>(b);
            else k_aggregate<T, V, G, NP, U, VWM, false><<<dim3((unsigned)gx, gy), 256, 0, st>>>(b);
        } else {
            k_aggregate<T, V, G, NP, U, VWM, false><<<dim3((unsigned)gx, gy), 256, 0, st>>>(b);
        }
        gt_trace_close(tr, st);
        GT_LAUNCH_CHECK("k_aggregate");
    }
    if (a.n_splits > 0 && !a.no_reduce) {
        const int64_t gx = (a.n_splits + 4 * NG - 1) / (4 * NG);
        k_reduce_partials<T, V, G, NP><<<dim3((unsigned)gx, gy), 256, 0, st>>>(a);
        GT_LAUNCH_CHECK("k_reduce_partials");
    }
    return GT_OK;
}

// Row loads kept in flight per lane.  Measured on MI355X: two are enough (and best) once the
// gathered table lives in HBM or rows are 512 bytes or more; narrow rows of a table that fits the
// last-level cache gain from eight.
template <typename T, int V, int G, int NP, int VWM = VWM_NONE>
gt_status launch_u(const AggArgs &a, hipStream_t st) {
    if constexpr (NP == 1 && G <= 16 && VWM == VWM_NONE) {
        if (a.table_bytes <= ((int64_t)96 << 20)) return launch<T, V, G, NP, 8>(a, st);
    }
    return launch<T, V, G, NP, 2, VWM>(a, st);
}

template <typename T, int V, int VWM = VWM_NONE>
gt_status dispatch(const AggArgs &a, hipStream_t st) {
    const int64_t nvec = (a.F + V - 1) / V;   // lanes needed to cover one row
    if (nvec <= 4) return launch_u<T, V, 4, 1, VWM>(a, st);
    if (nvec <= 8) return launch_u<T, V, 8, 1, VWM>(a, st);
    if (nvec <= 16) return launch_u<T, V, 16, 1, VWM>(a, st);
    if (nvec <= 32) return launch_u<T, V, 32, 1, VWM>(a, st);
    if (nvec <= 64) return launch_u<T, V, 64, 1, VWM>(a, st);
    if (nvec <= 128) return launch_u<T, V, 64, 2, VWM>(a, st);
    if (nvec <= 192) return launch_u<T, V, 64, 3, VWM>(a, st);
    return launch_u<T, V, 64, 4, VWM>(a, st);   // wider rows take several column tiles (grid.y)
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace
