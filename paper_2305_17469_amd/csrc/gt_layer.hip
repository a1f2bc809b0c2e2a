// One GNN layer with dynamic kernel placement (paper: GNN Kernel Orchestrator).
//
//   aggregation-first   H' = act( (A X) W + b )      sigma(W f(h(X)) + b)
//   combination-first   H' = act( A (X W) + b )      sigma(f(h(W X)) + b)
//
// Both are the same function because the aggregation is the linear map A; which one is cheaper
// depends on how much each kernel shrinks the tensor the other one has to process.  The paper's
// cost model expresses the gain of either order as (reduction factor) x (kernel execution
// factor); the two kernel-execution factors are kept here as kernel-time models
//     t_comb(rows, in, out) = rows * (alpha * in * out + beta * width)
//     t_aggr(E, n_out, F)   = F * (gamma * E + delta * n_out)
// whose differences between the two orders are exactly the four benefit formulas of the table
// "DKP cost model".  Summing kernel times instead of comparing benefits lets the same model
// cover the cases the table treats by a special rule (first layer: no backward aggregation at
// all when the forward ran aggregation-first) and the coupling of forward and backward through
// what was saved.
#include <math.h>

#include "gt_internal.h"
#include "gt_combine.h"

namespace {

typedef uint16_t bf16_t;

// Coefficients in seconds, one set per data type (index: gt_dtype).  Defaults are the values
// gt_calibrate fitted on an MI355X; gt_calibrate replaces them with values fitted on the device
// at hand.
gt_cost_coeffs g_cost[2] = {{1.06e-14, 1.39e-12, 4.87e-13, 1.06e-12, 8.78e-15, 1.66e-12, 4.48e-13, 1.27e-12, 4.3e-6},
                            {7.03e-15, 9.42e-13, 2.32e-13, 6.93e-13, 4.18e-15, 9.19e-13, 1.95e-13, 9.42e-13, 4.6e-6}};
const gt_cost_coeffs &cost_of(gt_dtype t) { return g_cost[t == GT_BF16 ? 1 : 0]; }

// An aggregation launch cannot finish faster than the chain of dependent loads of one work item
// (descriptor, neighbour ids, rows, a chunk of them for a hub row) however narrow the rows are:
// below the floor `aggr_floor` a narrower aggregation is not a faster one, so the model must not
// prefer it.  (4,096-vertex graph, 64 -> 16: both orders measure the same within launch jitter;
// without the floor the model picked the order that measured 9 % slower.)  The floor is fitted
// with the other coefficients (gt_calibrate times an aggregation on a tiny graph).

double t_comb(const gt_cost_coeffs &c, bool bwd, double rows, double in, double out) {
    return bwd ? rows * (c.alpha_bwd * in * out + c.beta_bwd * in) : rows * (c.alpha_fwd * in * out + c.beta_fwd * out);
}
double t_aggr(const gt_cost_coeffs &c, bool bwd, double E, double n_out, double F) {
    const double t = bwd ? F * (c.gamma_bwd * E + c.delta_bwd * n_out) : F * (c.gamma_fwd * E + c.delta_fwd * n_out);
    return t > c.aggr_floor ? t : c.aggr_floor;
}

__device__ inline float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ inline uint32_t f32_to_bf16(float f) { return gt_to_bf16(f); }
template <typename T> __device__ inline float ldf(const T *p);
template <> __device__ inline float ldf<float>(const float *p) { return *p; }
template <> __device__ inline float ldf<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void stf(T *p, float v);
template <> __device__ inline void stf<float>(float *p, float v) { *p = v; }
template <> __device__ inline void stf<bf16_t>(bf16_t *p, float v) { *p = (bf16_t)f32_to_bf16(v); }

// Rows per workgroup of the column-sum kernels: 512 on tall inputs, halved (down to 32) until there
// are about a thousand workgroups, so that the few thousand rows of a sampled batch still spread
// over all compute units (26.6 K rows x 256 columns: 30 -> 6 us measured on MI355X).
static inline int cs_rows(int64_t rows) {
    int r = 512;
    while (r > 32 && rows / r < 1024) r >>= 1;
    return r;
}

// dZ = dY * [Y > 0] (or dY when Y is null) and per-workgroup column sums of dZ.
// One workgroup covers rpb rows.  Its 256 threads form cw column lanes x 256/cw row lanes
// (cw = columns padded to a power of two, at most 256); a thread sums every (256/cw)-th row of
// its column, the row lanes are then added in lane order through LDS.  Every sum has a fixed
// order, so the result does not depend on scheduling.
template <typename T>
__global__ void __launch_bounds__(256) k_mask_colsum(const T *dY, int64_t lddy, const T *Y, int64_t ldy, T *dZ,
                                                     int64_t lddz, int64_t rows, int64_t cols, int cw, int rpb, float *partial) {
    __shared__ float red[256];
    const int rl_count = 256 / cw;
    const int cl = threadIdx.x % cw, rl = threadIdx.x / cw;
    const int64_t r0 = (int64_t)blockIdx.x * rpb;
    const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
    for (int64_t c0 = 0; c0 < cols; c0 += cw) {
        const int64_t c = c0 + cl;
        float s = 0.0f;
        if (c < cols) {
#pragma unroll 4
            for (int64_t r = r0 + rl; r < r1; r += rl_count) {
                float g = ldf<T>(dY + r * lddy + c);
                if (Y) {
                    g = ldf<T>(Y + r * ldy + c) > 0.0f ? g : 0.0f;
                    stf<T>(dZ + r * lddz + c, g);
                }
                s += g;
            }
        }
        if (partial) {
            red[threadIdx.x] = s;
            __syncthreads();
            if (rl == 0 && c < cols) {
                float t = 0.0f;
                for (int k = 0; k < rl_count; ++k) t += red[k * cw + cl];
                partial[(int64_t)blockIdx.x * cols + c] = t;
            }
            __syncthreads();
        }
    }
}

// 16-byte variant of k_mask_colsum for aligned, padded rows: a thread owns VE consecutive columns
// of every (256/cv)-th row; loads and stores are full vectors (padding columns are read and, in
// dZ, written; they never enter a sum that is stored).  Same fixed summation order as above.
template <typename T> struct MaskVec;
template <> struct MaskVec<float> {
    static constexpr int VE = 4;
    __device__ static void unpack(const uint4 &v, float (&o)[4]) {
        o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y); o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
    }
    __device__ static uint4 pack(const float (&o)[4]) {
        return make_uint4(__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3]));
    }
};
template <> struct MaskVec<bf16_t> {
    static constexpr int VE = 8;
    __device__ static void unpack(const uint4 &v, float (&o)[8]) {
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
        o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
        o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    __device__ static uint4 pack(const float (&o)[8]) {   // values are bf16 already: exact
        return make_uint4((__float_as_uint(o[0]) >> 16) | (__float_as_uint(o[1]) & 0xffff0000u),
                          (__float_as_uint(o[2]) >> 16) | (__float_as_uint(o[3]) & 0xffff0000u),
                          (__float_as_uint(o[4]) >> 16) | (__float_as_uint(o[5]) & 0xffff0000u),
                          (__float_as_uint(o[6]) >> 16) | (__float_as_uint(o[7]) & 0xffff0000u));
    }
};

template <typename T>
__global__ void __launch_bounds__(256) k_mask_colsum_vec(const T *dY, int64_t lddy, const T *Y, int64_t ldy, T *dZ,
                                                         int64_t lddz, int64_t rows, int64_t cols, int cv,
                                                         int rpb, float *partial) {
    constexpr int VE = MaskVec<T>::VE;
    __shared__ float red[256 * VE];
    const int rl_count = 256 / cv;
    const int cl = threadIdx.x % cv, rl = threadIdx.x / cv;
    const int64_t r0 = (int64_t)blockIdx.x * rpb;
    const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
    const int64_t nvec = (cols + VE - 1) / VE;
    for (int64_t v0 = 0; v0 < nvec; v0 += cv) {
        const int64_t vi = v0 + cl;
        const int64_t c = vi * VE;
        float s[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) s[e] = 0.0f;
        if (vi < nvec) {
#pragma unroll 4
            for (int64_t r = r0 + rl; r < r1; r += rl_count) {
                float g[VE];
                MaskVec<T>::unpack(*reinterpret_cast<const uint4 *>(dY + r * lddy + c), g);
                if (Y) {
                    float y[VE];
                    MaskVec<T>::unpack(*reinterpret_cast<const uint4 *>(Y + r * ldy + c), y);
#pragma unroll
                    for (int e = 0; e < VE; ++e) g[e] = y[e] > 0.0f ? g[e] : 0.0f;
                    *reinterpret_cast<uint4 *>(dZ + r * lddz + c) = MaskVec<T>::pack(g);
                }
#pragma unroll
                for (int e = 0; e < VE; ++e) s[e] += g[e];
            }
        }
        if (partial) {
#pragma unroll
            for (int e = 0; e < VE; ++e) red[threadIdx.x * VE + e] = s[e];
            __syncthreads();
            if (rl == 0 && vi < nvec) {
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    float t = 0.0f;
                    for (int k = 0; k < rl_count; ++k) t += red[(k * cv + cl) * VE + e];
                    if (c + e < cols) partial[(int64_t)blockIdx.x * cols + c + e] = t;
                }
            }
            __syncthreads();
        }
    }
}

// out[c] = sum over the nblk partial rows, 4 columns per workgroup, 64 row lanes per column; the
// lanes' sums are added in lane order, so the result does not depend on scheduling
__global__ void __launch_bounds__(256) k_colsum_final(const float *partial, int64_t nblk, int64_t cols, float *out) {
    __shared__ float red[256];
    const int cl = threadIdx.x & 3, rl = threadIdx.x >> 2;
    const int64_t c = (int64_t)blockIdx.x * 4 + cl;
    float s = 0.0f;
    if (c < cols)
        for (int64_t b = rl; b < nblk; b += 64) s += partial[b * cols + c];
    red[threadIdx.x] = s;
    __syncthreads();
    if (rl == 0 && c < cols) {
        float t = 0.0f;
        for (int k = 0; k < 64; ++k) t += red[k * 4 + cl];
        out[c] = t;
    }
}

int64_t pad_ld(int64_t F, gt_dtype t) {
    const int64_t v = t == GT_BF16 ? 8 : 4;
    return (F + v - 1) / v * v;
}

struct LayerLayout {
    // scratch regions (bytes offsets); forward and backward use the same buffer at different times
    size_t T;        // [n_src, ldo]  X W (combination-first forward)
    size_t dZ;       // [n_dst, ldo]
    size_t S;        // [n_src, ldo]  A^T dZ
    size_t dM;       // [n_dst, ldi]  dZ W^T
    size_t colsum;   // fp32 [ceil(n_dst / cs_rows(n_dst)), out]
    size_t agg_ws;   // aggregation partial rows
    size_t gemm_ws;  // split-k partials
    size_t total;
    size_t saved;    // bytes of `saved`: M = A X, [n_dst, ldi]
    int64_t ldi, ldo;
    size_t agg_ws_bytes, gemm_ws_bytes;
};

LayerLayout layer_layout(const gt_graph *g, const gt_layer_desc *d) {
    LayerLayout L{};
    const size_t es = gt_dtype_size(d->dtype);
    L.ldi = pad_ld(d->in_dim, d->dtype);
    L.ldo = pad_ld(d->out_dim, d->dtype);
    size_t off = 0;
    auto take = [&](size_t b) { size_t o = off; off += gt_align_up(b ? b : 4); return o; };
    L.T = take((size_t)g->n_src * L.ldo * es);
    L.dZ = take((size_t)g->n_dst * L.ldo * es);
    L.S = L.T;   // never live together: T belongs to the forward call, S to the backward call
    L.dM = take((size_t)g->n_dst * L.ldi * es);
    L.colsum = take((size_t)((g->n_dst + cs_rows(g->n_dst) - 1) / cs_rows(g->n_dst) + 1) * d->out_dim * 4);
    const int64_t fmax = d->in_dim > d->out_dim ? d->in_dim : d->out_dim;
    L.agg_ws_bytes = gt_aggregate_ws_bytes(g, fmax);
    L.agg_ws = take(L.agg_ws_bytes);
    // split-k partials: the largest need over every product either order may run
    L.gemm_ws_bytes = 0;
    for (const int64_t rows : {g->n_src, g->n_dst}) {
        const size_t need[3] = {gt_gemm_ws_bytes(1, d->in_dim, d->out_dim, rows),    // dW = X^T dZ
                                gt_gemm_ws_bytes(0, rows, d->out_dim, d->in_dim),    // X W
                                gt_gemm_ws_bytes(0, rows, d->in_dim, d->out_dim)};   // dZ W^T
        for (size_t nb : need)
            if (nb > L.gemm_ws_bytes) L.gemm_ws_bytes = nb;
    }
    L.gemm_ws = take(L.gemm_ws_bytes);
    L.total = off;
    L.saved = gt_align_up((size_t)g->n_dst * L.ldi * es);
    return L;
}

gt_status check_desc(const char *fn, const gt_graph *g, const gt_layer_desc *d) {
    if (!g || !d) return gt_fail(GT_ERR_INVALID_ARG, "%s: null graph or descriptor", fn);
    if (d->in_dim <= 0 || d->out_dim <= 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: in_dim and out_dim must be positive", fn);
    if (d->dtype != GT_F32 && d->dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown dtype", fn);
    if (d->reduce != GT_SUM && d->reduce != GT_MEAN && d->reduce != GT_SYMNORM)
        return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown reduce", fn);
    if (d->act != GT_ACT_NONE && d->act != GT_ACT_RELU) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown activation", fn);
    if (d->in_act != GT_ACT_NONE && d->in_act != GT_ACT_RELU) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown in_act", fn);
    if (d->reduce == GT_SYMNORM && g->n_dst != g->n_src)
        return gt_fail(GT_ERR_UNSUPPORTED, "%s: GT_SYMNORM needs a square graph", fn);
    if (d->has_root && g->n_dst > g->n_src)
        return gt_fail(GT_ERR_INVALID_ARG, "%s: has_root needs the destinations to be the first n_dst sources", fn);
    return GT_OK;
}

void *at(void *base, size_t off) { return static_cast<char *>(base) + off; }

bool ranges_overlap(const void *a, size_t a_elems, const void *b, size_t b_elems, size_t es) {
    const char *a0 = static_cast<const char *>(a), *b0 = static_cast<const char *>(b);
    return a0 < b0 + b_elems * es && b0 < a0 + a_elems * es;
}

// Forward-only aggregation-first layers: where the fused aggregation + combination kernel is used
// instead of the two kernels.  Measured on MI355X (ms, two kernels / fused): input rows of 64 bytes on a
// 2^20-vertex uniform graph, 16 -> 64 fp32 0.49 / 0.37, 16 -> 256 0.63 / 0.55: the gather of such
// rows is bound by the number of memory requests, and writing and re-reading A X costs as much as
// gathering it.  Wider rows lose: one workgroup per CU holds the weights, and eight wavefronts hide
// less gather latency than the aggregation kernel's two dozen (2^21-vertex power-law graph, bf16
// 100 -> 256: 1.96 / 2.52; 2^18 vertices, fp32 128 -> 41: 0.52 / 1.10; 41 -> 128: 0.27 / 0.57).  So do
// narrow rows of a table small enough to sit in the L2s, where the aggregation kernel is not request
// bound (2^18 vertices, 16 -> 64 fp32, a 16 MB table: 0.24 / 0.36; 2^21 vertices, 16 -> 64 bf16, 64 MB:
// 1.09 / 1.03).  Hence: rows of at most 64 bytes AND a gathered table of at least 32 MiB.
bool fused_preferred(const gt_graph *g, const gt_layer_desc *d, const void *X, int64_t ldx) {
    const int ve = d->dtype == GT_BF16 ? 8 : 4;
    if (!gt_fused_applicable(d->dtype, d->in_dim, d->out_dim) || ((uintptr_t)X & 15) || ldx % ve) return false;
    const int64_t row_bytes = d->in_dim * (int64_t)gt_dtype_size(d->dtype);
    return row_bytes <= 64 && g->n_src * row_bytes >= ((int64_t)32 << 20);
}

void decide(const gt_graph *g, const gt_layer_desc *d, gt_order *fwd, gt_order *bwd) {
    const gt_cost_coeffs &c = cost_of(d->dtype);
    const double ns = (double)g->n_src, nd = (double)g->n_dst, E = (double)g->n_edges;
    const double fi = (double)d->in_dim, fo = (double)d->out_dim;
    // forward
    const double f_agg = t_aggr(c, false, E, nd, fi) + t_comb(c, false, nd, fi, fo);
    const double f_comb = t_comb(c, false, ns, fi, fo) + t_aggr(c, false, E, nd, fo);
    // backward, by (forward order, backward order).  The weight gradient is (A X)^T dZ over n_dst
    // rows when A X was saved, else X^T (A^T dZ) over n_src rows, which needs A^T dZ.
    const double dw_agg = t_comb(c, true, nd, fi, fo), dw_comb = t_comb(c, true, ns, fi, fo);
    const double s_agg = t_aggr(c, true, E, ns, fo);   // A^T dZ
    double b[2][2];                                    // [fwd comb?][bwd comb?]
    if (d->need_dx) {
        const double dx_agg = t_comb(c, true, nd, fi, fo) + t_aggr(c, true, E, ns, fi);
        const double dx_comb = s_agg + t_comb(c, true, ns, fi, fo);
        b[0][0] = dw_agg + dx_agg;
        b[0][1] = dw_agg + dx_comb;
        b[1][0] = dw_comb + s_agg + dx_agg;
        b[1][1] = dw_comb + dx_comb;
    } else {
        // first layer: only parameter gradients; the backward order is immaterial but reported
        // as the forward's
        b[0][0] = b[0][1] = dw_agg;
        b[1][0] = b[1][1] = dw_comb + s_agg;
    }
    int bf = 0, bb = 0;
    double best = f_agg + b[0][0];
    const double cand[4] = {f_agg + b[0][0], f_agg + b[0][1], f_comb + b[1][0], f_comb + b[1][1]};
    for (int i = 1; i < 4; ++i) {
        if (cand[i] < best) { best = cand[i]; bf = i >> 1; bb = i & 1; }   // strict: ties keep aggregation-first
    }
    if (!d->need_dx) bb = bf;
    *fwd = bf ? GT_COMB_FIRST : GT_AGG_FIRST;
    *bwd = bb ? GT_COMB_FIRST : GT_AGG_FIRST;
}

template <typename T>
gt_status mask_colsum(const void *dY, int64_t lddy, const void *Y, int64_t ldy, void *dZ, int64_t lddz, int64_t rows,
                      int64_t cols, float *partial, float *db, hipStream_t st) {
    if (rows <= 0) {
        if (db) {   // empty sum: zeros, written by the same final kernel (no memset node)
            k_colsum_final<<<(unsigned)((cols + 3) / 4), 256, 0, st>>>(partial, 0, cols, db);
            GT_LAUNCH_CHECK("k_colsum_final");
        }
        return GT_OK;
    }
    const int rpb = cs_rows(rows);
    const int64_t nblk = (rows + rpb - 1) / rpb;
    constexpr int VE = MaskVec<T>::VE;
    const bool vec = (((uintptr_t)dY | (uintptr_t)Y | (uintptr_t)dZ) & 15) == 0 && lddy % VE == 0 &&
                     (!Y || (ldy % VE == 0 && lddz % VE == 0));
    if (vec) {
        int cv = 4;
        while (cv < 256 && cv * VE < cols) cv <<= 1;
        k_mask_colsum_vec<T><<<(unsigned)nblk, 256, 0, st>>>(static_cast<const T *>(dY), lddy, static_cast<const T *>(Y),
                                                             ldy, static_cast<T *>(dZ), lddz, rows, cols, cv, rpb,
                                                             db ? partial : nullptr);
    } else {
        int cw = 16;
        while (cw < 256 && cw < cols) cw <<= 1;
        k_mask_colsum<T><<<(unsigned)nblk, 256, 0, st>>>(static_cast<const T *>(dY), lddy, static_cast<const T *>(Y), ldy,
                                                         static_cast<T *>(dZ), lddz, rows, cols, cw, rpb,
                                                         db ? partial : nullptr);
    }
    GT_LAUNCH_CHECK("k_mask_colsum");
    if (db) {
        k_colsum_final<<<(unsigned)((cols + 3) / 4), 256, 0, st>>>(partial, nblk, cols, db);
        GT_LAUNCH_CHECK("k_colsum_final");
    }
    return GT_OK;
}

}  // namespace

static gt_status check_coeffs(const char *fn, const gt_cost_coeffs *c) {
    if (!c) return gt_fail(GT_ERR_INVALID_ARG, "%s: null", fn);
    const double v[9] = {c->alpha_fwd, c->beta_fwd, c->gamma_fwd, c->delta_fwd,
                         c->alpha_bwd, c->beta_bwd, c->gamma_bwd, c->delta_bwd, c->aggr_floor};
    for (double x : v)
        if (!(x >= 0.0) || !isfinite(x)) return gt_fail(GT_ERR_INVALID_ARG, "%s: coefficients must be finite and >= 0", fn);
    return GT_OK;
}

extern "C" gt_status gt_cost_get(gt_cost_coeffs *c) {
    if (!c) return gt_fail(GT_ERR_INVALID_ARG, "gt_cost_get: null");
    *c = g_cost[0];
    return GT_OK;
}

extern "C" gt_status gt_cost_set(const gt_cost_coeffs *c) {
    const gt_status s = check_coeffs("gt_cost_set", c);
    if (s != GT_OK) return s;
    g_cost[0] = *c;
    g_cost[1] = *c;
    return GT_OK;
}

extern "C" gt_status gt_cost_get_dtype(gt_dtype dtype, gt_cost_coeffs *c) {
    if (!c) return gt_fail(GT_ERR_INVALID_ARG, "gt_cost_get_dtype: null");
    if (dtype != GT_F32 && dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "gt_cost_get_dtype: unknown dtype");
    *c = g_cost[dtype == GT_BF16 ? 1 : 0];
    return GT_OK;
}

extern "C" gt_status gt_cost_set_dtype(gt_dtype dtype, const gt_cost_coeffs *c) {
    if (dtype != GT_F32 && dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "gt_cost_set_dtype: unknown dtype");
    const gt_status s = check_coeffs("gt_cost_set_dtype", c);
    if (s != GT_OK) return s;
    g_cost[dtype == GT_BF16 ? 1 : 0] = *c;
    return GT_OK;
}

extern "C" gt_status gt_cost_benefits(const gt_cost_coeffs *c, int64_t n_src, int64_t n_dst, int64_t n_edge,
                                      int64_t n_feat, int64_t n_hid, int first_layer, double *aggr_fwd,
                                      double *aggr_bwd, double *comb_fwd, double *comb_bwd) {
    if (!c) return gt_fail(GT_ERR_INVALID_ARG, "gt_cost_benefits: coefficients are null");
    const double ns = (double)n_src, nd = (double)n_dst, E = (double)n_edge, F = (double)n_feat, H = (double)n_hid;
    // table "DKP cost model": reduction factor x kernel execution factor
    if (aggr_fwd) *aggr_fwd = (ns - nd) * (c->alpha_fwd * H * F + c->beta_fwd * H);
    if (aggr_bwd) *aggr_bwd = (first_layer ? ns : (ns - nd)) * (c->alpha_bwd * H * F + c->beta_bwd * F);
    if (comb_fwd) *comb_fwd = (F - H) * (c->gamma_fwd * E + c->delta_fwd * nd);
    if (comb_bwd) *comb_bwd = (F - H) * (c->gamma_bwd * E + c->delta_bwd * ns);
    return GT_OK;
}

extern "C" gt_status gt_layer_decide(const gt_graph *g, const gt_layer_desc *d, gt_order *fwd, gt_order *bwd) {
    gt_status s = check_desc("gt_layer_decide", g, d);
    if (s != GT_OK) return s;
    gt_order f, b;
    decide(g, d, &f, &b);
    if (fwd) *fwd = f;
    if (bwd) *bwd = b;
    return GT_OK;
}

extern "C" gt_status gt_layer_ws_size(const gt_graph *g, const gt_layer_desc *d, size_t *saved_bytes,
                                      size_t *scratch_bytes) {
    gt_status s = check_desc("gt_layer_ws_size", g, d);
    if (s != GT_OK) return s;
    const LayerLayout L = layer_layout(g, d);
    if (saved_bytes) *saved_bytes = L.saved;
    if (scratch_bytes) *scratch_bytes = L.total;
    return GT_OK;
}

extern "C" gt_status gt_layer_fwd(const gt_graph *g, const gt_layer_desc *d, gt_order req, const void *X, int64_t ldx,
                                  const void *W, const void *W_root, const float *b, void *Y, int64_t ldy, void *saved,
                                  size_t saved_bytes, void *scratch, size_t scratch_bytes, gt_order *used,
                                  void *stream) {
    const char *fn = "gt_layer_fwd";
    gt_status s = check_desc(fn, g, d);
    if (s != GT_OK) return s;
    if (req != GT_AUTO && req != GT_AGG_FIRST && req != GT_COMB_FIRST) return gt_fail(GT_ERR_INVALID_ARG, "%s: bad order", fn);
    if (!X || !W || !Y) return gt_fail(GT_ERR_INVALID_ARG, "%s: X, W or Y is null", fn);
    if ((d->has_root != 0) != (W_root != nullptr)) return gt_fail(GT_ERR_INVALID_ARG, "%s: W_root must be given iff has_root", fn);
    if (ldx < d->in_dim || ldy < d->out_dim) return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension too small", fn);
    if (!scratch || ((uintptr_t)scratch & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: scratch null or not 256-byte aligned", fn);
    hipStream_t st = (hipStream_t)stream;
    const LayerLayout L = layer_layout(g, d);
    if (scratch_bytes < L.total)
        return gt_fail(GT_ERR_WORKSPACE, "%s: scratch_bytes %zu < required %zu", fn, scratch_bytes, L.total);
    if (ranges_overlap(X, (size_t)g->n_src * ldx, Y, (size_t)g->n_dst * ldy, gt_dtype_size(d->dtype)))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: X and Y overlap", fn);
    gt_order order = req;
    if (order == GT_AUTO) { gt_order bw; decide(g, d, &order, &bw); }
    if (order == GT_AGG_FIRST && saved) {
        if ((uintptr_t)saved & 255) return gt_fail(GT_ERR_WORKSPACE, "%s: saved not 256-byte aligned", fn);
        if (saved_bytes < L.saved)
            return gt_fail(GT_ERR_WORKSPACE, "%s: saved_bytes %zu < required %zu", fn, saved_bytes, L.saved);
    }
    if (used) *used = order;
    const gt_dtype t = d->dtype;
    const int64_t fi = d->in_dim, fo = d->out_dim;

    void *gws = at(scratch, L.gemm_ws);
    const bool pad_user = d->pad_writable != 0;   // the caller's Y has padded rows whose padding may be written
    if (order == GT_AGG_FIRST) {
        // forward only (no `saved`): A X is a temporary, or is never written at all where the fused
        // kernel applies and is the faster of the two
        if (!saved && !d->has_root && fused_preferred(g, d, X, ldx))
            return gt_fused_run(g, d->reduce, t, fi, fo, X, ldx, W, fo, b, d->act, Y, ldy, at(scratch, L.agg_ws),
                                L.agg_ws_bytes, st);
        void *M = saved ? saved : at(scratch, L.dM);
        // M = A X (kept for the weight gradient), then the combination on n_dst rows
        s = gt_aggregate_run(g, false, d->reduce, t, t, fi, X, ldx, M, L.ldi, nullptr, GT_ACT_NONE,
                             at(scratch, L.agg_ws), L.agg_ws_bytes, st, true, nullptr, 0, /*pad_out (own buffer)*/ true);
        if (s != GT_OK) return s;
        if (!d->has_root)
            return gt_gemm_run(fn, t, 0, 0, g->n_dst, fo, fi, M, L.ldi, W, fo, b, nullptr, d->act, nullptr, 0, Y, ldy,
                               t, gws, L.gemm_ws_bytes, st, nullptr, 0, nullptr, pad_user);
        s = gt_gemm_run(fn, t, 0, 0, g->n_dst, fo, fi, M, L.ldi, W, fo, nullptr, nullptr, GT_ACT_NONE, nullptr, 0, Y,
                        ldy, t, gws, L.gemm_ws_bytes, st);
        if (s != GT_OK) return s;
    } else {
        // T = X W on n_src rows, then the aggregation at width out_dim with bias and activation
        // applied as the row is written
        void *T = at(scratch, L.T);
        s = gt_gemm_run(fn, t, 0, 0, g->n_src, fo, fi, X, ldx, W, fo, nullptr, nullptr, GT_ACT_NONE, nullptr, 0, T, L.ldo,
                        t, gws, L.gemm_ws_bytes, st, nullptr, 0, nullptr, /*pad_c (own buffer)*/ true);
        if (s != GT_OK) return s;
        const bool fuse = !d->has_root;
        s = gt_aggregate_run(g, false, d->reduce, t, t, fo, T, L.ldo, Y, ldy, fuse ? b : nullptr,
                             fuse ? d->act : GT_ACT_NONE, at(scratch, L.agg_ws), L.agg_ws_bytes, st, true, nullptr, 0,
                             pad_user);
        if (s != GT_OK || fuse) return s;
    }
    // root term: Y = act(Y + X[0:n_dst] W_root + b)
    return gt_gemm_run(fn, t, 0, 0, g->n_dst, fo, fi, X, ldx, W_root, fo, b, nullptr, d->act, Y, ldy, Y, ldy, t, gws,
                       L.gemm_ws_bytes, st);
}

extern "C" gt_status gt_layer_bwd(const gt_graph *g, const gt_layer_desc *d, gt_order fwd_used, gt_order req,
                                  const void *dY, int64_t lddy, const void *X, int64_t ldx, const void *W,
                                  const void *W_root, const void *Y, int64_t ldy, const void *saved, size_t saved_bytes,
                                  void *scratch, size_t scratch_bytes, void *dX, int64_t lddx, float *dW,
                                  float *dW_root, float *db, gt_order *used, void *stream) {
    const char *fn = "gt_layer_bwd";
    gt_status s = check_desc(fn, g, d);
    if (s != GT_OK) return s;
    if (fwd_used != GT_AGG_FIRST && fwd_used != GT_COMB_FIRST)
        return gt_fail(GT_ERR_INVALID_ARG, "%s: fwd_used must be the order gt_layer_fwd reported", fn);
    if (req != GT_AUTO && req != GT_AGG_FIRST && req != GT_COMB_FIRST) return gt_fail(GT_ERR_INVALID_ARG, "%s: bad order", fn);
    if (!dY || !X || !W || !dW) return gt_fail(GT_ERR_INVALID_ARG, "%s: dY, X, W or dW is null", fn);
    if (d->act == GT_ACT_RELU && !d->dy_is_dz && !Y)
        return gt_fail(GT_ERR_INVALID_ARG, "%s: Y is needed for the ReLU derivative", fn);
    if ((d->has_root != 0) != (W_root != nullptr) || (d->has_root != 0) != (dW_root != nullptr))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: W_root and dW_root must be given iff has_root", fn);
    if ((d->need_dx != 0) != (dX != nullptr)) return gt_fail(GT_ERR_INVALID_ARG, "%s: dX must be given iff need_dx", fn);
    if (lddy < d->out_dim || ldx < d->in_dim || (Y && ldy < d->out_dim) || (dX && lddx < d->in_dim))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension too small", fn);
    if (fwd_used == GT_AGG_FIRST && !saved) return gt_fail(GT_ERR_INVALID_ARG, "%s: saved is null", fn);
    if (!scratch || ((uintptr_t)scratch & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: scratch null or not 256-byte aligned", fn);
    hipStream_t st = (hipStream_t)stream;
    const LayerLayout L = layer_layout(g, d);
    if (scratch_bytes < L.total)
        return gt_fail(GT_ERR_WORKSPACE, "%s: scratch_bytes %zu < required %zu", fn, scratch_bytes, L.total);
    if (fwd_used == GT_AGG_FIRST && saved_bytes < L.saved)
        return gt_fail(GT_ERR_WORKSPACE, "%s: saved_bytes %zu < required %zu", fn, saved_bytes, L.saved);
    if (dX && (ranges_overlap(dX, (size_t)g->n_src * lddx, dY, (size_t)g->n_dst * lddy, gt_dtype_size(d->dtype)) ||
               ranges_overlap(dX, (size_t)g->n_src * lddx, X, (size_t)g->n_src * ldx, gt_dtype_size(d->dtype))))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: dX overlaps dY or X", fn);
    const gt_dtype t = d->dtype;
    const int64_t fi = d->in_dim, fo = d->out_dim;

    gt_order order = req;
    if (order == GT_AUTO) {
        // best backward order given the forward order that actually ran
        gt_layer_desc dd = *d;
        gt_order f2, b2;
        decide(g, &dd, &f2, &b2);
        if (f2 == fwd_used) {
            order = b2;
        } else {
            const gt_cost_coeffs &c = cost_of(d->dtype);
            const double ns = (double)g->n_src, nd = (double)g->n_dst, E = (double)g->n_edges;
            const double dx_agg = t_comb(c, true, nd, fi, fo) + t_aggr(c, true, E, ns, fi) +
                                  (fwd_used == GT_COMB_FIRST ? t_aggr(c, true, E, ns, fo) : 0.0);
            const double dx_comb = t_aggr(c, true, E, ns, fo) + t_comb(c, true, ns, fi, fo);
            order = dx_comb < dx_agg ? GT_COMB_FIRST : GT_AGG_FIRST;
        }
        if (!d->need_dx) order = fwd_used;
    }
    if (used) *used = order;

    // dZ = dY * [Y > 0], db = column sums of dZ
    float *db_from_gemm = nullptr;
    const void *dZ = dY;
    int64_t lddz = lddy;
    float *partial = static_cast<float *>(at(scratch, L.colsum));
    if (d->act == GT_ACT_RELU && !d->dy_is_dz) {
        void *z = at(scratch, L.dZ);
        s = (t == GT_F32) ? mask_colsum<float>(dY, lddy, Y, ldy, z, L.ldo, g->n_dst, fo, partial, db, st)
                          : mask_colsum<bf16_t>(dY, lddy, Y, ldy, z, L.ldo, g->n_dst, fo, partial, db, st);
        dZ = z; lddz = L.ldo;
    } else if (db) {
        // dZ is dY as it is.  Its column sums come for free from a weight-gradient product that streams
        // dZ as its second operand (the root term's, or (A X)^T dZ); only a combination-first forward
        // without a root term has none, and sums dZ in a pass of its own.
        if (d->has_root || fwd_used == GT_AGG_FIRST) db_from_gemm = db;
        else
            s = (t == GT_F32) ? mask_colsum<float>(dY, lddy, nullptr, 0, nullptr, 0, g->n_dst, fo, partial, db, st)
                              : mask_colsum<bf16_t>(dY, lddy, nullptr, 0, nullptr, 0, g->n_dst, fo, partial, db, st);
    }
    if (s != GT_OK) return s;

    void *gws = at(scratch, L.gemm_ws);
    void *aws = at(scratch, L.agg_ws);
    if (d->has_root) {
        // dW_root = X[0:n_dst]^T dZ
        s = gt_gemm_run(fn, t, 1, 0, fi, fo, g->n_dst, X, ldx, dZ, lddz, nullptr, nullptr, GT_ACT_NONE, nullptr, 0, dW_root,
                        fo, GT_F32, gws, L.gemm_ws_bytes, st, nullptr, 0, db_from_gemm);
        if (s != GT_OK) return s;
        db_from_gemm = nullptr;
    }
    if (fwd_used == GT_AGG_FIRST) {
        // dW = (A X)^T dZ with the saved A X
        s = gt_gemm_run(fn, t, 1, 0, fi, fo, g->n_dst, saved, L.ldi, dZ, lddz, nullptr, nullptr, GT_ACT_NONE, nullptr, 0,
                        dW, fo, GT_F32, gws, L.gemm_ws_bytes, st, nullptr, 0, db_from_gemm);
        if (s != GT_OK) return s;
    }
    const bool need_S = (fwd_used == GT_COMB_FIRST) || (d->need_dx && order == GT_COMB_FIRST);
    void *S = at(scratch, L.S);
    if (need_S) {
        // S = A^T dZ: the aggregation's derivative, outputs on the source vertices, width out_dim
        s = gt_aggregate_run(g, true, d->reduce, t, t, fo, dZ, lddz, S, L.ldo, nullptr, GT_ACT_NONE, aws, L.agg_ws_bytes, st,
                             true, nullptr, 0, /*pad_out (own buffer)*/ true);
        if (s != GT_OK) return s;
    }
    if (fwd_used == GT_COMB_FIRST) {
        // dW = X^T (A^T dZ)
        s = gt_gemm_run(fn, t, 1, 0, fi, fo, g->n_src, X, ldx, S, L.ldo, nullptr, nullptr, GT_ACT_NONE, nullptr, 0, dW, fo,
                        GT_F32, gws, L.gemm_ws_bytes, st);
        if (s != GT_OK) return s;
    }
    if (!d->need_dx) return GT_OK;
    // in_act: dX leaves already multiplied by [X > 0] (X is a ReLU output: the derivative of the
    // layer below's activation).  The kernel that writes dX applies it as it stores the rows; with a
    // root term, whose product is added to part of dX afterwards, it is a pass of its own at the end.
    const bool mask_dx = d->in_act == GT_ACT_RELU;
    const void *mk = (mask_dx && !d->has_root) ? X : nullptr;
    if (order == GT_COMB_FIRST) {
        // dX = (A^T dZ) W^T
        s = gt_gemm_run(fn, t, 0, 1, g->n_src, fi, fo, S, L.ldo, W, fo, nullptr, nullptr, GT_ACT_NONE, nullptr, 0, dX, lddx,
                        t, gws, L.gemm_ws_bytes, st, mk, ldx, nullptr, d->pad_writable != 0);
    } else {
        // dM = dZ W^T (the combination's derivative uses the transposed weight), dX = A^T dM
        void *dM = at(scratch, L.dM);
        s = gt_gemm_run(fn, t, 0, 1, g->n_dst, fi, fo, dZ, lddz, W, fo, nullptr, nullptr, GT_ACT_NONE, nullptr, 0, dM, L.ldi,
                        t, gws, L.gemm_ws_bytes, st, nullptr, 0, nullptr, /*pad_c (own buffer)*/ true);
        if (s != GT_OK) return s;
        s = gt_aggregate_run(g, true, d->reduce, t, t, fi, dM, L.ldi, dX, lddx, nullptr, GT_ACT_NONE, aws, L.agg_ws_bytes, st,
                             true, mk, ldx, d->pad_writable != 0);
    }
    if (s != GT_OK) return s;
    if (d->has_root) {
        // dX[0:n_dst] += dZ W_root^T
        s = gt_gemm_run(fn, t, 0, 1, g->n_dst, fi, fo, dZ, lddz, W_root, fo, nullptr, nullptr, GT_ACT_NONE, dX, lddx, dX,
                        lddx, t, gws, L.gemm_ws_bytes, st);
        if (s != GT_OK) return s;
        if (mask_dx)
            s = (t == GT_F32) ? mask_colsum<float>(dX, lddx, X, ldx, dX, lddx, g->n_src, fi, nullptr, nullptr, st)
                              : mask_colsum<bf16_t>(dX, lddx, X, ldx, dX, lddx, g->n_src, fi, nullptr, nullptr, st);
    }
    return s;
}
