// Edge weighting: the paper's NeighborApply primitive (the edge-weight function g of the source
// and destination embeddings, i.e. SDDMM) and Pull with per-call edge weights (the function h that
// transforms the source embedding with g's output before the aggregation f), forward and backward.
//
// Kept from the paper (Frontend section, NeighborApply / Pull): traversal is destination-centric
// and feature-wise; the destination's row is loaded once per work item and reused for all of its
// in-edges; the edge tensor produced by NeighborApply is what Pull consumes.  As for the plain
// aggregation, a group of G lanes of a 64-lane wavefront owns a work item and long rows are cut
// into chunk-sized items.  Three kernel shapes cover every call:
//   gather     out[r]  = sum_e c_e * h(X[nbr e], W_e)           (k_aggregate with vector weights)
//   edge-out   W_e     = s_r * (R[r] (.) X[nbr e])  or  s_r * R[r]        (k_edge_out)
//   edge-dot   w_e     = s_r * <R[r], X[nbr e]>                           (k_edge_dot)
// Derivatives with outputs on the source vertices run over the transposed structure and reach the
// per-edge data through its permutation (no atomics; results are reproducible).
#include "gt_aggregate_kernel.h"

namespace {

struct EdgeArgs {
    const gt_item *items;
    int64_t n_items;
    const int32_t *nbr;
    const void *R;        // row operand [n_rows][ldr]
    int64_t ldr;
    const float *rscale;  // per-row scale or null
    const void *X;        // gathered operand [n_in][ldx] (unused for broadcast)
    int64_t ldx;
    void *W;              // output: [E][ldw] of T (edge-out) or float[E] (edge-dot)
    int64_t ldw;
    int64_t F;
    int xcd_run;          // item blocks per XCD run (set at launch)
};

enum { EO_MUL = 0, EO_BCAST = 1 };

// W[e, :] = s_r * R[r, :] (.) X[nbr[e], :]   (EO_MUL)   or   s_r * R[r, :]   (EO_BCAST)
template <typename T, int V, int G, int NP, int MODE>
__global__ void __launch_bounds__(256) k_edge_out(const EdgeArgs a) {
    constexpr int NG = 64 / G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gl = lane & (G - 1), grp = lane / G;
    const int64_t item_id = (agg_item_block(a.xcd_run) * 4 + wave) * NG + grp;
    if (item_id >= a.n_items) return;
    const int4 raw = reinterpret_cast<const int4 *>(a.items)[item_id];
    const int row = raw.x, e0 = raw.y, e1 = raw.z;
    const int64_t col0 = (int64_t)blockIdx.y * (G * V * NP);
    const T *X = static_cast<const T *>(a.X);
    const T *R = static_cast<const T *>(a.R) + (int64_t)row * a.ldr;
    T *W = static_cast<T *>(a.W);
    typedef typename Raw<T, V>::type raw_t;

    float r[NP][V];
    const float s = a.rscale ? a.rscale[row] : 1.0f;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int64_t col = col0 + (int64_t)(p * G + gl) * V;
        raw_t rv = raw_t{};
        if (col < a.F && e0 < e1) rv = load_raw<T, V>(R + col);
        unpack_raw(rv, r[p]);
#pragma unroll
        for (int i = 0; i < V; ++i) r[p][i] *= s;
    }
    for (int base = e0; base < e1; base += G) {
        int idx = 0;
        if (MODE == EO_MUL && base + gl < e1) idx = a.nbr[base + gl];
        const int cnt = (e1 - base) < G ? (e1 - base) : G;
        for (int j = 0; j < cnt; j += 2) {
            raw_t v[2][NP];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int jj = j + u;
                const bool live = jj < cnt;
                if constexpr (MODE == EO_MUL) {
                    const int src = __shfl(idx, jj & (G - 1), G);
                    const T *xr = X + (int64_t)src * a.ldx;
#pragma unroll
                    for (int p = 0; p < NP; ++p) {
                        const int64_t col = col0 + (int64_t)(p * G + gl) * V;
                        v[u][p] = raw_t{};
                        if (live && col < a.F) v[u][p] = load_raw<T, V>(xr + col);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int jj = j + u;
                if (jj >= cnt) continue;
                T *wr = W + (int64_t)(base + jj) * a.ldw;
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const int64_t col = col0 + (int64_t)(p * G + gl) * V;
                    if (col >= a.F) continue;
                    const int n = (int)((a.F - col) < V ? (a.F - col) : V);
                    float o[V];
                    if constexpr (MODE == EO_MUL) {
                        float x[V];
                        unpack_raw(v[u][p], x);
#pragma unroll
                        for (int i = 0; i < V; ++i) o[i] = r[p][i] * x[i];
                    } else {
#pragma unroll
                        for (int i = 0; i < V; ++i) o[i] = r[p][i];
                    }
                    store_vec<T, V>(wr + col, o, n);
                }
            }
        }
    }
}

// w[e] = s_r * <R[r, :], X[nbr[e], :]>   (all columns inside one column tile)
template <typename T, int V, int G, int NP>
__global__ void __launch_bounds__(256) k_edge_dot(const EdgeArgs a) {
    constexpr int NG = 64 / G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gl = lane & (G - 1), grp = lane / G;
    const int64_t item_id = (agg_item_block(a.xcd_run) * 4 + wave) * NG + grp;
    if (item_id >= a.n_items) return;
    const int4 raw = reinterpret_cast<const int4 *>(a.items)[item_id];
    const int row = raw.x, e0 = raw.y, e1 = raw.z;
    const T *X = static_cast<const T *>(a.X);
    const T *R = static_cast<const T *>(a.R) + (int64_t)row * a.ldr;
    float *W = static_cast<float *>(a.W);
    typedef typename Raw<T, V>::type raw_t;

    const float s = a.rscale ? a.rscale[row] : 1.0f;
    constexpr int TILE = G * V * NP;
    for (int base = e0; base < e1; base += G) {
        int idx = 0;
        if (base + gl < e1) idx = a.nbr[base + gl];
        const int cnt = (e1 - base) < G ? (e1 - base) : G;
        float mine = 0.0f;   // lane gl keeps the result of edge base + gl
        // rows wider than one column tile are walked tile by tile; the row operand is re-read per
        // tile (it stays in the vector cache), the common single-tile case reads it once per batch
        for (int64_t c0 = 0; c0 < a.F; c0 += TILE) {
            float r[NP][V];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int64_t col = c0 + (int64_t)(p * G + gl) * V;
                raw_t rv = raw_t{};
                if (col < a.F) rv = load_raw<T, V>(R + col);
                unpack_raw(rv, r[p]);
            }
            for (int j = 0; j < cnt; j += 2) {
                raw_t v[2][NP];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int jj = j + u;
                    const int src = __shfl(idx, jj & (G - 1), G);
                    const T *xr = X + (int64_t)src * a.ldx;
#pragma unroll
                    for (int p = 0; p < NP; ++p) {
                        const int64_t col = c0 + (int64_t)(p * G + gl) * V;
                        v[u][p] = raw_t{};
                        if (jj < cnt && col < a.F) v[u][p] = load_raw<T, V>(xr + col);
                    }
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    float part = 0.0f;
#pragma unroll
                    for (int p = 0; p < NP; ++p) {
                        float x[V];
                        unpack_raw(v[u][p], x);
                        const int64_t col = c0 + (int64_t)(p * G + gl) * V;
#pragma unroll
                        for (int i = 0; i < V; ++i)   // padding elements of the last vector may hold anything
                            part += (col + i < a.F) ? r[p][i] * x[i] : 0.0f;
                    }
                    // butterfly over the group's lanes: every lane ends with the full sum, fixed order
#pragma unroll
                    for (int o = G / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, G);
                    if (gl == ((j + u) & (G - 1))) mine += part;
                }
            }
        }
        if (base + gl < e1) W[base + gl] = s * mine;   // one coalesced store of up to G results
    }
}

template <typename T, int V, int G, int NP>
gt_status launch_edge(const EdgeArgs &a, int kind, hipStream_t st) {
    constexpr int NG = 64 / G;
    if (a.n_items <= 0) return GT_OK;
    const int64_t tile = (int64_t)G * V * NP;
    const unsigned gy = kind == 2 ? 1u : (unsigned)((a.F + tile - 1) / tile);
    const int64_t gx = (a.n_items + 4 * NG - 1) / (4 * NG);
    const dim3 grid((unsigned)gx, gy);
    EdgeArgs b = a;
    b.xcd_run = agg_xcd_run(gx);
    if (kind == 0) k_edge_out<T, V, G, NP, EO_MUL><<<grid, 256, 0, st>>>(b);
    else if (kind == 1) k_edge_out<T, V, G, NP, EO_BCAST><<<grid, 256, 0, st>>>(b);
    else k_edge_dot<T, V, G, NP><<<grid, 256, 0, st>>>(b);
    GT_LAUNCH_CHECK("k_edge");
    return GT_OK;
}

template <typename T, int V>
gt_status dispatch_edge(const EdgeArgs &a, int kind, hipStream_t st) {
    const int64_t nvec = (a.F + V - 1) / V;
    if (nvec <= 4) return launch_edge<T, V, 4, 1>(a, kind, st);
    if (nvec <= 8) return launch_edge<T, V, 8, 1>(a, kind, st);
    if (nvec <= 16) return launch_edge<T, V, 16, 1>(a, kind, st);
    if (nvec <= 32) return launch_edge<T, V, 32, 1>(a, kind, st);
    if (nvec <= 64) return launch_edge<T, V, 64, 1>(a, kind, st);
    if (nvec <= 128) return launch_edge<T, V, 64, 2>(a, kind, st);
    if (nvec <= 192) return launch_edge<T, V, 64, 3>(a, kind, st);
    return launch_edge<T, V, 64, 4>(a, kind, st);
}

bool vec_ok(gt_dtype t, const void *p, int64_t ld) {
    const int64_t ve = t == GT_BF16 ? 8 : 4;
    return p == nullptr || (aligned16(p) && ld % ve == 0);
}

// kind: 0 edge-out product, 1 edge-out broadcast, 2 edge-dot
gt_status run_edge(const gt_graph *g, int kind, gt_dtype t, int64_t F, const void *R, int64_t ldr, const float *rscale,
                   const void *X, int64_t ldx, void *W, int64_t ldw, hipStream_t st) {
    EdgeArgs a{};
    a.items = g->fwd.items; a.n_items = g->fwd.n_items; a.nbr = g->colidx;
    a.R = R; a.ldr = ldr; a.rscale = rscale; a.X = X; a.ldx = ldx; a.W = W; a.ldw = ldw; a.F = F;
    const bool vec = vec_ok(t, R, ldr) && vec_ok(t, X, ldx) && (kind == 2 || vec_ok(t, W, ldw));
    if (t == GT_F32) return vec ? dispatch_edge<float, 4>(a, kind, st) : dispatch_edge<float, 1>(a, kind, st);
    return vec ? dispatch_edge<bf16_t, 8>(a, kind, st) : dispatch_edge<bf16_t, 1>(a, kind, st);
}

// gather: Y[r] = post( sum_e coef[ei] * coef2[e] * h(X[nbr e], VW[ei]) ), over the given or the
// transposed structure
gt_status run_gather(const gt_graph *g, bool transposed, gt_dtype t, int64_t F, const void *X, int64_t ldx, void *Y,
                     int64_t ldy, const float *coef, bool via_perm, const float *coef2, const void *VW, int64_t ldvw,
                     int vwm, int post_mode, void *ws, hipStream_t st) {
    const gt_sched &sc = transposed ? g->bwd : g->fwd;
    if (sc.n_rows == 0) return GT_OK;
    AggArgs a{};
    a.items = sc.items; a.n_items = sc.n_items; a.rowptr = sc.rowptr; a.nbr = sc.nbr;
    a.coef = coef; a.eidx = via_perm ? g->perm : nullptr; a.coef2 = coef2;
    a.VW = VW; a.ldvw = ldvw; a.post_mode = post_mode;
    a.bias = nullptr; a.relu = 0;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy; a.F = F;
    a.partials = static_cast<float *>(ws); a.ldp = (F + 7) / 8 * 8;
    a.splits = sc.splits; a.n_splits = sc.n_splits;
    a.table_bytes = ((int64_t)1 << 40);   // keep the two-loads-in-flight variant
    a.trace_kind = transposed ? GT_TRACE_AGG_BWD : GT_TRACE_AGG_FWD;
    a.n_rows = sc.n_rows; a.n_edges = g->n_edges;
    const bool vec = vec_ok(t, X, ldx) && vec_ok(t, Y, ldy) && vec_ok(t, VW, ldvw);
#define GT_GATHER(T_, V_)                                                      \
    (vwm == VWM_ADD ? dispatch<T_, V_, VWM_ADD>(a, st)                          \
                    : vwm == VWM_MUL ? dispatch<T_, V_, VWM_MUL>(a, st) : dispatch<T_, V_, VWM_NONE>(a, st))
    if (t == GT_F32) return vec ? GT_GATHER(float, 4) : GT_GATHER(float, 1);
    return vec ? GT_GATHER(bf16_t, 8) : GT_GATHER(bf16_t, 1);
#undef GT_GATHER
}

gt_status check_common(const char *fn, const gt_graph *g, gt_dtype t, int64_t F, void *ws, size_t ws_bytes,
                       bool needs_ws) {
    if (!g) return gt_fail(GT_ERR_INVALID_ARG, "%s: g is null", fn);
    if (t != GT_F32 && t != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown dtype", fn);
    if (F < 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: F < 0", fn);
    if (g->ew) return gt_fail(GT_ERR_UNSUPPORTED, "%s: the graph carries static edge weights; per-call edge weights "
                                                  "need a plan built without them", fn);
    if (needs_ws && (g->fwd.n_partials > 0 || g->bwd.n_partials > 0)) {
        const size_t need = gt_aggregate_ws_bytes(g, F);
        if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: ws null or not 256-byte aligned", fn);
        if (ws_bytes < need) return gt_fail(GT_ERR_WORKSPACE, "%s: ws_bytes %zu < required %zu", fn, ws_bytes, need);
    }
    return GT_OK;
}

}  // namespace

extern "C" gt_status gt_neighbor_apply_fwd(const gt_graph *g, gt_edge_fn fn_g, gt_dtype t, int64_t F, const void *Xs,
                                           int64_t ldxs, const void *Xd, int64_t ldxd, void *W, int64_t ldw,
                                           void *stream) {
    const char *fn = "gt_neighbor_apply_fwd";
    gt_status s = check_common(fn, g, t, F, nullptr, 0, false);
    if (s != GT_OK) return s;
    if (fn_g != GT_G_DOT && fn_g != GT_G_MUL) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown edge function", fn);
    if (g->n_edges == 0) return GT_OK;
    if (!W) return gt_fail(GT_ERR_INVALID_ARG, "%s: W is null", fn);
    if (F > 0 && (!Xs || !Xd)) return gt_fail(GT_ERR_INVALID_ARG, "%s: Xs or Xd is null", fn);
    if (ldxs < F || ldxd < F || (fn_g == GT_G_MUL && ldw < F))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension smaller than F", fn);
    if (F == 0 && fn_g == GT_G_MUL) return GT_OK;
    return run_edge(g, fn_g == GT_G_DOT ? 2 : 0, t, F, Xd, ldxd, nullptr, Xs, ldxs, W, ldw, (hipStream_t)stream);
}

extern "C" gt_status gt_neighbor_apply_bwd(const gt_graph *g, gt_edge_fn fn_g, gt_dtype t, int64_t F, const void *dW,
                                           int64_t lddw, const void *Xs, int64_t ldxs, const void *Xd, int64_t ldxd,
                                           void *dXs, int64_t lddxs, void *dXd, int64_t lddxd, void *ws,
                                           size_t ws_bytes, void *stream) {
    const char *fn = "gt_neighbor_apply_bwd";
    gt_status s = check_common(fn, g, t, F, ws, ws_bytes, true);
    if (s != GT_OK) return s;
    if (fn_g != GT_G_DOT && fn_g != GT_G_MUL) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown edge function", fn);
    if (F == 0) return GT_OK;
    if (!Xs || !Xd || !dXs || !dXd || (g->n_edges > 0 && !dW)) return gt_fail(GT_ERR_INVALID_ARG, "%s: null pointer", fn);
    if (ldxs < F || ldxd < F || lddxs < F || lddxd < F || (fn_g == GT_G_MUL && lddw < F))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension smaller than F", fn);
    hipStream_t st = (hipStream_t)stream;
    if (fn_g == GT_G_DOT) {
        // dXd[v] = sum_{e in in(v)} dw_e Xs[u];   dXs[u] = sum_{e in out(u)} dw_e Xd[v]
        s = run_gather(g, false, t, F, Xs, ldxs, dXd, lddxd, static_cast<const float *>(dW), false, nullptr, nullptr, 0,
                       VWM_NONE, 0, ws, st);
        if (s != GT_OK) return s;
        return run_gather(g, true, t, F, Xd, ldxd, dXs, lddxs, static_cast<const float *>(dW), true, nullptr, nullptr, 0,
                          VWM_NONE, 0, ws, st);
    }
    // dXd[v] = sum_e dW_e (.) Xs[u];   dXs[u] = sum_e dW_e (.) Xd[v]
    s = run_gather(g, false, t, F, Xs, ldxs, dXd, lddxd, nullptr, false, nullptr, dW, lddw, VWM_MUL, 0, ws, st);
    if (s != GT_OK) return s;
    return run_gather(g, true, t, F, Xd, ldxd, dXs, lddxs, nullptr, true, nullptr, dW, lddw, VWM_MUL, 0, ws, st);
}

extern "C" gt_status gt_pull_fwd(const gt_graph *g, gt_reduce reduce, gt_weight_fn h, gt_dtype t, int64_t F,
                                 const void *Xs, int64_t ldxs, const void *W, int64_t ldw, void *Y, int64_t ldy,
                                 void *ws, size_t ws_bytes, void *stream) {
    const char *fn = "gt_pull_fwd";
    gt_status s = check_common(fn, g, t, F, ws, ws_bytes, true);
    if (s != GT_OK) return s;
    if (reduce != GT_SUM && reduce != GT_MEAN) return gt_fail(GT_ERR_UNSUPPORTED, "%s: reduce must be GT_SUM or GT_MEAN", fn);
    if (h != GT_H_SCALE && h != GT_H_ADD && h != GT_H_MUL) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown weight function", fn);
    if (F == 0 || g->n_dst == 0) return GT_OK;
    if (!Y || (g->n_src > 0 && !Xs) || (g->n_edges > 0 && !W)) return gt_fail(GT_ERR_INVALID_ARG, "%s: null pointer", fn);
    if (ldxs < F || ldy < F || (h != GT_H_SCALE && ldw < F)) return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension smaller than F", fn);
    const int post = reduce == GT_MEAN ? 2 : 0;
    hipStream_t st = (hipStream_t)stream;
    if (h == GT_H_SCALE)
        return run_gather(g, false, t, F, Xs, ldxs, Y, ldy, static_cast<const float *>(W), false, nullptr, nullptr, 0,
                          VWM_NONE, post, ws, st);
    return run_gather(g, false, t, F, Xs, ldxs, Y, ldy, nullptr, false, nullptr, W, ldw, h == GT_H_ADD ? VWM_ADD : VWM_MUL,
                      post, ws, st);
}

extern "C" gt_status gt_pull_bwd(const gt_graph *g, gt_reduce reduce, gt_weight_fn h, gt_dtype t, int64_t F,
                                 const void *dY, int64_t lddy, const void *Xs, int64_t ldxs, const void *W, int64_t ldw,
                                 void *dXs, int64_t lddxs, void *dW, int64_t lddw, void *ws, size_t ws_bytes,
                                 void *stream) {
    const char *fn = "gt_pull_bwd";
    gt_status s = check_common(fn, g, t, F, ws, ws_bytes, true);
    if (s != GT_OK) return s;
    if (reduce != GT_SUM && reduce != GT_MEAN) return gt_fail(GT_ERR_UNSUPPORTED, "%s: reduce must be GT_SUM or GT_MEAN", fn);
    if (h != GT_H_SCALE && h != GT_H_ADD && h != GT_H_MUL) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown weight function", fn);
    if (F == 0) return GT_OK;
    if (!dY && g->n_dst > 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: dY is null", fn);
    if ((g->n_src > 0 && (!Xs || !dXs)) || (g->n_edges > 0 && (!W || !dW))) return gt_fail(GT_ERR_INVALID_ARG, "%s: null pointer", fn);
    if (lddy < F || ldxs < F || lddxs < F || (h != GT_H_SCALE && (ldw < F || lddw < F)))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension smaller than F", fn);
    hipStream_t st = (hipStream_t)stream;
    const bool mean = reduce == GT_MEAN;
    const float *cmean = (mean && g->n_edges > 0) ? g->coef_mean_b : nullptr;   // 1 / indeg(dst) per transposed entry
    const float *rdeg = mean ? g->rdeg : nullptr;                                // 1 / indeg per destination row
    // gradient of the source embeddings: outputs on the source vertices, transposed structure
    if (h == GT_H_SCALE) {
        s = run_gather(g, true, t, F, dY, lddy, dXs, lddxs, static_cast<const float *>(W), true, cmean, nullptr, 0,
                       VWM_NONE, 0, ws, st);
    } else if (h == GT_H_ADD) {
        s = run_gather(g, true, t, F, dY, lddy, dXs, lddxs, nullptr, false, cmean, nullptr, 0, VWM_NONE, 0, ws, st);
    } else {
        s = run_gather(g, true, t, F, dY, lddy, dXs, lddxs, nullptr, true, cmean, W, ldw, VWM_MUL, 0, ws, st);
    }
    if (s != GT_OK || g->n_edges == 0) return s;
    // gradient of the edge weights: one value (or row) per edge, destination-centric
    if (h == GT_H_SCALE) return run_edge(g, 2, t, F, dY, lddy, rdeg, Xs, ldxs, dW, 0, st);
    if (h == GT_H_ADD) return run_edge(g, 1, t, F, dY, lddy, rdeg, nullptr, 0, dW, lddw, st);
    return run_edge(g, 0, t, F, dY, lddy, rdeg, Xs, ldxs, dW, lddw, st);
}
