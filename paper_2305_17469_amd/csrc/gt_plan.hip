// Graph plan: degrees, the transposed (by-source) structure as a stable radix sort, and the
// degree-binned work lists of both aggregation directions.  Integer work only; every output
// is exactly defined, so it can be compared bit for bit.
//
// The paper keeps CSR for the forward pass and observes that CSC suits the backward pass
// ("Training for GNNs") and that per-batch format translation is pure overhead ("Graph
// simulation approach" and the kernel breakdown of its evaluation); here the translation is
// done once per graph and reused by every layer and epoch.
#include <stdarg.h>
#include <stdio.h>
#include <new>

#include "gt_internal.h"
#include "gt_prims.h"

// ---------------------------------------------------------------------------------------------
// status / error plumbing
// ---------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

void gt_set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

gt_status gt_fail(gt_status s, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return s;
}

gt_status gt_hip_fail(hipError_t e, const char *what) {
    snprintf(g_err, sizeof(g_err), "HIP error %d (%s) at %s", (int)e, hipGetErrorString(e), what);
    return GT_ERR_HIP;
}

extern "C" const char *gt_last_error(void) { return g_err; }

extern "C" const char *gt_status_string(gt_status s) {
    switch (s) {
        case GT_OK: return "GT_OK";
        case GT_ERR_INVALID_ARG: return "GT_ERR_INVALID_ARG";
        case GT_ERR_UNSUPPORTED: return "GT_ERR_UNSUPPORTED";
        case GT_ERR_WORKSPACE: return "GT_ERR_WORKSPACE";
        case GT_ERR_HIP: return "GT_ERR_HIP";
        case GT_ERR_INTERNAL: return "GT_ERR_INTERNAL";
    }
    return "GT_ERR_UNKNOWN";
}

extern "C" const char *gt_version(void) { return "gt 0.1 (gfx950)"; }

namespace {

// ---------------------------------------------------------------------------------------------
// plan kernels
// ---------------------------------------------------------------------------------------------
constexpr int PT = 256;
inline unsigned nblocks(int64_t n, int per = PT) { return (unsigned)((n + per - 1) / per); }

__global__ void k_row_degrees(const int32_t *rowptr, int64_t n_rows, int32_t *deg, float *rdeg, float *dinv) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    const int32_t d = rowptr[r + 1] - rowptr[r];
    deg[r] = d;
    if (rdeg) rdeg[r] = d > 0 ? 1.0f / (float)d : 0.0f;
    if (dinv) dinv[r] = d > 0 ? 1.0f / sqrtf((float)d) : 0.0f;
}

// rowptr_t from the sorted source keys: rowptr_t[u] = first position whose key >= u.
__global__ void k_boundaries(const uint32_t *skeys, int64_t E, int64_t n_src, int32_t *rowptr_t) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k > E) return;
    // position k closes the gap (key[k-1], key[k]]; k == E closes (key[E-1], n_src]
    const int64_t lo = (k == 0) ? -1 : (int64_t)skeys[k - 1];
    const int64_t hi = (k == E) ? n_src : (int64_t)skeys[k];
    for (int64_t u = lo + 1; u <= hi; ++u) rowptr_t[u] = (int32_t)k;
}

// Per transposed entry k (position e = perm[k] in the given CSR): its destination, its weight, and
// the per-entry coefficients of the normalised reduce modes, written in both entry orders:
//   symmetric norm  w_e / sqrt(d(src) d(dst))   (coef_sym_f[e], coef_sym_b[k]; square graphs)
//   mean, backward  w_e / indeg(dst)            (coef_mean_b[k])
__global__ void k_transposed_entries(const int32_t *rowptr, int64_t n_dst, const int32_t *perm, int64_t E,
                                     const int32_t *colidx, const float *ew, const float *dinv, const float *rdeg,
                                     int32_t *colidx_t, float *ew_t, float *coef_sym_f, float *coef_sym_b,
                                     float *coef_mean_b) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= E) return;
    const int32_t e = perm[k];
    // destination of entry e: the last row v with rowptr[v] <= e
    int64_t lo = 0, hi = n_dst;   // invariant: rowptr[lo] <= e < rowptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= e) lo = mid; else hi = mid;
    }
    colidx_t[k] = (int32_t)lo;
    const float w = ew ? ew[e] : 1.0f;
    if (ew_t) ew_t[k] = w;
    if (dinv) {
        const float c = (w * dinv[colidx[e]]) * dinv[lo];
        coef_sym_f[e] = c;
        coef_sym_b[k] = c;
    }
    coef_mean_b[k] = w * rdeg[lo];
}

// per-row item / partial / split counts
__global__ void k_item_counts(const int32_t *rowptr, int64_t n_rows, int chunk, int32_t *c_items, int32_t *c_parts,
                              int32_t *c_splits) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r > n_rows) return;
    if (r == n_rows) {   // the extra entry makes the exclusive scans end with the totals
        c_items[r] = 0; c_parts[r] = 0; c_splits[r] = 0;
        return;
    }
    const int32_t d = rowptr[r + 1] - rowptr[r];
    const bool split = d > chunk + chunk / 2;
    const int32_t chunks = (d + chunk - 1) / chunk;
    c_items[r] = split ? chunks : 1;
    c_parts[r] = split ? chunks : 0;
    c_splits[r] = split ? 1 : 0;
}

__global__ void k_collect_counts(const int32_t *ca, const int32_t *cb, const int32_t *cc, int64_t n_rows, int32_t *cnt3) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        cnt3[0] = ca[n_rows]; cnt3[1] = cb[n_rows]; cnt3[2] = cc[n_rows];
    }
}

__device__ inline uint32_t length_key(int32_t len) {
    // Descending-length sort key, half-octave resolution (exact below 4).  Measured on MI355X with
    // quarter-octave, half-octave and octave classes: coarser classes leave more of the order to
    // the locality key (better L2 reuse), finer ones balance the groups of a wavefront better;
    // half an octave was the best or within 2 % of it on every width of configs 2 and 3.
    uint32_t k;
    if (len < 4) {
        k = (uint32_t)len;
    } else {
        const int lg = 31 - __clz(len);
        k = 4u + (uint32_t)(lg - 2) * 2u + (((uint32_t)len >> (lg - 1)) & 1u);
    }
    return 255u - k;
}

// Sort key of an item: length class (longest first) in bits 8-15, then the range its MEDIAN
// neighbour id falls in (256 ranges) in bits 0-7, so that items running at the same time gather
// from the same region of the table and reuse each other's rows in the L2.  (Rows are sorted by
// neighbour id; on power-law graphs the first neighbour is a hub for almost every row and tells
// little, the median separates rows much better: config 3, width 256, 3.47 -> 3.27 ms.)
__device__ inline uint32_t item_key(int32_t len, const int32_t *nbr, int32_t e0, int64_t n_in) {
    uint32_t loc = 0;
    if (len > 0 && n_in > 0) loc = (uint32_t)(((int64_t)nbr[e0 + len / 2] << 8) / n_in) & 255u;
    return (length_key(len) << 8) | loc;
}

__global__ void k_fill_items(const int32_t *rowptr, const int32_t *nbr, int64_t n_in, int64_t n_rows, int chunk,
                             const int32_t *o_items, const int32_t *o_parts, const int32_t *o_splits, gt_item *items,
                             uint32_t *keys, gt_split *splits) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    const int32_t b = rowptr[r], e = rowptr[r + 1], d = e - b;
    int32_t it = o_items[r];
    if (d > chunk + chunk / 2) {
        const int32_t chunks = (d + chunk - 1) / chunk;
        const int32_t p0 = o_parts[r];
        gt_split s;
        s.row = (int32_t)r; s.first = p0; s.count = chunks; s.pad = 0;
        splits[o_splits[r]] = s;
        for (int32_t c = 0; c < chunks; ++c) {
            gt_item x;
            x.row = (int32_t)r;
            x.e0 = b + c * chunk;
            x.e1 = min(e, x.e0 + chunk);
            x.slot = p0 + c;
            items[it + c] = x;
            keys[it + c] = item_key(x.e1 - x.e0, nbr, x.e0, n_in);
        }
    } else {
        gt_item x;
        x.row = (int32_t)r; x.e0 = b; x.e1 = e; x.slot = -1;
        items[it] = x;
        keys[it] = item_key(d, nbr, b, n_in);
    }
}

__global__ void k_gather_items(const gt_item *src, const uint32_t *idx, int64_t n, gt_item *dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[idx[i]];
}

__global__ void k_validate(const int32_t *rowptr, const int32_t *colidx, int64_t n_dst, int64_t n_src, int64_t E,
                           unsigned long long *bad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long v = 0;
    if (i < n_dst && rowptr[i + 1] < rowptr[i]) v++;
    if (i == 0 && rowptr[0] != 0) v++;
    if (i == 0 && (int64_t)rowptr[n_dst] != E) v++;
    if (i < E && (colidx[i] < 0 || (int64_t)colidx[i] >= n_src)) v++;
    if (v) atomicAdd(bad, v);   // integer atomic: the count does not depend on the order
}

// ---------------------------------------------------------------------------------------------
// workspace layout
// ---------------------------------------------------------------------------------------------
struct PlanLayout {
    size_t in_deg, out_deg, rowptr_t, colidx_t, perm, ew_t, dinv, rdeg;
    size_t items_f, splits_f, items_b, splits_b;
    size_t counts;                       // 8 int32 read back by the host
    size_t ca, cb, cc;                   // per-row count arrays (max(n_dst, n_src) + 1 each), forward direction
    size_t ca2, cb2, cc2;                // the same for the transposed direction
    size_t items_tmp, item_keys, item_keys2, item_idx, item_idx2;   // unsorted items, sort keys / indices
    size_t k0, v0, k1, v1;               // sort ping-pong (E each); k0, v0, v1 hold the coefficient arrays afterwards
    size_t hist, scan_tmp;
    size_t total;
};

int64_t max_items(int64_t n_rows, int64_t E) { return n_rows + E / gt_chunk_for(E) + 1; }
int64_t max_splits(int64_t E) { return E / gt_split_min(gt_chunk_for(E)) + 1; }

PlanLayout plan_layout(int64_t n_dst, int64_t n_src, int64_t E, bool has_ew) {
    PlanLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += gt_align_up(bytes ? bytes : 4); return o; };
    const int64_t nmax = (n_dst > n_src ? n_dst : n_src);
    const int64_t imax = max_items(nmax, E);
    L.in_deg = take((size_t)n_dst * 4);
    L.out_deg = take((size_t)n_src * 4);
    L.rowptr_t = take((size_t)(n_src + 1) * 4);
    L.colidx_t = take((size_t)E * 4);
    L.perm = take((size_t)E * 4);
    L.ew_t = take(has_ew ? (size_t)E * 4 : 0);
    L.dinv = take((size_t)nmax * 4);
    L.rdeg = take((size_t)n_dst * 4);
    L.items_f = take((size_t)max_items(n_dst, E) * sizeof(gt_item));
    L.splits_f = take((size_t)max_splits(E) * sizeof(gt_split));
    L.items_b = take((size_t)max_items(n_src, E) * sizeof(gt_item));
    L.splits_b = take((size_t)max_splits(E) * sizeof(gt_split));
    L.counts = take(128);
    L.ca = take((size_t)(nmax + 1) * 4);
    L.cb = take((size_t)(nmax + 1) * 4);
    L.cc = take((size_t)(nmax + 1) * 4);
    L.ca2 = take((size_t)(nmax + 1) * 4);
    L.cb2 = take((size_t)(nmax + 1) * 4);
    L.cc2 = take((size_t)(nmax + 1) * 4);
    L.items_tmp = take((size_t)imax * sizeof(gt_item));
    L.item_keys = take((size_t)imax * 4);
    L.item_keys2 = take((size_t)imax * 4);
    L.item_idx = take((size_t)imax * 4);
    L.item_idx2 = take((size_t)imax * 4);
    L.k0 = take((size_t)E * 4);
    L.v0 = take((size_t)E * 4);
    L.k1 = take((size_t)E * 4);
    L.v1 = take((size_t)E * 4);
    const int64_t nsort = E > imax ? E : imax;
    const int64_t hist_n = (int64_t)256 * (rs_blocks(nsort) + 1);
    L.hist = take((size_t)hist_n * 4);
    const int64_t scan_n = hist_n > nmax + 1 ? hist_n : nmax + 1;
    L.scan_tmp = take(scan_tmp_ints(scan_n) * 4);
    L.total = off;
    return L;
}

template <typename T>
T *at(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }

// counts of one direction into cnt[0..2] (items, partials, splits): scans of the per-row counts;
// the exclusive scan over n_rows + 1 entries (last input 0) leaves the total in element n_rows.
gt_status count_direction(const int32_t *rowptr, int64_t n_rows, int chunk, void *ws, const PlanLayout &L,
                          bool transposed, int32_t *cnt3, hipStream_t st) {
    int32_t *ca = at<int32_t>(ws, transposed ? L.ca2 : L.ca), *cb = at<int32_t>(ws, transposed ? L.cb2 : L.cb);
    int32_t *cc = at<int32_t>(ws, transposed ? L.cc2 : L.cc);
    int32_t *stmp = at<int32_t>(ws, L.scan_tmp);
    k_item_counts<<<nblocks(n_rows + 1), PT, 0, st>>>(rowptr, n_rows, chunk, ca, cb, cc);
    GT_LAUNCH_CHECK("k_item_counts");
    gt_status s;
    const int32_t *in3[3] = {ca, cb, cc};
    int32_t *out3[3] = {ca, cb, cc};
    if ((s = scan_exclusive_batch(3, in3, out3, n_rows + 1, stmp, st)) != GT_OK) return s;
    k_collect_counts<<<1, 64, 0, st>>>(ca, cb, cc, n_rows, cnt3);
    GT_LAUNCH_CHECK("k_collect_counts");
    return GT_OK;
}

// items of one direction, sorted longest first (stable, so equal lengths keep row order).
constexpr int64_t GT_SORT_ITEMS_MIN = 16384;
gt_status build_direction(const int32_t *rowptr, const int32_t *nbr, int64_t n_in, int64_t n_rows, int chunk,
                          int64_t n_items, void *ws, const PlanLayout &L, bool transposed, gt_item *items_out,
                          gt_split *splits_out, hipStream_t st) {
    if (n_rows <= 0 || n_items <= 0) return GT_OK;
    int32_t *ca = at<int32_t>(ws, transposed ? L.ca2 : L.ca), *cb = at<int32_t>(ws, transposed ? L.cb2 : L.cb);
    int32_t *cc = at<int32_t>(ws, transposed ? L.cc2 : L.cc);
    gt_item *tmp = at<gt_item>(ws, L.items_tmp);
    uint32_t *keys = at<uint32_t>(ws, L.item_keys), *keys2 = at<uint32_t>(ws, L.item_keys2);
    uint32_t *idx = at<uint32_t>(ws, L.item_idx), *idx2 = at<uint32_t>(ws, L.item_idx2);
    // A small graph is bound by launch latency, not by load balance or locality: its items stay in
    // row order and the two sort passes and the gather are saved.
    const bool sorted = n_items > GT_SORT_ITEMS_MIN;
    k_fill_items<<<nblocks(n_rows), PT, 0, st>>>(rowptr, nbr, n_in, n_rows, chunk, ca, cb, cc, sorted ? tmp : items_out, keys,
                                                 splits_out);
    GT_LAUNCH_CHECK("k_fill_items");
    if (!sorted) return GT_OK;
    SortTmp t{at<int32_t>(ws, L.hist), at<int32_t>(ws, L.scan_tmp)};
    gt_status s = radix_pass(keys, nullptr, keys2, idx, n_items, 0, t, st);      // neighbour range
    if (s != GT_OK) return s;
    s = radix_pass(keys2, idx, keys, idx2, n_items, 8, t, st);                   // length class (stable)
    if (s != GT_OK) return s;
    k_gather_items<<<nblocks(n_items), PT, 0, st>>>(tmp, idx2, n_items, items_out);
    GT_LAUNCH_CHECK("k_gather_items");
    return GT_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" gt_status gt_graph_plan_size(int64_t n_dst, int64_t n_src, int64_t n_edges, int has_edge_weight,
                                        size_t *ws_bytes) {
    if (!ws_bytes) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_plan_size: ws_bytes is null");
    if (n_dst < 0 || n_src < 0 || n_edges < 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_plan_size: negative size");
    // int32 indices everywhere; the kernels step through an entry list in strides of up to 512 and
    // look one stride ahead, so the largest entry index plus two strides must still fit an int32
    const int64_t lim = 2147483648LL - 1024;
    if (n_dst >= lim || n_src >= lim || n_edges >= lim)
        return gt_fail(GT_ERR_UNSUPPORTED, "gt_graph_plan_size: sizes must be below 2^31 - 1024 (int32 indices)");
    *ws_bytes = plan_layout(n_dst, n_src, n_edges, has_edge_weight != 0).total;
    return GT_OK;
}

extern "C" gt_status gt_graph_create(gt_graph **out, int64_t n_dst, int64_t n_src, int64_t E, const int32_t *rowptr,
                                     const int32_t *colidx, const float *ew, void *ws, size_t ws_bytes, void *stream) {
    if (!out) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_create: g is null");
    *out = nullptr;
    size_t need = 0;
    gt_status s = gt_graph_plan_size(n_dst, n_src, E, ew != nullptr, &need);
    if (s != GT_OK) return s;
    if (!rowptr) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_create: rowptr is null");
    if (E > 0 && !colidx) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_create: colidx is null with n_edges > 0");
    if (E > 0 && n_src == 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_create: edges but n_src == 0");
    if (E > 0 && n_dst == 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_create: edges but n_dst == 0");
    if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "gt_graph_create: ws null or not 256-byte aligned");
    if (ws_bytes < need) return gt_fail(GT_ERR_WORKSPACE, "gt_graph_create: ws_bytes %zu < required %zu", ws_bytes, need);
    hipStream_t st = (hipStream_t)stream;
    const PlanLayout L = plan_layout(n_dst, n_src, E, ew != nullptr);

    gt_graph *g = new (std::nothrow) gt_graph();
    if (!g) return gt_fail(GT_ERR_INTERNAL, "gt_graph_create: out of host memory");
    g->n_dst = n_dst; g->n_src = n_src; g->n_edges = E;
    g->rowptr = rowptr; g->colidx = colidx; g->ew = ew;
    g->in_deg = at<int32_t>(ws, L.in_deg);
    g->out_deg = at<int32_t>(ws, L.out_deg);
    g->rowptr_t = at<int32_t>(ws, L.rowptr_t);
    g->colidx_t = at<int32_t>(ws, L.colidx_t);
    g->perm = at<int32_t>(ws, L.perm);
    g->ew_t = ew ? at<float>(ws, L.ew_t) : nullptr;
    g->dinv = (n_dst == n_src) ? at<float>(ws, L.dinv) : nullptr;
    g->rdeg = at<float>(ws, L.rdeg);
    g->vcount = at<unsigned long long>(ws, L.counts + 64);

    auto fail = [&](gt_status rc) { delete g; return rc; };
#define PLAN_HIP(call) do { hipError_t e__ = (call); if (e__ != hipSuccess) return fail(gt_hip_fail(e__, #call)); } while (0)
#define PLAN_LAUNCH(what) do { hipError_t e__ = hipGetLastError(); if (e__ != hipSuccess) return fail(gt_hip_fail(e__, what)); } while (0)

    // degrees of the given CSR
    if (n_dst > 0) {
        k_row_degrees<<<nblocks(n_dst), PT, 0, st>>>(rowptr, n_dst, g->in_deg, g->rdeg, g->dinv);
        PLAN_LAUNCH("k_row_degrees");
    }
    // transposed structure: stable sort of (source, position) pairs by source
    SortTmp t{at<int32_t>(ws, L.hist), at<int32_t>(ws, L.scan_tmp)};
    uint32_t *k0 = at<uint32_t>(ws, L.k0), *v0 = at<uint32_t>(ws, L.v0);
    uint32_t *k1 = at<uint32_t>(ws, L.k1), *v1 = at<uint32_t>(ws, L.v1);
    const uint32_t *sorted_keys = reinterpret_cast<const uint32_t *>(colidx);
    if (E > 0) {
        int bits = 1;
        while (bits < 32 && ((int64_t)1 << bits) < n_src) ++bits;
        const int passes = (bits + 7) / 8;
        const uint32_t *kin = reinterpret_cast<const uint32_t *>(colidx);
        const uint32_t *vin = nullptr;
        SortPasses sp{};
        sp.passes = passes;
        for (int p = 0; p < passes; ++p) {
            uint32_t *ko = (p & 1) ? k1 : k0;
            uint32_t *vo = (p == passes - 1) ? reinterpret_cast<uint32_t *>(g->perm) : ((p & 1) ? v1 : v0);
            sp.kin[p] = kin; sp.vin[p] = vin; sp.kout[p] = ko; sp.vout[p] = vo;
            kin = ko; vin = vo;
        }
        if ((s = radix_sort(sp, E, t, st)) != GT_OK) return fail(s);
        sorted_keys = kin;
    }
    if (n_src >= 0) {
        k_boundaries<<<nblocks(E + 1), PT, 0, st>>>(sorted_keys, E, n_src, g->rowptr_t);
        PLAN_LAUNCH("k_boundaries");
    }
    if (n_src > 0) {
        k_row_degrees<<<nblocks(n_src), PT, 0, st>>>(g->rowptr_t, n_src, g->out_deg, nullptr, nullptr);
        PLAN_LAUNCH("k_row_degrees(out)");
    }
    if (E > 0) {
        // the sort's ping-pong buffers are dead from here on; three of them hold the coefficients
        g->coef_sym_f = g->dinv ? reinterpret_cast<float *>(v0) : nullptr;
        g->coef_sym_b = g->dinv ? reinterpret_cast<float *>(v1) : nullptr;
        g->coef_mean_b = reinterpret_cast<float *>(k0);
        k_transposed_entries<<<nblocks(E), PT, 0, st>>>(rowptr, n_dst, g->perm, E, colidx, ew, g->dinv, g->rdeg,
                                                        g->colidx_t, g->ew_t, g->coef_sym_f, g->coef_sym_b,
                                                        g->coef_mean_b);
        PLAN_LAUNCH("k_transposed_entries");
    }
    // work-list sizes of both directions, read back once
    int32_t *d_counts = at<int32_t>(ws, L.counts);
    int32_t h_counts[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    g->chunk = gt_chunk_for(E);
    if ((s = count_direction(rowptr, n_dst, g->chunk, ws, L, false, d_counts, st)) != GT_OK) return fail(s);
    if ((s = count_direction(g->rowptr_t, n_src, g->chunk, ws, L, true, d_counts + 4, st)) != GT_OK) return fail(s);
    PLAN_HIP(hipMemcpyAsync(h_counts, d_counts, 8 * 4, hipMemcpyDeviceToHost, st));
    PLAN_HIP(hipStreamSynchronize(st));
    g->fwd.rowptr = rowptr; g->fwd.nbr = colidx; g->fwd.wt = ew; g->fwd.n_rows = n_dst;
    g->fwd.coef_sym = g->coef_sym_f;
    g->fwd.n_items = h_counts[0]; g->fwd.n_partials = h_counts[1]; g->fwd.n_splits = h_counts[2];
    g->fwd.items = at<gt_item>(ws, L.items_f); g->fwd.splits = at<gt_split>(ws, L.splits_f);
    if (g->fwd.n_items > max_items(n_dst, E) || g->fwd.n_splits > max_splits(E))
        return fail(gt_fail(GT_ERR_INTERNAL, "gt_graph_create: forward work list exceeds its bound (is rowptr valid?)"));
    g->bwd.rowptr = g->rowptr_t; g->bwd.nbr = g->colidx_t; g->bwd.wt = g->ew_t; g->bwd.n_rows = n_src;
    g->bwd.coef_sym = g->coef_sym_b; g->bwd.coef_mean = g->coef_mean_b;
    g->bwd.n_items = h_counts[4]; g->bwd.n_partials = h_counts[5]; g->bwd.n_splits = h_counts[6];
    g->bwd.items = at<gt_item>(ws, L.items_b); g->bwd.splits = at<gt_split>(ws, L.splits_b);
    if (g->bwd.n_items > max_items(n_src, E) || g->bwd.n_splits > max_splits(E))
        return fail(gt_fail(GT_ERR_INTERNAL, "gt_graph_create: transposed work list exceeds its bound"));
    if ((s = build_direction(rowptr, colidx, n_src, n_dst, g->chunk, g->fwd.n_items, ws, L, false,
                             at<gt_item>(ws, L.items_f), at<gt_split>(ws, L.splits_f), st)) != GT_OK) return fail(s);
    if ((s = build_direction(g->rowptr_t, g->colidx_t, n_dst, n_src, g->chunk, g->bwd.n_items, ws, L, true,
                             at<gt_item>(ws, L.items_b), at<gt_split>(ws, L.splits_b), st)) != GT_OK) return fail(s);
    PLAN_HIP(hipStreamSynchronize(st));
#undef PLAN_HIP
#undef PLAN_LAUNCH
    *out = g;
    return GT_OK;
}

extern "C" gt_status gt_graph_destroy(gt_graph *g) {
    delete g;
    return GT_OK;
}

extern "C" gt_status gt_graph_outputs(const gt_graph *g, const int32_t **in_deg, const int32_t **out_deg,
                                      const int32_t **rowptr_t, const int32_t **colidx_t, const int32_t **perm) {
    if (!g) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_outputs: g is null");
    if (in_deg) *in_deg = g->in_deg;
    if (out_deg) *out_deg = g->out_deg;
    if (rowptr_t) *rowptr_t = g->rowptr_t;
    if (colidx_t) *colidx_t = g->colidx_t;
    if (perm) *perm = g->perm;
    return GT_OK;
}

extern "C" gt_status gt_graph_info(const gt_graph *g, int64_t *n_dst, int64_t *n_src, int64_t *n_edges,
                                   int64_t *fwd_items, int64_t *fwd_split_rows, int64_t *bwd_items,
                                   int64_t *bwd_split_rows) {
    if (!g) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_info: g is null");
    if (n_dst) *n_dst = g->n_dst;
    if (n_src) *n_src = g->n_src;
    if (n_edges) *n_edges = g->n_edges;
    if (fwd_items) *fwd_items = g->fwd.n_items;
    if (fwd_split_rows) *fwd_split_rows = g->fwd.n_splits;
    if (bwd_items) *bwd_items = g->bwd.n_items;
    if (bwd_split_rows) *bwd_split_rows = g->bwd.n_splits;
    return GT_OK;
}

extern "C" gt_status gt_graph_validate(const gt_graph *g, int64_t *n_violations, void *stream) {
    if (!g || !n_violations) return gt_fail(GT_ERR_INVALID_ARG, "gt_graph_validate: null argument");
    hipStream_t st = (hipStream_t)stream;
    GT_HIP(hipMemsetAsync(g->vcount, 0, 8, st));
    const int64_t n = (g->n_edges > g->n_dst ? g->n_edges : g->n_dst);
    k_validate<<<nblocks(n > 0 ? n : 1), PT, 0, st>>>(g->rowptr, g->colidx, g->n_dst, g->n_src, g->n_edges, g->vcount);
    GT_LAUNCH_CHECK("k_validate");
    unsigned long long h = 0;
    GT_HIP(hipMemcpyAsync(&h, g->vcount, 8, hipMemcpyDeviceToHost, st));
    GT_HIP(hipStreamSynchronize(st));
    *n_violations = (int64_t)h;
    return GT_OK;
}
