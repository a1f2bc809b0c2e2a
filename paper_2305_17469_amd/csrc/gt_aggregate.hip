// Neighbour aggregation (the paper's Pull primitive without per-call weights) and its derivative:
// host side of gt_aggregate_fwd / gt_aggregate_bwd.  The kernels live in gt_aggregate_kernel.h.
#include "gt_aggregate_kernel.h"

// tables above this size are gathered in column passes (the MI355X last-level cache holds 256 MiB)
static const int64_t GT_COLUMN_PASS_TABLE_BYTES = (int64_t)256 << 20;
// ... and only when a pass gathers about a gigabyte or more: below that the extra launches cost more
// than the passes save (a sampled block with 4,353-wide rows would run 68 launches of 11 MB each)
static const int64_t GT_COLUMN_PASS_MIN_EDGES = (int64_t)4 << 20;

size_t gt_aggregate_ws_bytes(const gt_graph *g, int64_t F) {
    const int64_t ldp = (F + 7) / 8 * 8;
    const int64_t parts = g->fwd.n_partials > g->bwd.n_partials ? g->fwd.n_partials : g->bwd.n_partials;
    return gt_align_up((size_t)parts * (size_t)ldp * 4);
}

gt_status gt_aggregate_run(const gt_graph *g, bool transposed, gt_reduce reduce, gt_dtype in_dtype, gt_dtype out_dtype,
                           int64_t F, const void *X, int64_t ldx, void *Y, int64_t ldy, const float *bias, gt_act act,
                           void *ws, size_t ws_bytes, hipStream_t st, bool traced, const void *mask, int64_t ldmask, bool pad_out) {
    const char *fn = transposed ? "gt_aggregate_bwd" : "gt_aggregate_fwd";
    if (!g) return gt_fail(GT_ERR_INVALID_ARG, "%s: g is null", fn);
    if (F < 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: F < 0", fn);
    if (reduce != GT_SUM && reduce != GT_MEAN && reduce != GT_SYMNORM)
        return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown reduce %d", fn, (int)reduce);
    if (in_dtype != GT_F32 && in_dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown dtype", fn);
    if (in_dtype != out_dtype) return gt_fail(GT_ERR_UNSUPPORTED, "%s: input and output dtype must match", fn);
    if (reduce == GT_SYMNORM && g->n_dst != g->n_src)
        return gt_fail(GT_ERR_UNSUPPORTED, "%s: GT_SYMNORM needs a square graph (n_src == n_dst)", fn);
    const gt_sched &sc = transposed ? g->bwd : g->fwd;
    const int64_t n_in = transposed ? g->n_dst : g->n_src;
    const int64_t n_out = sc.n_rows;
    if (F == 0 || n_out == 0) return GT_OK;
    if (!Y) return gt_fail(GT_ERR_INVALID_ARG, "%s: output pointer is null", fn);
    if (!X && n_in > 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: input pointer is null", fn);
    if (ldx < F || ldy < F) return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension smaller than F", fn);
    const size_t es = gt_dtype_size(in_dtype);
    if (((uintptr_t)X % es) || ((uintptr_t)Y % es)) return gt_fail(GT_ERR_INVALID_ARG, "%s: pointer misaligned for dtype", fn);
    {
        const char *xb = (const char *)X, *xe = xb + (size_t)n_in * ldx * es;
        const char *yb = (const char *)Y, *ye = yb + (size_t)n_out * ldy * es;
        if (X && xb < ye && yb < xe) return gt_fail(GT_ERR_INVALID_ARG, "%s: input and output overlap", fn);
    }
    const size_t need = sc.n_partials > 0 ? gt_aggregate_ws_bytes(g, F) : 0;
    if (need > 0) {
        if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: ws null or not 256-byte aligned", fn);
        if (ws_bytes < need) return gt_fail(GT_ERR_WORKSPACE, "%s: ws_bytes %zu < required %zu", fn, ws_bytes, need);
    }

    AggArgs a{};
    a.items = sc.items; a.n_items = sc.n_items;
    a.rowptr = sc.rowptr; a.nbr = sc.nbr;
    a.coef = sc.wt; a.post_mode = 0;
    if (reduce == GT_MEAN) {
        if (!transposed) a.post_mode = 2;   // divide by the destination's in-degree (exact for ones)
        else a.coef = sc.coef_mean;         // w_e / indeg(dst), stored per transposed entry
    } else if (reduce == GT_SYMNORM) {
        a.coef = sc.coef_sym;               // w_e / sqrt(d(u) d(v)), stored per entry
    }
    a.bias = bias; a.relu = (act == GT_ACT_RELU);
    a.mask = mask; a.ldmask = ldmask;
    a.pad_out = pad_out ? 1 : 0;
    if (mask && ldmask < F) return gt_fail(GT_ERR_INVALID_ARG, "%s: mask leading dimension smaller than F", fn);
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy; a.F = F;
    a.partials = static_cast<float *>(ws); a.ldp = (F + 7) / 8 * 8;
    a.splits = sc.splits; a.n_splits = sc.n_splits;
    a.table_bytes = n_in * ldx * (int64_t)es;
    a.trace_kind = !traced ? -1 : transposed ? GT_TRACE_AGG_BWD : GT_TRACE_AGG_FWD;
    a.n_rows = n_out; a.n_edges = g->n_edges;

    const int ve = in_dtype == GT_F32 ? 4 : 8;
    const bool vec = aligned16(X) && aligned16(Y) && (ldx % ve == 0) && (ldy % ve == 0) &&
                     (!mask || (aligned16(mask) && ldmask % ve == 0));
    // A gathered table far larger than the last-level cache, with rows of 512 bytes or more, is
    // aggregated in column passes of 256 bytes, one launch each: every pass gathers from a table
    // slice a fraction of the size, so more of the popular rows stay cached, and the narrow launch
    // shape keeps more loads in flight (measured on MI355X: 1 GiB bf16 table, 512-byte rows,
    // 3.93 -> 3.65 ms; 4.3 GB fp32 table, 4 KB rows, 12.0 -> 10.2 ms).  Results are unchanged:
    // columns are independent.
    int64_t pass = F;
    if (vec && a.table_bytes > GT_COLUMN_PASS_TABLE_BYTES && F * (int64_t)es >= 512 && g->n_edges >= GT_COLUMN_PASS_MIN_EDGES)
        pass = 256 / (int64_t)es;
    // what one launch gathers from: the slice of a pass, not the whole table (picks the unroll)
    if (pass < F) a.table_bytes = n_in * pass * (int64_t)es;
    for (int64_t c0 = 0; c0 < F; c0 += pass) {
        const int64_t fp = F - c0 < pass ? F - c0 : pass;
        a.X = static_cast<const char *>(X) + c0 * es;
        a.Y = static_cast<char *>(Y) + c0 * es;
        a.F = fp;
        a.ldp = (fp + 7) / 8 * 8;
        a.bias = bias ? bias + c0 : nullptr;
        a.mask = mask ? static_cast<const char *>(mask) + c0 * es : nullptr;
        gt_status s;
        if (in_dtype == GT_F32) s = vec ? dispatch<float, 4>(a, st) : dispatch<float, 1>(a, st);
        else s = vec ? dispatch<bf16_t, 8>(a, st) : dispatch<bf16_t, 1>(a, st);
        if (s != GT_OK) return s;
    }
    return GT_OK;
}

extern "C" gt_status gt_aggregate_ws_size(const gt_graph *g, int64_t F, size_t *ws_bytes) {
    if (!g || !ws_bytes) return gt_fail(GT_ERR_INVALID_ARG, "gt_aggregate_ws_size: null argument");
    if (F < 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_aggregate_ws_size: F < 0");
    const bool any = g->fwd.n_partials > 0 || g->bwd.n_partials > 0;
    *ws_bytes = any ? gt_aggregate_ws_bytes(g, F) : 0;
    return GT_OK;
}

extern "C" gt_status gt_aggregate_fwd(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t F, const void *X,
                                      int64_t ldx, void *Y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
    return gt_aggregate_run(g, false, reduce, dtype, dtype, F, X, ldx, Y, ldy, nullptr, GT_ACT_NONE, ws, ws_bytes,
                            (hipStream_t)stream);
}

extern "C" gt_status gt_aggregate_bwd(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t F, const void *dY,
                                      int64_t lddy, void *dX, int64_t lddx, void *ws, size_t ws_bytes, void *stream) {
    return gt_aggregate_run(g, true, reduce, dtype, dtype, F, dY, lddy, dX, lddx, nullptr, GT_ACT_NONE, ws, ws_bytes,
                            (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// gt_aggregate_fwd for callers that cannot allocate: the fp32 partial rows of the split long rows
// live in a fixed array inside the library instead of a caller workspace.
// ---------------------------------------------------------------------------------------------
#include <mutex>

#define GT_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
// No kernel names the array (they receive its address as an argument); the host-side reference in
// static_scratch() below is what makes the compiler keep it and export its device symbol.  (Marking
// it `used` as well leaves the device symbol with local binding, and the runtime's lookup fails.)
static __device__ __align__(256) unsigned char scratch[GT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int GT_MAX_DEVICES = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[GT_MAX_DEVICES] = {};   // device address of `scratch` on each device, looked up once

// `scratch` names a host-side stand-in here; its device address is different on every GPU and
// comes from hipGetSymbolAddress with that GPU current.
gt_status static_scratch(void **ptr) {
    int dev = -1;
    GT_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= GT_MAX_DEVICES) return gt_fail(GT_ERR_UNSUPPORTED, "gt_aggregate_fwd_static: device index %d", dev);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        GT_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255)) return gt_fail(GT_ERR_INTERNAL, "gt_aggregate_fwd_static: bad address of the static scratch");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return GT_OK;
}
}  // namespace

extern "C" gt_status gt_aggregate_static_capacity(size_t *bytes) {
    if (!bytes) return gt_fail(GT_ERR_INVALID_ARG, "gt_aggregate_static_capacity: null");
    *bytes = GT_STATIC_SCRATCH_BYTES;
    return GT_OK;
}

extern "C" gt_status gt_aggregate_fwd_static(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t F, const void *X,
                                             int64_t ldx, void *Y, int64_t ldy, void *stream) {
    if (!g) return gt_fail(GT_ERR_INVALID_ARG, "gt_aggregate_fwd_static: g is null");
    if (F < 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_aggregate_fwd_static: F < 0");
    const size_t need = g->fwd.n_partials > 0 ? gt_aggregate_ws_bytes(g, F) : 0;
    if (need > GT_STATIC_SCRATCH_BYTES)
        return gt_fail(GT_ERR_WORKSPACE, "gt_aggregate_fwd_static: %zu bytes of partial rows exceed the built-in %zu; "
                       "use gt_aggregate_fwd with a caller workspace", need, (size_t)GT_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (need > 0) {
        const gt_status s = static_scratch(&ws);
        if (s != GT_OK) return s;
    }
    // every partial slot is written by its work item before the second kernel reads it: nothing in
    // the array has to start at zero; kernel timing is off for this call (it would create events)
    return gt_aggregate_run(g, false, reduce, dtype, dtype, F, X, ldx, Y, ldy, nullptr, GT_ACT_NONE, ws,
                            GT_STATIC_SCRATCH_BYTES, (hipStream_t)stream, false);
}
