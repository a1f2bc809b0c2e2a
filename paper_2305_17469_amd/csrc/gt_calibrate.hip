// Fitting the cost-model coefficients on the device (paper: "DKP cost model and parameters":
// the coefficients depend on the system, so they are fitted by least squares from measured
// kernel times at the start of training and reused afterwards).
//
// The measurements are synthetic: a regular random graph and dense matrices built inside the
// caller's workspace.  Each kernel-time model has two unknowns,
//     t_aggr = gamma * (F * E) + delta * (F * n_out),    t_comb = alpha * (rows*in*out) + beta * (rows*width),
// and is fitted through the 2x2 normal equations of its samples.  The backward combination
// samples are the two products a backward pass runs: dZ W^T and the weight gradient X^T dZ
// (reduction over the rows).  The floor of an aggregation's time is measured directly: the time
// per launch of a narrow aggregation on a graph of 1,024 vertices, back to back on the stream.
#include <math.h>

#include "gt_internal.h"
#include "gt_combine.h"

namespace {

constexpr int64_t CAL_N = 1 << 16;      // vertices
constexpr int64_t CAL_DMAX = 32;        // largest degree tried
constexpr int64_t CAL_FMAX = 256;       // widest feature row tried

__global__ void k_cal_graph(int32_t *rowptr, int32_t *colidx, int64_t n, int64_t d) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e <= n) rowptr[e] = (int32_t)(e * d);
    if (e < n * d) {
        uint64_t x = (uint64_t)e * 0x9E3779B97F4A7C15ull + 0x632BE59BD9B4E019ull;
        x ^= x >> 29; x *= 0xBF58476D1CE4E5B9ull; x ^= x >> 32;
        colidx[e] = (int32_t)(x % (uint64_t)n);
    }
}

__global__ void k_cal_fill(float *p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (float)((i * 2654435761u >> 8) & 1023) * (1.0f / 1024.0f) - 0.5f;
}

struct Fit2 {   // least squares for t = a*x + b*y, constrained to a, b >= 0
    double sxx = 0, sxy = 0, syy = 0, sxt = 0, syt = 0;
    void add(double x, double y, double t) { sxx += x * x; sxy += x * y; syy += y * y; sxt += x * t; syt += y * t; }
    void solve(double *a, double *b) const {
        const double det = sxx * syy - sxy * sxy;
        double A = 0, B = 0;
        if (fabs(det) > 1e-300) { A = (sxt * syy - syt * sxy) / det; B = (syt * sxx - sxt * sxy) / det; }
        if (!(A >= 0) || !(B >= 0) || fabs(det) <= 1e-300) {   // fall back to the better one-term fit
            const double a1 = sxx > 0 ? sxt / sxx : 0, b1 = syy > 0 ? syt / syy : 0;
            if (!(A >= 0)) { A = 0; B = b1 > 0 ? b1 : 0; } else { B = 0; A = a1 > 0 ? a1 : 0; }
        }
        *a = A; *b = B;
    }
};

struct CalLayout { size_t rowptr, colidx, plan, X, Y, W, agg_ws, total; size_t plan_bytes; };

gt_status cal_layout(CalLayout *L) {
    size_t off = 0;
    auto take = [&](size_t b) { size_t o = off; off += gt_align_up(b); return o; };
    size_t plan = 0;
    gt_status s = gt_graph_plan_size(CAL_N, CAL_N, CAL_N * CAL_DMAX, 0, &plan);
    if (s != GT_OK) return s;
    L->rowptr = take((size_t)(CAL_N + 1) * 4);
    L->colidx = take((size_t)CAL_N * CAL_DMAX * 4);
    L->plan_bytes = plan;
    L->plan = take(plan);
    L->X = take((size_t)CAL_N * CAL_FMAX * 4);
    L->Y = take((size_t)CAL_N * CAL_FMAX * 4);
    L->W = take((size_t)CAL_FMAX * CAL_FMAX * 4);
    L->agg_ws = take((size_t)64 << 20);
    L->total = off;
    return GT_OK;
}

template <typename F>
gt_status time_it(F &&fn, hipStream_t st, double *seconds) {
    hipEvent_t e0, e1;
    GT_HIP(hipEventCreate(&e0));
    GT_HIP(hipEventCreate(&e1));
    gt_status s = fn();   // warm-up
    const int reps = 3;
    if (s == GT_OK) {
        (void)hipEventRecord(e0, st);
        for (int i = 0; i < reps && s == GT_OK; ++i) s = fn();
        (void)hipEventRecord(e1, st);
        (void)hipEventSynchronize(e1);
        float ms = 0;
        (void)hipEventElapsedTime(&ms, e0, e1);
        *seconds = (double)ms * 1e-3 / reps;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return s;
}

}  // namespace

extern "C" gt_status gt_calibrate_ws_size(size_t *ws_bytes) {
    if (!ws_bytes) return gt_fail(GT_ERR_INVALID_ARG, "gt_calibrate_ws_size: null");
    CalLayout L;
    gt_status s = cal_layout(&L);
    if (s != GT_OK) return s;
    *ws_bytes = L.total;
    return GT_OK;
}

extern "C" gt_status gt_calibrate_dtype(gt_dtype dtype, void *ws, size_t ws_bytes, gt_cost_coeffs *fitted,
                                        void *stream) {
    if (dtype != GT_F32 && dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "gt_calibrate_dtype: unknown dtype");
    CalLayout L;
    gt_status s = cal_layout(&L);
    if (s != GT_OK) return s;
    if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "gt_calibrate: ws null or not 256-byte aligned");
    if (ws_bytes < L.total) return gt_fail(GT_ERR_WORKSPACE, "gt_calibrate: ws_bytes %zu < required %zu", ws_bytes, L.total);
    hipStream_t st = (hipStream_t)stream;
    char *base = static_cast<char *>(ws);
    int32_t *rowptr = reinterpret_cast<int32_t *>(base + L.rowptr);
    int32_t *colidx = reinterpret_cast<int32_t *>(base + L.colidx);
    // The buffers are sized for fp32 and filled with fp32 values in (-0.5, 0.5); read as bf16 the
    // same bytes are finite values of the same range (the timing does not depend on them).
    float *Xf = reinterpret_cast<float *>(base + L.X), *Yf = reinterpret_cast<float *>(base + L.Y);
    float *Wf = reinterpret_cast<float *>(base + L.W);
    void *X = Xf, *Y = Yf, *W = Wf;
    const int64_t nx = CAL_N * CAL_FMAX;
    k_cal_fill<<<(unsigned)((nx + 255) / 256), 256, 0, st>>>(Xf, nx);
    k_cal_fill<<<(unsigned)((nx + 255) / 256), 256, 0, st>>>(Yf, nx);
    k_cal_fill<<<(unsigned)((CAL_FMAX * CAL_FMAX + 255) / 256), 256, 0, st>>>(Wf, CAL_FMAX * CAL_FMAX);
    GT_LAUNCH_CHECK("k_cal_fill");

    Fit2 agg_f, agg_b, gemm_f, gemm_b;
    // rows of 2, 8 and 32 entries: the per-row term (delta) is what a graph of very short rows is bound by
    const int64_t degs[3] = {2, 8, CAL_DMAX};
    const int64_t widths[3] = {32, 128, 256};
    for (int64_t d : degs) {
        const int64_t E = CAL_N * d;
        k_cal_graph<<<(unsigned)((E + 256) / 256), 256, 0, st>>>(rowptr, colidx, CAL_N, d);
        GT_LAUNCH_CHECK("k_cal_graph");
        gt_graph *g = nullptr;
        s = gt_graph_create(&g, CAL_N, CAL_N, E, rowptr, colidx, nullptr, base + L.plan, L.plan_bytes, st);
        if (s != GT_OK) return s;
        for (int64_t F : widths) {
            double t = 0;
            s = time_it([&] { return gt_aggregate_run(g, false, GT_SUM, dtype, dtype, F, X, CAL_FMAX, Y, CAL_FMAX, nullptr,
                                                      GT_ACT_NONE, base + L.agg_ws, (size_t)64 << 20, st); }, st, &t);
            if (s != GT_OK) { gt_graph_destroy(g); return s; }
            agg_f.add((double)F * E, (double)F * CAL_N, t);
            s = time_it([&] { return gt_aggregate_run(g, true, GT_SUM, dtype, dtype, F, Y, CAL_FMAX, X, CAL_FMAX, nullptr,
                                                      GT_ACT_NONE, base + L.agg_ws, (size_t)64 << 20, st); }, st, &t);
            if (s != GT_OK) { gt_graph_destroy(g); return s; }
            agg_b.add((double)F * E, (double)F * CAL_N, t);
        }
        gt_graph_destroy(g);
    }
    const int64_t shapes[5][2] = {{64, 64}, {256, 64}, {64, 256}, {256, 256}, {128, 16}};
    for (auto &sh : shapes) {
        const int64_t in = sh[0], out = sh[1];
        double t = 0;
        s = time_it([&] { return gt_gemm_run("gt_calibrate", dtype, 0, 0, CAL_N, out, in, X, CAL_FMAX, W, out, nullptr, nullptr,
                                             GT_ACT_NONE, nullptr, 0, Y, CAL_FMAX, dtype, nullptr, 0, st); }, st, &t);
        if (s != GT_OK) return s;
        gemm_f.add((double)CAL_N * in * out, (double)CAL_N * out, t);
        s = time_it([&] { return gt_gemm_run("gt_calibrate", dtype, 0, 1, CAL_N, in, out, Y, CAL_FMAX, W, out, nullptr, nullptr,
                                             GT_ACT_NONE, nullptr, 0, X, CAL_FMAX, dtype, nullptr, 0, st); }, st, &t);
        if (s != GT_OK) return s;
        gemm_b.add((double)CAL_N * in * out, (double)CAL_N * in, t);
        // the weight gradient X^T dZ: [in, out] fp32 over CAL_N rows, split over workgroups (partials in agg_ws)
        s = time_it([&] { return gt_gemm_run("gt_calibrate", dtype, 1, 0, in, out, CAL_N, X, CAL_FMAX, Y, CAL_FMAX, nullptr,
                                             nullptr, GT_ACT_NONE, nullptr, 0, Wf, out, GT_F32, base + L.agg_ws,
                                             (size_t)64 << 20, st); }, st, &t);
        if (s != GT_OK) return s;
        gemm_b.add((double)CAL_N * in * out, (double)CAL_N * in, t);
    }
    // floor of an aggregation launch: 1,024 vertices, 8 neighbours each, 16 columns
    double floor_s = 0.0;
    {
        const int64_t n = 1024, d = 8, E = n * d;
        k_cal_graph<<<(unsigned)((E + 256) / 256), 256, 0, st>>>(rowptr, colidx, n, d);
        GT_LAUNCH_CHECK("k_cal_graph");
        gt_graph *g = nullptr;
        s = gt_graph_create(&g, n, n, E, rowptr, colidx, nullptr, base + L.plan, L.plan_bytes, st);
        if (s != GT_OK) return s;
        double best = 1e30;
        for (int rep = 0; rep < 3 && s == GT_OK; ++rep) {   // the smallest of three: launch jitter only adds
            double t = 0;
            s = time_it([&] { return gt_aggregate_run(g, false, GT_SUM, dtype, dtype, 16, X, CAL_FMAX, Y, CAL_FMAX, nullptr,
                                                      GT_ACT_NONE, base + L.agg_ws, (size_t)64 << 20, st); }, st, &t);
            if (t < best) best = t;
        }
        gt_graph_destroy(g);
        if (s != GT_OK) return s;
        floor_s = best < 1e-6 ? 1e-6 : (best > 2e-5 ? 2e-5 : best);
    }
    gt_cost_coeffs c;
    c.aggr_floor = floor_s;
    gemm_f.solve(&c.alpha_fwd, &c.beta_fwd);
    gemm_b.solve(&c.alpha_bwd, &c.beta_bwd);
    agg_f.solve(&c.gamma_fwd, &c.delta_fwd);
    agg_b.solve(&c.gamma_bwd, &c.delta_bwd);
    s = gt_cost_set_dtype(dtype, &c);
    if (s != GT_OK) return s;
    if (fitted) *fitted = c;
    return GT_OK;
}

extern "C" gt_status gt_calibrate(void *ws, size_t ws_bytes, gt_cost_coeffs *fitted, void *stream) {
    gt_status s = gt_calibrate_dtype(GT_BF16, ws, ws_bytes, nullptr, stream);
    if (s != GT_OK) return s;
    return gt_calibrate_dtype(GT_F32, ws, ws_bytes, fitted, stream);
}
