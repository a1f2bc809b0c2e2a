// Optional kernel timing: when enabled, the library brackets each aggregation kernel launch and
// each combination kernel launch with HIP events recorded on the launch's own stream, so a
// caller can read per-kernel durations of the very launches it timed as a whole (the paper
// measures GPU kernel time the same way, with a profiler, to exclude framework overhead).
// Off by default; costs two event records per launch when on.
#include <vector>

#include "gt_internal.h"
#include "gt_trace.h"

namespace {
struct Rec { hipEvent_t a, b; int kind; int64_t width, rows, work; int V = 0, G = 0, NP = 0, U = 0, MK = 0; };
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
bool g_on = false;

hipEvent_t take_event() {
    if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

bool gt_trace_on() { return g_on; }

int gt_trace_open(int kind, int64_t width, int64_t rows, int64_t work, hipStream_t st) {
    if (!g_on || kind < 0) return -1;
    Rec r{};
    r.a = take_event(); r.b = take_event(); r.kind = kind; r.width = width; r.rows = rows; r.work = work;
    if (!r.a || !r.b) return -1;
    if (hipEventRecord(r.a, st) != hipSuccess) return -1;
    g_recs.push_back(r);
    return (int)g_recs.size() - 1;
}

void gt_trace_variant(int id, int V, int G, int NP, int U, int masked) {
    if (id < 0 || id >= (int)g_recs.size()) return;
    g_recs[id].V = V; g_recs[id].G = G; g_recs[id].NP = NP; g_recs[id].U = U; g_recs[id].MK = masked;
}

void gt_trace_close(int id, hipStream_t st) {
    if (id < 0 || id >= (int)g_recs.size()) return;
    (void)hipEventRecord(g_recs[id].b, st);
}

extern "C" gt_status gt_trace_enable(int on) {
    g_on = on != 0;
    return GT_OK;
}

extern "C" gt_status gt_trace_reset(void) {
    for (Rec &r : g_recs) { g_pool.push_back(r.a); g_pool.push_back(r.b); }
    g_recs.clear();
    return GT_OK;
}

extern "C" gt_status gt_trace_count(int64_t *n) {
    if (!n) return gt_fail(GT_ERR_INVALID_ARG, "gt_trace_count: null");
    *n = (int64_t)g_recs.size();
    return GT_OK;
}

extern "C" gt_status gt_trace_get(int64_t i, int *kind, int64_t *width, int64_t *rows, int64_t *work, double *ms) {
    if (i < 0 || i >= (int64_t)g_recs.size()) return gt_fail(GT_ERR_INVALID_ARG, "gt_trace_get: index out of range");
    const Rec &r = g_recs[(size_t)i];
    if (kind) *kind = r.kind;
    if (width) *width = r.width;
    if (rows) *rows = r.rows;
    if (work) *work = r.work;
    if (ms) {
        GT_HIP(hipEventSynchronize(r.b));
        float t = 0.0f;
        GT_HIP(hipEventElapsedTime(&t, r.a, r.b));
        *ms = (double)t;
    }
    return GT_OK;
}

extern "C" gt_status gt_trace_get_variant(int64_t i, int *V, int *G, int *NP, int *U, int *masked) {
    if (i < 0 || i >= (int64_t)g_recs.size()) return gt_fail(GT_ERR_INVALID_ARG, "gt_trace_get_variant: index out of range");
    const Rec &r = g_recs[(size_t)i];
    if (V) *V = r.V;
    if (G) *G = r.G;
    if (NP) *NP = r.NP;
    if (U) *U = r.U;
    if (masked) *masked = r.MK;
    return GT_OK;
}
