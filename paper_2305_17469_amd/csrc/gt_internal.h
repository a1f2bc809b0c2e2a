// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gt.h"

// fp32 -> bf16, round to nearest even, NaN stays NaN: gfx950 converts a pair in one instruction
// (v_cvt_pk_bf16_f32), which is what the vector conversion below compiles to.  For every non-NaN
// input the result is the one of the integer form  (u + 0x7fff + ((u >> 16) & 1)) >> 16.
typedef __bf16 gt_bf16x2 __attribute__((ext_vector_type(2)));
typedef float gt_f32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t gt_pack_bf16(float lo, float hi) {   // lo in bits 0..15, hi in bits 16..31
    const gt_f32x2 v = {lo, hi};
    const gt_bf16x2 r = __builtin_convertvector(v, gt_bf16x2);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}
__device__ inline uint32_t gt_to_bf16(float f) { return gt_pack_bf16(f, 0.0f) & 0xffffu; }

// Work decomposition of one aggregation direction.  A row with more than 1.5 x chunk entries is
// cut into chunks of `chunk` entries; every chunk becomes a work item that writes an fp32
// partial row, and a second kernel adds a row's partials in chunk order.  All other rows are
// one item each and are written directly.  Items are ordered longest first.
// The chunk is 512 entries on large graphs and shrinks (down to 64) on small ones, so that a
// small graph with a few long rows still yields enough items to occupy the GPU.
#define GT_CHUNK_MAX 512
#define GT_CHUNK_MIN 64
static inline int gt_chunk_for(int64_t n_edges) {
    int c = GT_CHUNK_MAX;
    while (c > GT_CHUNK_MIN && n_edges / c < 4096) c >>= 1;
    return c;
}
static inline int gt_split_min(int chunk) { return chunk + chunk / 2; }

struct gt_item {   // 16 bytes, loaded as one int4
    int32_t row;   // output row
    int32_t e0;    // first entry
    int32_t e1;    // one past the last entry
    int32_t slot;  // < 0: write the output row;  >= 0: write partial row `slot`
};

struct gt_split {  // one per split row
    int32_t row;
    int32_t first;  // first partial slot
    int32_t count;  // number of partial slots
    int32_t pad;
};

struct gt_sched {
    const int32_t *rowptr = nullptr;  // [n_rows + 1]
    const int32_t *nbr = nullptr;     // [E] neighbour (gathered row) of every entry
    const float *wt = nullptr;        // [E] per-entry weight or null
    const float *coef_sym = nullptr;  // [E] w_e / sqrt(d(u) d(v)) (square graphs), in this direction's entry order
    const float *coef_mean = nullptr; // [E] w_e / indeg(dst) (transposed direction only)
    const gt_item *items = nullptr;
    const gt_split *splits = nullptr;
    int64_t n_rows = 0, n_items = 0, n_splits = 0, n_partials = 0;
};

struct gt_graph {
    int64_t n_dst = 0, n_src = 0, n_edges = 0;
    int chunk = GT_CHUNK_MAX;   // entries per work item of a split row
    const int32_t *rowptr = nullptr, *colidx = nullptr;
    const float *ew = nullptr;
    // plan (device, inside the caller's workspace)
    int32_t *in_deg = nullptr, *out_deg = nullptr, *rowptr_t = nullptr, *colidx_t = nullptr, *perm = nullptr;
    float *ew_t = nullptr;
    float *dinv = nullptr;  // in_deg^-1/2 (square graphs only), 0 where the degree is 0
    float *rdeg = nullptr;  // 1 / in_deg, 0 where the degree is 0
    float *coef_sym_f = nullptr, *coef_sym_b = nullptr, *coef_mean_b = nullptr;   // per-entry coefficients
    unsigned long long *vcount = nullptr;  // device counter of gt_graph_validate
    gt_sched fwd, bwd;
};

void gt_set_error(const char *fmt, ...);
gt_status gt_fail(gt_status s, const char *fmt, ...);
gt_status gt_hip_fail(hipError_t e, const char *what);

#define GT_HIP(call)                                                \
    do {                                                            \
        hipError_t e__ = (call);                                    \
        if (e__ != hipSuccess) return gt_hip_fail(e__, #call);      \
    } while (0)

#define GT_LAUNCH_CHECK(what)                                       \
    do {                                                            \
        hipError_t e__ = hipGetLastError();                         \
        if (e__ != hipSuccess) return gt_hip_fail(e__, what);       \
    } while (0)

static inline size_t gt_align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

static inline size_t gt_dtype_size(gt_dtype t) { return t == GT_BF16 ? 2 : 4; }

// internal entry points used across translation units
gt_status gt_aggregate_run(const gt_graph *g, bool transposed, gt_reduce reduce, gt_dtype in_dtype,
                           gt_dtype out_dtype, int64_t F, const void *X, int64_t ldx, void *Y, int64_t ldy,
                           const float *bias, gt_act act, void *ws, size_t ws_bytes, hipStream_t stream,
                           bool traced = true, const void *mask = nullptr, int64_t ldmask = 0, bool pad_out = false);
// pad_out: the output rows are padded and the padding is the library's to write (see gt_layer_desc.pad_writable)

size_t gt_aggregate_ws_bytes(const gt_graph *g, int64_t F);

// fused aggregation-first forward (gt_fused.hip): Y = act((A X) W + b) without writing A X
bool gt_fused_applicable(gt_dtype dtype, int64_t in_dim, int64_t out_dim);
gt_status gt_fused_run(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t fi, int64_t fo, const void *X, int64_t ldx,
                       const void *W, int64_t ldw, const float *bias, gt_act act, void *Y, int64_t ldy, void *ws,
                       size_t ws_bytes, hipStream_t st);
