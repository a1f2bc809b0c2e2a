// Batch preparation on the GPU: neighbour sampling (S), renumbering (R), embedding lookup (K).
//
// Paper: Preliminaries "Preprocessing for GNNs" (what S, R and K compute: at most n distinct
// random neighbours per destination; new ids handed out from zero in first-met order) and the
// service-wide tensor scheduler's "High-performance preprocessing" (S/R/K/T as separate
// subtasks).  The paper's versions are host threads around a shared hash table, whose lock
// contention it has to schedule around.  With the whole graph in HBM the same results come
// from data-parallel integer kernels:
//   S  one wavefront per destination; the picks are the first `fanout` values of a keyed
//      permutation of the list positions, evaluated independently per lane (no state shared
//      between picks, so no table and no rejection loop);
//   R  a stable radix sort of (id, position) groups equal ids with their first position in
//      front; two scans turn "first position of each group" into the first-met numbering;
//   K  a row gather, 16 bytes per lane.
// Integer work: every result is exactly defined.
#include "gt_internal.h"
#include "gt_prims.h"

namespace {

constexpr uint32_t GOLD = 0x9E3779B9u;
constexpr int FEISTEL_ROUNDS = 6;
constexpr int SMALL_LIST = 64;   // lists up to one wavefront are ordered by per-position keys

__device__ __host__ inline uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

constexpr int PT = 256;
inline unsigned nblocks(int64_t n, int per = PT) { return (unsigned)((n + per - 1) / per); }

// ---------------------------------------------------------------------------------------------
// S
// ---------------------------------------------------------------------------------------------
__global__ void k_sample_counts(const int32_t *rowptr, int64_t n_vertices, const int32_t *dst, int64_t n_dst,
                                int32_t fanout, int32_t *cnt) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n_dst) return;
    int32_t c = 0;
    if (i < n_dst) {
        const int64_t v = dst[i];
        if (v >= 0 && v < n_vertices) {
            const int32_t d = rowptr[v + 1] - rowptr[v];
            c = d < fanout ? d : fanout;
        }
    }
    cnt[i] = c;   // entry n_dst is 0, so the exclusive scan ends with the total
}

__global__ void __launch_bounds__(PT) k_sample_pick(const int32_t *rowptr, const int32_t *colidx, int64_t n_vertices,
                                                    const int32_t *dst, int64_t n_dst, int32_t fanout, uint32_t skey,
                                                    const int32_t *out_rowptr, int32_t *out_nbr) {
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * (PT / 64) + (threadIdx.x >> 6);   // one wavefront per destination
    if (i >= n_dst) return;
    const int64_t v = dst[i];
    if (v < 0 || v >= n_vertices) return;
    const int32_t e0 = rowptr[v];
    const int32_t d = rowptr[v + 1] - e0;
    int32_t *out = out_nbr + out_rowptr[i];
    if (d <= fanout) {   // the whole list, list order
        for (int32_t t = lane; t < d; t += 64) out[t] = colidx[e0 + t];
        return;
    }
    const uint32_t rk = mix32(skey ^ (uint32_t)v);
    if (d <= SMALL_LIST) {
        // lane j holds position j; its rank among the keys is its place in the permutation
        const uint32_t key = mix32(rk + GOLD * (uint32_t)(lane + 1));
        int rank = 0;
        for (int s = 0; s < d; ++s) {
            const uint32_t ks = (uint32_t)__shfl((int)key, s, 64);
            rank += ks < key ? 1 : 0;
        }
        if (lane < d && rank < fanout) out[rank] = colidx[e0 + lane];
        return;
    }
    const int b = 32 - __clz((uint32_t)(d - 1));
    const int h = (b + 1) >> 1;
    const uint32_t mask = (1u << h) - 1u;
    uint32_t rkey[FEISTEL_ROUNDS];
#pragma unroll
    for (int r = 0; r < FEISTEL_ROUNDS; ++r) rkey[r] = mix32(rk + GOLD * (uint32_t)(r + 1));
    for (int32_t t = lane; t < fanout; t += 64) {
        uint32_t x = (uint32_t)t;
        do {   // cycle walking: x returns to a value < d because t < d lies on its cycle
            uint32_t L = x >> h, R = x & mask;
#pragma unroll
            for (int r = 0; r < FEISTEL_ROUNDS; ++r) {
                const uint32_t nr = L ^ (mix32(R ^ rkey[r]) & mask);
                L = R;
                R = nr;
            }
            x = (L << h) | R;
        } while (x >= (uint32_t)d);
        out[t] = colidx[e0 + (int32_t)x];
    }
}

// ---------------------------------------------------------------------------------------------
// R
// ---------------------------------------------------------------------------------------------
__global__ void k_concat_ids(const int32_t *dst, int64_t n_dst, const int32_t *picked, int64_t n, uint32_t *keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    keys[i] = (uint32_t)(i < n_dst ? dst[i] : picked[i - n_dst]);
}

// head[i] = 1 where a new id starts in the sorted order; first[pos] = 1 where position pos is the
// first occurrence of its id (the sort is stable, so the head of a group carries the smallest
// position).  Both arrays have n + 1 entries, the last one 0.
__global__ void k_mark_heads(const uint32_t *skeys, const uint32_t *spos, int64_t n, int32_t *head, int32_t *first) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    if (i == n) { head[n] = 0; first[n] = 0; return; }
    const int32_t hd = (i == 0 || skeys[i] != skeys[i - 1]) ? 1 : 0;
    head[i] = hd;
    first[spos[i]] = hd;
}

// group_lid[g] = new id of the g-th distinct id in sorted order = number of first occurrences
// before its first position
__global__ void k_group_ids(const uint32_t *skeys, const uint32_t *spos, int64_t n, const int32_t *head_scan,
                            const int32_t *first_scan, int32_t *group_lid, int32_t *src_global) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (head_scan[i + 1] == head_scan[i]) return;   // not a head
    const int32_t lid = first_scan[spos[i]];
    group_lid[head_scan[i]] = lid;
    src_global[lid] = (int32_t)skeys[i];
}

__global__ void k_emit_local(const uint32_t *spos, int64_t n, int64_t n_dst, const int32_t *head_scan,
                             const int32_t *first_scan, const int32_t *group_lid, int32_t *colidx_local,
                             int32_t *counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        counts[0] = first_scan[n];        // distinct ids in all
        counts[1] = first_scan[n_dst];    // distinct ids among the destinations
    }
    if (i >= n) return;
    const int64_t pos = spos[i];
    if (pos >= n_dst) colidx_local[pos - n_dst] = group_lid[head_scan[i + 1] - 1];
}

struct ReindexLayout {
    size_t keysA, keysB, valsA, valsB, head, first, group, hist, scan_tmp, total;
    int nblk;
};

ReindexLayout reindex_layout(int64_t n) {
    ReindexLayout L{};
    size_t off = 0;
    auto take = [&](size_t b) { size_t o = off; off += gt_align_up(b ? b : 4); return o; };
    L.keysA = take((size_t)n * 4);
    L.keysB = take((size_t)n * 4);
    L.valsA = take((size_t)n * 4);
    L.valsB = take((size_t)n * 4);
    L.head = take((size_t)(n + 1) * 4);
    L.first = take((size_t)(n + 1) * 4);
    L.group = take((size_t)(n + 1) * 4);
    L.nblk = rs_blocks(n > 0 ? n : 1);
    L.hist = take((size_t)256 * L.nblk * 4);
    size_t st = scan_tmp_ints((int64_t)256 * L.nblk), st2 = scan_tmp_ints(n + 1);
    L.scan_tmp = take((st > st2 ? st : st2) * 4);
    L.total = off;
    return L;
}

// ---------------------------------------------------------------------------------------------
// K
// ---------------------------------------------------------------------------------------------
// One group of G lanes per output row, 16 bytes per lane and step; the ragged end of a row
// (fewer than 16 bytes) and unaligned layouts go element by element.
template <typename T, bool VEC>
__global__ void __launch_bounds__(PT) k_lookup(const T *table, int64_t n_rows, int64_t ld, const int32_t *ids, int64_t n,
                                               int64_t F, T *out, int64_t ldo, int G) {
    constexpr int VE = 16 / sizeof(T);
    const int64_t row = ((int64_t)blockIdx.x * PT + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (row >= n) return;
    const int64_t v = ids[row];
    const bool ok = v >= 0 && v < n_rows;
    const T *src = table + (ok ? v : 0) * ld;
    T *dstp = out + row * ldo;
    int64_t c0 = 0;
    if (VEC) {
        const int64_t full = F / VE;
        for (int64_t c = gl; c < full; c += G) {
            uint4 q = make_uint4(0, 0, 0, 0);
            if (ok) q = *reinterpret_cast<const uint4 *>(src + c * VE);
            *reinterpret_cast<uint4 *>(dstp + c * VE) = q;
        }
        c0 = full * VE;
    }
    for (int64_t c = c0 + gl; c < F; c += G) dstp[c] = ok ? src[c] : T(0);
}

}  // namespace

extern "C" gt_status gt_sample_ws_size(int64_t n_dst, size_t *ws_bytes) {
    if (!ws_bytes) return gt_fail(GT_ERR_INVALID_ARG, "gt_sample_ws_size: ws_bytes is null");
    if (n_dst < 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_sample_ws_size: negative size");
    *ws_bytes = gt_align_up((size_t)(n_dst + 1) * 4) + gt_align_up(scan_tmp_ints(n_dst + 1) * 4);
    return GT_OK;
}

extern "C" gt_status gt_sample_neighbors(const int32_t *rowptr, const int32_t *colidx, int64_t n_vertices,
                                         const int32_t *dst, int64_t n_dst, int32_t fanout, uint32_t seed,
                                         uint32_t stream_id, int32_t *out_rowptr, int32_t *out_nbr, void *ws,
                                         size_t ws_bytes, void *stream) {
    const char *fn = "gt_sample_neighbors";
    if (n_vertices < 0 || n_dst < 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: negative size", fn);
    if (fanout < 1) return gt_fail(GT_ERR_INVALID_ARG, "%s: fanout must be at least 1", fn);
    if (!rowptr || !out_rowptr) return gt_fail(GT_ERR_INVALID_ARG, "%s: rowptr or out_rowptr is null", fn);
    if (n_dst > 0 && (!dst || !out_nbr || !colidx)) return gt_fail(GT_ERR_INVALID_ARG, "%s: dst, colidx or out_nbr is null", fn);
    if (n_dst * (int64_t)fanout >= ((int64_t)1 << 31))
        return gt_fail(GT_ERR_UNSUPPORTED, "%s: n_dst * fanout must be below 2^31", fn);
    size_t need = 0;
    gt_sample_ws_size(n_dst, &need);
    if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: ws null or not 256-byte aligned", fn);
    if (ws_bytes < need) return gt_fail(GT_ERR_WORKSPACE, "%s: ws_bytes %zu < required %zu", fn, ws_bytes, need);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t *cnt = static_cast<int32_t *>(ws);
    int32_t *tmp = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + gt_align_up((size_t)(n_dst + 1) * 4));
    k_sample_counts<<<nblocks(n_dst + 1), PT, 0, st>>>(rowptr, n_vertices, dst, n_dst, fanout, cnt);
    GT_LAUNCH_CHECK("k_sample_counts");
    gt_status s = scan_exclusive(cnt, out_rowptr, n_dst + 1, tmp, st);
    if (s != GT_OK) return s;
    if (n_dst == 0) return GT_OK;
    const uint32_t skey = mix32(seed + GOLD * stream_id);
    k_sample_pick<<<nblocks(n_dst, PT / 64), PT, 0, st>>>(rowptr, colidx, n_vertices, dst, n_dst, fanout, skey, out_rowptr,
                                                          out_nbr);
    GT_LAUNCH_CHECK("k_sample_pick");
    return GT_OK;
}

extern "C" gt_status gt_reindex_ws_size(int64_t n_dst, int64_t n_picked, size_t *ws_bytes) {
    if (!ws_bytes) return gt_fail(GT_ERR_INVALID_ARG, "gt_reindex_ws_size: ws_bytes is null");
    if (n_dst < 0 || n_picked < 0) return gt_fail(GT_ERR_INVALID_ARG, "gt_reindex_ws_size: negative size");
    if (n_dst + n_picked >= ((int64_t)1 << 31)) return gt_fail(GT_ERR_UNSUPPORTED, "gt_reindex_ws_size: n_dst + n_picked must be below 2^31");
    *ws_bytes = reindex_layout(n_dst + n_picked).total;
    return GT_OK;
}

extern "C" gt_status gt_reindex(const int32_t *dst, int64_t n_dst, const int32_t *picked, int64_t n_picked,
                                int64_t n_vertices, int32_t *src_global, int32_t *colidx_local, int32_t *counts,
                                void *ws, size_t ws_bytes, void *stream) {
    const char *fn = "gt_reindex";
    if (n_dst < 0 || n_picked < 0 || n_vertices < 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: negative size", fn);
    const int64_t n = n_dst + n_picked;
    if (n >= ((int64_t)1 << 31) || n_vertices > ((int64_t)1 << 31))
        return gt_fail(GT_ERR_UNSUPPORTED, "%s: n_dst + n_picked and n_vertices must be below 2^31", fn);
    if (!counts) return gt_fail(GT_ERR_INVALID_ARG, "%s: counts is null", fn);
    if ((n_dst > 0 && !dst) || (n_picked > 0 && (!picked || !colidx_local)) || (n > 0 && !src_global))
        return gt_fail(GT_ERR_INVALID_ARG, "%s: null array", fn);
    const ReindexLayout L = reindex_layout(n);
    if (!ws || ((uintptr_t)ws & 255)) return gt_fail(GT_ERR_WORKSPACE, "%s: ws null or not 256-byte aligned", fn);
    if (ws_bytes < L.total) return gt_fail(GT_ERR_WORKSPACE, "%s: ws_bytes %zu < required %zu", fn, ws_bytes, L.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws);
    uint32_t *kA = reinterpret_cast<uint32_t *>(w + L.keysA), *kB = reinterpret_cast<uint32_t *>(w + L.keysB);
    uint32_t *vA = reinterpret_cast<uint32_t *>(w + L.valsA), *vB = reinterpret_cast<uint32_t *>(w + L.valsB);
    int32_t *head = reinterpret_cast<int32_t *>(w + L.head), *first = reinterpret_cast<int32_t *>(w + L.first);
    int32_t *group = reinterpret_cast<int32_t *>(w + L.group);
    SortTmp tmp{reinterpret_cast<int32_t *>(w + L.hist), reinterpret_cast<int32_t *>(w + L.scan_tmp)};
    if (n > 0) {
        k_concat_ids<<<nblocks(n), PT, 0, st>>>(dst, n_dst, picked, n, kA);
        GT_LAUNCH_CHECK("k_concat_ids");
    }
    // ids below n_vertices: sort only the bytes that can differ (at least one pass, which also
    // produces the position array)
    int bits = 1;
    while (bits < 32 && ((int64_t)1 << bits) < n_vertices) ++bits;
    const int passes = (bits + 7) / 8;
    const uint32_t *vin = nullptr;   // first pass: value = position
    SortPasses sp{};
    sp.passes = passes;
    for (int p = 0; p < passes; ++p) {
        sp.kin[p] = kA; sp.vin[p] = vin; sp.kout[p] = kB; sp.vout[p] = vB;
        uint32_t *t = kA; kA = kB; kB = t;
        t = vA; vA = vB; vB = t;
        vin = vA;
    }
    {
        const gt_status rs = radix_sort(sp, n, tmp, st);
        if (rs != GT_OK) return rs;
    }
    // kA / vA: ids ascending, positions ascending within equal ids
    k_mark_heads<<<nblocks(n + 1), PT, 0, st>>>(kA, vA, n, head, first);
    GT_LAUNCH_CHECK("k_mark_heads");
    const int32_t *in2[2] = {head, first};
    int32_t *out2[2] = {head, first};
    gt_status s = scan_exclusive_batch(2, in2, out2, n + 1, tmp.scan_tmp, st);
    if (s != GT_OK) return s;
    if (n > 0) {
        k_group_ids<<<nblocks(n), PT, 0, st>>>(kA, vA, n, head, first, group, src_global);
        GT_LAUNCH_CHECK("k_group_ids");
    }
    k_emit_local<<<nblocks(n > 0 ? n : 1), PT, 0, st>>>(vA, n, n_dst, head, first, group, colidx_local, counts);
    GT_LAUNCH_CHECK("k_emit_local");
    return GT_OK;
}

extern "C" gt_status gt_lookup(gt_dtype dtype, const void *table, int64_t n_rows, int64_t ld, const int32_t *ids,
                               int64_t n, int64_t F, void *out, int64_t ldo, void *stream) {
    const char *fn = "gt_lookup";
    if (dtype != GT_F32 && dtype != GT_BF16) return gt_fail(GT_ERR_INVALID_ARG, "%s: unknown dtype", fn);
    if (n_rows < 0 || n < 0 || F < 0) return gt_fail(GT_ERR_INVALID_ARG, "%s: negative size", fn);
    if (n == 0 || F == 0) return GT_OK;
    if (!table || !ids || !out) return gt_fail(GT_ERR_INVALID_ARG, "%s: null array", fn);
    if (ld < F || ldo < F) return gt_fail(GT_ERR_INVALID_ARG, "%s: leading dimension too small", fn);
    const size_t es = gt_dtype_size(dtype);
    if (((uintptr_t)table % es) || ((uintptr_t)out % es)) return gt_fail(GT_ERR_INVALID_ARG, "%s: pointer misaligned for dtype", fn);
    if (table == out) return gt_fail(GT_ERR_INVALID_ARG, "%s: out aliases table", fn);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool vec = (((uintptr_t)table | (uintptr_t)out) & 15) == 0 && (ld * es) % 16 == 0 && (ldo * es) % 16 == 0;
    const int64_t chunks = vec ? (int64_t)((F * es + 15) / 16) : F;
    int G = 4;
    while (G < 64 && G < chunks) G <<= 1;
    const unsigned grid = nblocks(n * G);
    if (dtype == GT_F32) {
        if (vec) k_lookup<float, true><<<grid, PT, 0, st>>>(static_cast<const float *>(table), n_rows, ld, ids, n, F, static_cast<float *>(out), ldo, G);
        else k_lookup<float, false><<<grid, PT, 0, st>>>(static_cast<const float *>(table), n_rows, ld, ids, n, F, static_cast<float *>(out), ldo, G);
    } else {
        typedef uint16_t b16;
        if (vec) k_lookup<b16, true><<<grid, PT, 0, st>>>(static_cast<const b16 *>(table), n_rows, ld, ids, n, F, static_cast<b16 *>(out), ldo, G);
        else k_lookup<b16, false><<<grid, PT, 0, st>>>(static_cast<const b16 *>(table), n_rows, ld, ids, n, F, static_cast<b16 *>(out), ldo, G);
    }
    GT_LAUNCH_CHECK("k_lookup");
    return GT_OK;
}
