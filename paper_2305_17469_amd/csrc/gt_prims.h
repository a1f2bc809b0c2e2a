// Device-wide primitives shared by the plan builder and the batch-preparation kernels: an
// exclusive int32 scan and a stable LSD radix sort of (key, value) pairs.  Header-only with
// internal linkage: every translation unit that includes it gets its own copy of the kernels.
#pragma once
#include "gt_internal.h"

namespace {

// ---------------------------------------------------------------------------------------------
// exclusive scan of int32 (reduce-then-scan, recursive over block sums)
// ---------------------------------------------------------------------------------------------

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_PER_THREAD = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_PER_THREAD;

__device__ inline int32_t block_exclusive_scan(int32_t v, int32_t *total) {
    // 256 threads; returns exclusive prefix of v over the block, *total = block sum
    __shared__ int32_t wave_sums[SCAN_THREADS / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int32_t o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    int32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SCAN_THREADS / 64; ++w) {
        int32_t s = wave_sums[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ void __launch_bounds__(SCAN_THREADS) k_scan_tiles(const int32_t *in, int32_t *out, int64_t n,
                                                             int32_t *tile_sums) {
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_PER_THREAD;
    int32_t v[SCAN_PER_THREAD];
    int32_t s = 0;
#pragma unroll
    for (int i = 0; i < SCAN_PER_THREAD; ++i) {
        v[i] = (base + i < n) ? in[base + i] : 0;
        s += v[i];
    }
    int32_t total;
    int32_t ex = block_exclusive_scan(s, &total);
#pragma unroll
    for (int i = 0; i < SCAN_PER_THREAD; ++i) {
        if (base + i < n) out[base + i] = ex;
        ex += v[i];
    }
    if (threadIdx.x == 0 && tile_sums) tile_sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(SCAN_THREADS) k_scan_add(int32_t *out, int64_t n, const int32_t *tile_offs) {
    const int32_t add = tile_offs[blockIdx.x];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_PER_THREAD;
#pragma unroll
    for (int i = 0; i < SCAN_PER_THREAD; ++i)
        if (base + i < n) out[base + i] += add;
}

size_t scan_tmp_ints(int64_t n) {
    size_t t = 0;
    while (n > SCAN_TILE) {
        int64_t tiles = (n + SCAN_TILE - 1) / SCAN_TILE;
        t += gt_align_up((size_t)tiles * 4) / 4;
        n = tiles;
    }
    return t + 64;
}

// Up to three arrays of the same short length in one launch: one workgroup of 1,024 threads per
// array walks it in steps of 8,192 elements and carries the running total.  A sampled batch's scans
// (a few thousand rows) are bound by launch latency; this takes one launch where the tiled form
// takes three per array.  Only up to two steps: beyond that the single workgroup's serial walk
// costs more than the launches it saves (measured on MI355X: 6.6 us at 13 K elements, 16.6 us
// average on 20-64 K against about 10 us for the three tiled launches).
constexpr int SCAN_SMALL_THREADS = 1024;
constexpr int64_t SCAN_SMALL_MAX = 16384;
struct ScanBatch { const int32_t *in[3]; int32_t *out[3]; };

__global__ void __launch_bounds__(SCAN_SMALL_THREADS) k_scan_small(const ScanBatch b, int64_t n) {
    __shared__ int32_t wave_sums[SCAN_SMALL_THREADS / 64];
    const int32_t *in = b.in[blockIdx.x];
    int32_t *out = b.out[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t carry = 0;
    for (int64_t t0 = 0; t0 < n; t0 += (int64_t)SCAN_SMALL_THREADS * SCAN_PER_THREAD) {
        const int64_t base = t0 + (int64_t)threadIdx.x * SCAN_PER_THREAD;
        int32_t v[SCAN_PER_THREAD];
        int32_t s = 0;
#pragma unroll
        for (int i = 0; i < SCAN_PER_THREAD; ++i) {
            v[i] = (base + i < n) ? in[base + i] : 0;
            s += v[i];
        }
        int32_t inc = s;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t o = __shfl_up(inc, d, 64);
            if (lane >= d) inc += o;
        }
        if (lane == 63) wave_sums[wave] = inc;
        __syncthreads();
        int32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < SCAN_SMALL_THREADS / 64; ++w) {
            const int32_t ws = wave_sums[w];
            if (w < wave) before += ws;
            total += ws;
        }
        __syncthreads();   // wave_sums is rewritten in the next step
        int32_t ex = carry + before + inc - s;
#pragma unroll
        for (int i = 0; i < SCAN_PER_THREAD; ++i) {
            if (base + i < n) out[base + i] = ex;
            ex += v[i];
        }
        carry += total;
    }
}

gt_status scan_exclusive(const int32_t *in, int32_t *out, int64_t n, int32_t *tmp, hipStream_t st);

// out[k][i] = sum_{j<i} in[k][j] for `count` (1..3) arrays of n elements each (in == out allowed).
// tmp: scan_tmp_ints(n) int32.
gt_status scan_exclusive_batch(int count, const int32_t *const *in, int32_t *const *out, int64_t n, int32_t *tmp,
                               hipStream_t st) {
    if (n <= 0 || count <= 0) return GT_OK;
    if (count > 3) return gt_fail(GT_ERR_INTERNAL, "scan_exclusive_batch: more than three arrays");
    if (n <= SCAN_SMALL_MAX) {
        ScanBatch b{};
        for (int k = 0; k < count; ++k) { b.in[k] = in[k]; b.out[k] = out[k]; }
        k_scan_small<<<count, SCAN_SMALL_THREADS, 0, st>>>(b, n);
        GT_LAUNCH_CHECK("k_scan_small");
        return GT_OK;
    }
    for (int k = 0; k < count; ++k) {
        const gt_status s = scan_exclusive(in[k], out[k], n, tmp, st);
        if (s != GT_OK) return s;
    }
    return GT_OK;
}

// out[i] = sum_{j<i} in[j] for i < n (in == out allowed).  tmp: scan_tmp_ints(n) int32.
gt_status scan_exclusive(const int32_t *in, int32_t *out, int64_t n, int32_t *tmp, hipStream_t st) {
    if (n <= 0) return GT_OK;
    if (n <= SCAN_SMALL_MAX) return scan_exclusive_batch(1, &in, &out, n, tmp, st);
    const int64_t tiles = (n + SCAN_TILE - 1) / SCAN_TILE;
    if (tiles == 1) {
        k_scan_tiles<<<1, SCAN_THREADS, 0, st>>>(in, out, n, nullptr);
        GT_LAUNCH_CHECK("k_scan_tiles");
        return GT_OK;
    }
    k_scan_tiles<<<(unsigned)tiles, SCAN_THREADS, 0, st>>>(in, out, n, tmp);
    GT_LAUNCH_CHECK("k_scan_tiles");
    int32_t *next = tmp + gt_align_up((size_t)tiles * 4) / 4;
    gt_status s = scan_exclusive(tmp, tmp, tiles, next, st);
    if (s != GT_OK) return s;
    k_scan_add<<<(unsigned)tiles, SCAN_THREADS, 0, st>>>(out, n, tmp);
    GT_LAUNCH_CHECK("k_scan_add");
    return GT_OK;
}

// ---------------------------------------------------------------------------------------------
// stable LSD radix sort of (key, value) pairs, 8 bits per pass
// ---------------------------------------------------------------------------------------------
constexpr int RS_THREADS = 256;
constexpr int RS_WAVES = RS_THREADS / 64;
constexpr int RS_CHUNKS = 16;                       // 64-item chunks per wave
constexpr int RS_WAVE_ITEMS = RS_CHUNKS * 64;       // 1024
constexpr int RS_TILE = RS_WAVES * RS_WAVE_ITEMS;   // 4096 items per block

__global__ void __launch_bounds__(RS_THREADS) k_rs_hist(const uint32_t *keys, int64_t n, int shift,
                                                        int32_t *hist, int nblk) {
    __shared__ int32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * RS_TILE + threadIdx.x;
    uint32_t k[RS_TILE / RS_THREADS];
#pragma unroll
    for (int i = 0; i < RS_TILE / RS_THREADS; ++i) {
        const int64_t p = base + (int64_t)i * RS_THREADS;
        k[i] = p < n ? keys[p] : 0u;
    }
#pragma unroll
    for (int i = 0; i < RS_TILE / RS_THREADS; ++i)
        if (base + (int64_t)i * RS_THREADS < n) atomicAdd(&h[(k[i] >> shift) & 255u], 1);
    __syncthreads();
    hist[(int64_t)threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}

// Scatter phase of one pass for the tile of this workgroup.  `digit_off` is, for digit
// d = threadIdx.x, the output position of the tile's first item with that digit.
// vals_in == nullptr means value = position (iota).
__device__ inline void rs_scatter_tile(const uint32_t *keys_in, const uint32_t *vals_in, uint32_t *keys_out,
                                       uint32_t *vals_out, int64_t n, int shift, int32_t digit_off) {
    __shared__ int32_t cnt[RS_WAVES][256];
    __shared__ int32_t wbase[RS_WAVES][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < RS_WAVES * 256; i += RS_THREADS) (&cnt[0][0])[i] = 0;
    __syncthreads();
    const int64_t wstart = (int64_t)blockIdx.x * RS_TILE + (int64_t)wave * RS_WAVE_ITEMS;
    uint32_t key[RS_CHUNKS];
    int32_t rank[RS_CHUNKS];
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    // all loads first, so that their latencies overlap instead of adding up chunk by chunk
#pragma unroll
    for (int c = 0; c < RS_CHUNKS; ++c) {
        const int64_t p = wstart + (int64_t)c * 64 + lane;
        key[c] = p < n ? keys_in[p] : 0u;
    }
#pragma unroll
    for (int c = 0; c < RS_CHUNKS; ++c) {
        rank[c] = 0;
        if (wstart + (int64_t)c * 64 >= n) continue;   // wavefront-uniform: the chunk is empty
        const int64_t p = wstart + (int64_t)c * 64 + lane;
        const bool valid = p < n;
        const uint32_t digit = (key[c] >> shift) & 255u;
        uint64_t m = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (digit >> b) & 1u;
            const uint64_t bal = __ballot(valid && bit);
            m &= bit ? bal : ~bal;
        }
        // m: valid lanes of this chunk with the same digit (meaningful on valid lanes)
        const int before = __popcll(m & lt_mask);
        int32_t prev = 0;
        if (valid) prev = cnt[wave][digit];
        rank[c] = prev + before;
        if (valid && before == 0) cnt[wave][digit] = prev + __popcll(m);
    }
    __syncthreads();
    {
        const int d = threadIdx.x;   // 256 threads <-> 256 digits
        int32_t run = digit_off;
#pragma unroll
        for (int w = 0; w < RS_WAVES; ++w) {
            wbase[w][d] = run;
            run += cnt[w][d];
        }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < RS_CHUNKS; ++c) {
        const int64_t p = wstart + (int64_t)c * 64 + lane;
        if (p < n) {
            const uint32_t digit = (key[c] >> shift) & 255u;
            const int64_t dst = (int64_t)wbase[wave][digit] + rank[c];
            keys_out[dst] = key[c];
            vals_out[dst] = vals_in ? vals_in[p] : (uint32_t)p;
        }
    }
}

__global__ void __launch_bounds__(RS_THREADS) k_rs_scatter(const uint32_t *keys_in, const uint32_t *vals_in,
                                                           uint32_t *keys_out, uint32_t *vals_out, int64_t n,
                                                           int shift, const int32_t *offs, int nblk) {
    rs_scatter_tile(keys_in, vals_in, keys_out, vals_out, n, shift, offs[(int64_t)threadIdx.x * nblk + blockIdx.x]);
}

// A whole pass in one launch for inputs of at most RS_SMALL_TILES tiles: every workgroup counts
// the digits of all tiles itself (the input is small enough to come from the L2), which gives it
// the global digit bases and the counts of the tiles before its own without a histogram kernel,
// a device-wide scan and their launch latencies.
constexpr int RS_SMALL_TILES = 8;

__global__ void __launch_bounds__(RS_THREADS) k_rs_pass_small(const uint32_t *keys_in, const uint32_t *vals_in,
                                                              uint32_t *keys_out, uint32_t *vals_out, int64_t n,
                                                              int shift, int nblk) {
    __shared__ int32_t h[256];
    const int d = threadIdx.x;
    int32_t before = 0, total = 0;
    for (int t = 0; t < nblk; ++t) {
        h[d] = 0;
        __syncthreads();
        const int64_t base = (int64_t)t * RS_TILE + threadIdx.x;
        uint32_t k[RS_TILE / RS_THREADS];
#pragma unroll
        for (int i = 0; i < RS_TILE / RS_THREADS; ++i) {
            const int64_t p = base + (int64_t)i * RS_THREADS;
            k[i] = p < n ? keys_in[p] : 0u;
        }
#pragma unroll
        for (int i = 0; i < RS_TILE / RS_THREADS; ++i)
            if (base + (int64_t)i * RS_THREADS < n) atomicAdd(&h[(k[i] >> shift) & 255u], 1);
        __syncthreads();
        const int32_t c = h[d];
        if (t < (int)blockIdx.x) before += c;
        total += c;
        __syncthreads();
    }
    int32_t all;
    const int32_t digit_base = block_exclusive_scan(total, &all);
    rs_scatter_tile(keys_in, vals_in, keys_out, vals_out, n, shift, digit_base + before);
}

// All passes of a sort of at most 16,384 pairs in one launch: a single workgroup of 16 wavefronts,
// each owning 1,024 consecutive items, keeps keys and values in LDS (128 KB) between the passes:
// a pass reads its items from LDS in order, ranks them exactly as rs_scatter_tile does (so the
// order is the same stable one) and writes them back to LDS at their sorted positions; the last
// pass is followed by one coalesced copy to the caller's output.  A sampled batch sorts a few
// thousand keys in 2-3 passes: one launch instead of one per pass, and no scattered 4-byte stores
// to memory, which a single compute unit retires at about one cache line per clock (measured on
// MI355X, 15 K pairs, 3 passes: 54 us as three launches, 47 us as one launch through memory).
constexpr int RS_ONE_THREADS = 1024;
constexpr int RS_ONE_WAVES = RS_ONE_THREADS / 64;
constexpr int64_t RS_ONE_MAX = (int64_t)RS_ONE_WAVES * RS_WAVE_ITEMS;
constexpr int RS_MAX_PASSES = 4;
constexpr size_t RS_ONE_LDS = (size_t)RS_ONE_MAX * 8 + (size_t)RS_ONE_WAVES * 256 * 2 * 2;

struct SortPasses {
    const uint32_t *kin[RS_MAX_PASSES];
    const uint32_t *vin[RS_MAX_PASSES];   // null: value = position
    uint32_t *kout[RS_MAX_PASSES];
    uint32_t *vout[RS_MAX_PASSES];
    int passes;                           // pass p sorts by bits [8p, 8p + 8)
};

__global__ void __launch_bounds__(RS_ONE_THREADS) k_rs_sort_one(const uint32_t *keys_in, const uint32_t *vals_in,
                                                                uint32_t *keys_out, uint32_t *vals_out, int64_t n,
                                                                int passes) {
    extern __shared__ __align__(16) unsigned char rs_one_smem[];
    uint32_t *lk = reinterpret_cast<uint32_t *>(rs_one_smem);       // [RS_ONE_MAX]
    uint32_t *lv = lk + RS_ONE_MAX;                                  // [RS_ONE_MAX]
    uint16_t *cnt = reinterpret_cast<uint16_t *>(lv + RS_ONE_MAX);   // [RS_ONE_WAVES][256], at most 1,024 each
    uint16_t *wbase = cnt + RS_ONE_WAVES * 256;                      // [RS_ONE_WAVES][256], below 16,384
    __shared__ int32_t wsum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    const int wstart = wave * RS_WAVE_ITEMS;
    const int nn = (int)n;
    uint32_t key[RS_CHUNKS], val[RS_CHUNKS];
#pragma unroll
    for (int c = 0; c < RS_CHUNKS; ++c) {
        const int q = wstart + c * 64 + lane;
        key[c] = q < nn ? keys_in[q] : 0u;
        val[c] = (q < nn && vals_in) ? vals_in[q] : (uint32_t)q;
    }
    for (int p = 0; p < passes; ++p) {
        const int shift = 8 * p;
        for (int i = threadIdx.x; i < RS_ONE_WAVES * 256; i += RS_ONE_THREADS) cnt[i] = 0;
        if (p > 0) {
#pragma unroll
            for (int c = 0; c < RS_CHUNKS; ++c) {
                const int q = wstart + c * 64 + lane;
                key[c] = q < nn ? lk[q] : 0u;
                val[c] = q < nn ? lv[q] : 0u;
            }
        }
        __syncthreads();
        int rank[RS_CHUNKS];
#pragma unroll
        for (int c = 0; c < RS_CHUNKS; ++c) {
            rank[c] = 0;
            if (wstart + c * 64 >= nn) continue;   // wavefront-uniform: the chunk is empty
            const bool valid = wstart + c * 64 + lane < nn;
            const uint32_t digit = (key[c] >> shift) & 255u;
            uint64_t m = __ballot(valid);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const bool bit = (digit >> b) & 1u;
                const uint64_t bal = __ballot(valid && bit);
                m &= bit ? bal : ~bal;
            }
            const int before = __popcll(m & lt_mask);
            int prev = 0;
            if (valid) prev = cnt[wave * 256 + digit];
            rank[c] = prev + before;
            if (valid && before == 0) cnt[wave * 256 + digit] = (uint16_t)(prev + __popcll(m));
        }
        __syncthreads();
        // threads 0..255 <-> digits: per-wavefront bases within the digit, then the digits' starts
        const int d = threadIdx.x & 255;
        int tot = 0;
        int wb[RS_ONE_WAVES];
        if (threadIdx.x < 256) {
#pragma unroll
            for (int w = 0; w < RS_ONE_WAVES; ++w) {
                wb[w] = tot;
                tot += cnt[w * 256 + d];
            }
        }
        int inc = tot;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const int o = __shfl_up(inc, s, 64);
            if (lane >= s) inc += o;
        }
        if (threadIdx.x < 256 && lane == 63) wsum[wave] = inc;
        __syncthreads();
        if (threadIdx.x < 256) {
            int start = inc - tot;
            for (int w = 0; w < wave; ++w) start += wsum[w];
#pragma unroll
            for (int w = 0; w < RS_ONE_WAVES; ++w) wbase[w * 256 + d] = (uint16_t)(start + wb[w]);
        }
        __syncthreads();
        // every wavefront has its items in registers: the LDS copies may be overwritten
#pragma unroll
        for (int c = 0; c < RS_CHUNKS; ++c) {
            const int q = wstart + c * 64 + lane;
            if (q < nn) {
                const uint32_t digit = (key[c] >> shift) & 255u;
                const int dst = (int)wbase[wave * 256 + digit] + rank[c];
                lk[dst] = key[c];
                lv[dst] = val[c];
            }
        }
        __syncthreads();
    }
    if (passes <= 0) {   // nothing sorted: the registers still hold the input
#pragma unroll
        for (int c = 0; c < RS_CHUNKS; ++c) {
            const int q = wstart + c * 64 + lane;
            if (q < nn) { keys_out[q] = key[c]; vals_out[q] = val[c]; }
        }
        return;
    }
    for (int q = threadIdx.x; q < nn; q += RS_ONE_THREADS) {
        keys_out[q] = lk[q];
        vals_out[q] = lv[q];
    }
}

struct SortTmp {
    int32_t *hist;      // 256 * nblk
    int32_t *scan_tmp;  // scan_tmp_ints(256 * nblk)
};

int rs_blocks(int64_t n) { return (int)((n + RS_TILE - 1) / RS_TILE); }

gt_status radix_pass(const uint32_t *kin, const uint32_t *vin, uint32_t *kout, uint32_t *vout, int64_t n,
                     int shift, const SortTmp &t, hipStream_t st) {
    if (n <= 0) return GT_OK;
    const int nblk = rs_blocks(n);
    if (nblk <= RS_SMALL_TILES) {
        k_rs_pass_small<<<nblk, RS_THREADS, 0, st>>>(kin, vin, kout, vout, n, shift, nblk);
        GT_LAUNCH_CHECK("k_rs_pass_small");
        return GT_OK;
    }
    k_rs_hist<<<nblk, RS_THREADS, 0, st>>>(kin, n, shift, t.hist, nblk);
    GT_LAUNCH_CHECK("k_rs_hist");
    gt_status s = scan_exclusive(t.hist, t.hist, (int64_t)256 * nblk, t.scan_tmp, st);
    if (s != GT_OK) return s;
    k_rs_scatter<<<nblk, RS_THREADS, 0, st>>>(kin, vin, kout, vout, n, shift, t.hist, nblk);
    GT_LAUNCH_CHECK("k_rs_scatter");
    return GT_OK;
}

// Runs the passes of `a` in order: one launch when the input is short, one pass at a time otherwise.
gt_status radix_sort(const SortPasses &a, int64_t n, const SortTmp &t, hipStream_t st) {
    if (n <= 0 || a.passes <= 0) return GT_OK;
    if (a.passes > RS_MAX_PASSES) return gt_fail(GT_ERR_INTERNAL, "radix_sort: too many passes");
    if (n <= RS_ONE_MAX) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_rs_sort_one),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)RS_ONE_LDS);
        if (e != hipSuccess) return gt_hip_fail(e, "hipFuncSetAttribute(k_rs_sort_one)");
        k_rs_sort_one<<<1, RS_ONE_THREADS, RS_ONE_LDS, st>>>(a.kin[0], a.vin[0], a.kout[a.passes - 1],
                                                              a.vout[a.passes - 1], n, a.passes);
        GT_LAUNCH_CHECK("k_rs_sort_one");
        return GT_OK;
    }
    for (int p = 0; p < a.passes; ++p) {
        const gt_status s = radix_pass(a.kin[p], a.vin[p], a.kout[p], a.vout[p], n, 8 * p, t, st);
        if (s != GT_OK) return s;
    }
    return GT_OK;
}

}  // namespace
