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

// out[i] = sum_{j<i} in[j] for i < n (in == out allowed).  tmp: scan_tmp_ints(n) int32.
gt_status scan_exclusive(const int32_t *in, int32_t *out, int64_t n, int32_t *tmp, hipStream_t st) {
    if (n <= 0) return GT_OK;
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

}  // namespace
