// Device-wide primitives of the adjacency builders: exclusive scan and LSD radix
// sort of 64-bit keys (hand-written; one wavefront per sort tile, stable ranks
// from wave votes).  Included by the builder translation units only.
#pragma once

#include "common.h"

namespace {

// ---------------------------------------------------------------- helpers
struct DevBuf {
    void *p = nullptr;
    ~DevBuf() { reset(); }
    void reset()
    {
        if (p)
            (void)hipFree(p);
        p = nullptr;
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 8); }
    template <typename T> T *as() { return (T *)p; }
    void *release()
    {
        void *q = p;
        p = nullptr;
        return q;
    }
};

static inline unsigned blocks_for(int64_t n, int per_block)
{
    return (unsigned)((n + per_block - 1) / per_block);
}

// ---------------------------------------------------------------- scan
constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;

// Exclusive scan of `v` across the 256 threads of a block; returns the
// exclusive prefix of this thread and the block total through `total`.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *total)
{
    __shared__ uint32_t wave_sum[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d, 64);
        if (lane >= d)
            inc += o;
    }
    __syncthreads(); // protects wave_sum against the previous call
    if (lane == 63)
        wave_sum[wave] = inc;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        const uint32_t s = wave_sum[w];
        if (w < wave)
            before += s;
        all += s;
    }
    *total = all;
    return before + inc - v;
}

__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(const uint32_t *__restrict__ in,
                                                                   uint32_t n,
                                                                   uint32_t *__restrict__ sums)
{
    const uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
        if (base + k < n)
            s += in[base + k];
    uint32_t total;
    (void)block_exclusive_scan(s, &total);
    if (threadIdx.x == 0)
        sums[blockIdx.x] = total;
}

// In-place exclusive scan of one tile, plus the tile's offset (0 if null).
__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(uint32_t *__restrict__ data,
                                                                  uint32_t n,
                                                                  const uint32_t *__restrict__ offs)
{
    const uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    uint32_t v[kScanItems];
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = (base + k < n) ? data[base + k] : 0;
        s += v[k];
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan(s, &total) + (offs ? offs[blockIdx.x] : 0);
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < n)
            data[base + k] = run;
        run += v[k];
    }
}

// Exclusive scan of data[0..n) in place.  `ws` must hold scan_ws_words(n) words.
static size_t scan_ws_words(uint64_t n)
{
    size_t w = 0;
    while (n > (uint64_t)kScanTile) {
        n = (n + kScanTile - 1) / kScanTile;
        w += n;
    }
    return w + 1;
}

static void scan_inplace(uint32_t *data, uint32_t n, uint32_t *ws, hipStream_t s)
{
    const uint32_t tiles = (n + kScanTile - 1) / kScanTile;
    if (tiles <= 1) {
        scan_apply_kernel<<<1, kScanThreads, 0, s>>>(data, n, nullptr);
        return;
    }
    scan_reduce_kernel<<<tiles, kScanThreads, 0, s>>>(data, n, ws);
    scan_inplace(ws, tiles, ws + tiles, s);
    scan_apply_kernel<<<tiles, kScanThreads, 0, s>>>(data, n, ws);
}

// ---------------------------------------------------------------- radix sort
constexpr int kSortItems = 32;
constexpr int kSortTile = 64 * kSortItems; // keys per wavefront

__global__ __launch_bounds__(64) void radix_hist_kernel(const uint64_t *__restrict__ keys,
                                                        uint32_t n, int shift,
                                                        uint32_t *__restrict__ hist,
                                                        uint32_t tiles)
{
    __shared__ uint32_t h[256];
    const int lane = threadIdx.x;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        h[lane + 64 * q] = 0;
    __syncthreads();
    const uint32_t base = blockIdx.x * kSortTile;
    for (int it = 0; it < kSortItems; ++it) {
        const uint32_t idx = base + it * 64 + lane;
        if (idx < n)
            atomicAdd(&h[(uint32_t)(keys[idx] >> shift) & 255u], 1u);
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q)
        hist[(uint64_t)(lane + 64 * q) * tiles + blockIdx.x] = h[lane + 64 * q];
}

__global__ __launch_bounds__(64) void radix_scatter_kernel(const uint64_t *__restrict__ in,
                                                           uint64_t *__restrict__ out, uint32_t n,
                                                           int shift,
                                                           const uint32_t *__restrict__ offsets,
                                                           uint32_t tiles)
{
    __shared__ uint32_t next[256]; // next output slot of each digit for this tile
    const int lane = threadIdx.x;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        next[lane + 64 * q] = offsets[(uint64_t)(lane + 64 * q) * tiles + blockIdx.x];
    __syncthreads();
    const uint32_t base = blockIdx.x * kSortTile;
    for (int it = 0; it < kSortItems; ++it) {
        const uint32_t idx = base + it * 64 + lane;
        const bool valid = idx < n;
        const uint64_t key = valid ? in[idx] : 0;
        const uint32_t d = (uint32_t)(key >> shift) & 255u;
        // lanes holding the same digit: intersect the 8 vote masks
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const uint32_t rank = __builtin_amdgcn_mbcnt_hi(
            (uint32_t)(peers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
        const uint32_t cnt = (uint32_t)__popcll(peers);
        uint32_t pos = 0;
        if (valid)
            pos = next[d] + rank;
        __syncthreads(); // every lane has read next[] before a leader bumps it
        if (valid && rank == 0)
            next[d] += cnt;
        __syncthreads();
        if (valid)
            out[pos] = key;
    }
}

// Sorts keys[0..n) on bits [0, bits) (LSD, 8 bits a pass).  Returns the buffer
// that holds the result (a or b).
static uint64_t *radix_sort(uint64_t *a, uint64_t *b, uint32_t n, int bits, uint32_t *hist,
                            uint32_t *scan_ws, hipStream_t s)
{
    const uint32_t tiles = (n + kSortTile - 1) / kSortTile;
    for (int shift = 0; shift < bits; shift += 8) {
        radix_hist_kernel<<<tiles, 64, 0, s>>>(a, n, shift, hist, tiles);
        scan_inplace(hist, 256u * tiles, scan_ws, s);
        radix_scatter_kernel<<<tiles, 64, 0, s>>>(a, b, n, shift, hist, tiles);
        uint64_t *t = a;
        a = b;
        b = t;
    }
    return a;
}

} // namespace
