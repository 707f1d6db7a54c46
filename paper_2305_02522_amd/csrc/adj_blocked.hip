// Column-blocked, length-balanced form of the adjacency for the LDS-staged
// bit-SpMM (the role of the paper's fine-representing / dynamic-coarsening
// scheme, Section 3.2.1: store the sparse bit matrix finely, coarsen on chip).
//
// Why: a 16-byte activation row gathered from global memory costs a whole
// 128-byte cache line (measured ~0.33 gathers/clock/CU on MI355X), while the
// same gather from LDS runs ~11x faster.  So the activation matrix is cut into
// column blocks of `cbn` nodes that fit the 160 KB LDS, and the adjacency is
// stored so that a workgroup streams, per column block, only 16-bit column ids
// local to the block.
//
// Layout decisions
//  - nodes are renumbered by decreasing degree ("slot"), so that hub columns
//    share the first blocks and rows of similar length sit together;
//  - a row's neighbour list (sorted by column slot) is cut into parts of at
//    most `part_len` entries ("virtual rows"): a hub row becomes many parts,
//    each touching one or two column blocks; partial counts are merged later.
//    This bounds the work of one lane, which balances wavefronts on a
//    power-law graph;
//  - parts are ordered by (first block, last block, entries in the first block,
//    entries in the second block), so that the lanes of a tile have similar
//    step counts; 64 consecutive parts form a slice (one wavefront, one part per lane), 16 slices a
//    workgroup.  For every (slice, block) tile the ids are stored lane-
//    interleaved in groups of kGroupSteps steps: group g holds
//    idx16[(g*64+lane)*kGroupSteps+k], padded with ids cbn .. cbn+15, which address
//    all-zero LDS rows.  The groups of a slice are consecutive, so a wavefront
//    reads one contiguous stream; one padding group closes the array so that
//    reading one group ahead is always in bounds.
#include "prims.h"

#include <stdlib.h>

namespace {

constexpr uint32_t kVidMask = (1u << 30) - 1;

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = __shfl_xor(v, d, 64);
        v = o < v ? o : v;
    }
    return v;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = __shfl_xor(v, d, 64);
        v = o > v ? o : v;
    }
    return v;
}

// slot numbering, degrees in slot order, parts per row
__global__ void slot_kernel(const int32_t *__restrict__ order, const int32_t *__restrict__ deg,
                            uint32_t n, int part_len, int32_t *__restrict__ rank,
                            uint32_t *__restrict__ deg_sorted, uint32_t *__restrict__ nparts,
                            uint32_t *__restrict__ n_multi)
{
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s > n)
        return;
    if (s == n) { // terminators of the two scans
        deg_sorted[n] = 0;
        nparts[n] = 0;
        return;
    }
    const int32_t i = order[s];
    rank[i] = (int32_t)s;
    const uint32_t d = (uint32_t)deg[i];
    deg_sorted[s] = d;
    const uint32_t np = (d + part_len - 1) / part_len;
    nparts[s] = np ? np : 1u;
    if (np > 1) // rows are in decreasing degree order: these are the first *n_multi slots
        atomicAdd(n_multi, 1u);
}

// keys (row slot << cbits | column slot), one wavefront per row
__global__ __launch_bounds__(256) void blocked_keys_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, const int32_t *__restrict__ rank,
    const uint32_t *__restrict__ rp2, uint32_t n, int cbits, uint64_t *__restrict__ keys)
{
    const uint32_t s = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (s >= n)
        return;
    const int32_t i = order[s];
    const uint32_t beg = rowptr[i], d = rowptr[i + 1] - beg, o = rp2[s];
    for (uint32_t k = lane; k < d; k += 64)
        keys[o + k] = ((uint64_t)s << cbits) | (uint32_t)rank[col[beg + k]];
}

// part descriptors and their sort keys
__global__ void vrow_kernel(const uint64_t *__restrict__ skeys, const uint32_t *__restrict__ rp2,
                            const uint32_t *__restrict__ vptr, uint32_t n, int cbits, int cbn,
                            uint32_t *__restrict__ v_beg, uint32_t *__restrict__ v_end,
                            uint32_t *__restrict__ v_slot, uint64_t *__restrict__ vkeys)
{
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n)
        return;
    const uint64_t mask = (1ull << cbits) - 1;
    const uint32_t r0 = rp2[s], d = rp2[s + 1] - r0;
    const uint32_t v0 = vptr[s], np = vptr[s + 1] - v0;
    const uint32_t plen = (d + np - 1) / np; // np >= 1
    for (uint32_t p = 0; p < np; ++p) {
        const uint32_t b = r0 + min(d, p * plen), e = r0 + min(d, (p + 1) * plen);
        const uint32_t len = e - b;
        const uint64_t lo = len ? (skeys[b] & mask) / (uint32_t)cbn : 0;
        const uint64_t hi = len ? (skeys[e - 1] & mask) / (uint32_t)cbn : 0;
        const uint32_t v = v0 + p;
        v_beg[v] = b;
        v_end[v] = e;
        v_slot[v] = s | (np == 1 ? 0x80000000u : 0u); // bit 31: the row's only part
        // Entries in the part's first two blocks (its heaviest: columns are in degree
        // order).  The parts of a slice share their tiles' step counts (the longest lane's),
        // so within a block range they are ordered by these two counts rather than by
        // length: on a Reddit-shaped graph 12 % fewer stored ids than ordering by length.
        uint32_t c0 = 0, c1 = 0;
        if (len) {
            uint32_t a = b, z = e; // first entry with column >= (lo + 1) cbn
            const uint64_t lim0 = (lo + 1) * (uint32_t)cbn, lim1 = lim0 + (uint32_t)cbn;
            while (a < z) {
                const uint32_t m = (a + z) >> 1;
                if ((skeys[m] & mask) < lim0)
                    a = m + 1;
                else
                    z = m;
            }
            c0 = a - b;
            z = e; // first entry with column >= (lo + 2) cbn, searched from there on
            while (a < z) {
                const uint32_t m = (a + z) >> 1;
                if ((skeys[m] & mask) < lim1)
                    a = m + 1;
                else
                    z = m;
            }
            c1 = a - b - c0;
        }
        const uint64_t sig =
            ((uint64_t)(31u - min(c0 >> 3, 31u)) << 5) | (31u - min(c1 >> 2, 31u));
        vkeys[v] = (lo << 52) | (hi << 40) | (sig << 30) | v;
    }
}

// per slice: range of column blocks its parts touch
__global__ __launch_bounds__(64) void slice_range_kernel(const uint64_t *__restrict__ svkeys,
                                                         uint32_t V, uint32_t S,
                                                         uint32_t *__restrict__ sl_cb,
                                                         uint32_t *__restrict__ sl_ntiles)
{
    const uint32_t slice = blockIdx.x;
    const int lane = threadIdx.x;
    if (slice == S) { // scan terminator
        if (lane == 0)
            sl_ntiles[S] = 0;
        return;
    }
    const uint32_t pos = slice * 64 + lane;
    const bool valid = pos < V;
    const uint64_t key = valid ? svkeys[pos] : 0;
    const uint32_t lo = wave_min_u32(valid ? (uint32_t)(key >> 52) : 0xFFFu);
    const uint32_t hi = wave_max_u32(valid ? (uint32_t)(key >> 40) & 0xFFFu : 0u);
    if (lane == 0) {
        sl_cb[slice] = lo | (hi << 16);
        sl_ntiles[slice] = hi - lo + 1;
    }
}

// Sixteen byte counters in two registers (dynamic index without spilling an array).
struct cls16 {
    uint64_t lo = 0, hi = 0;
    __device__ __forceinline__ uint32_t get(uint32_t c) const
    {
        return (uint32_t)(((c & 8u) ? hi : lo) >> ((c & 7u) * 8u)) & 255u;
    }
    __device__ __forceinline__ void set(uint32_t c, uint32_t v)
    {
        const uint64_t m = ~(255ull << ((c & 7u) * 8u)), b = (uint64_t)v << ((c & 7u) * 8u);
        if (c & 8u)
            hi = (hi & m) | b;
        else
            lo = (lo & m) | b;
    }
};

// per (slice, block) tile: steps = longest lane; FILL = false counts groups,
// FILL = true writes the lane-interleaved ids.
//
// Order of a lane's ids inside a tile (free: the sum does not depend on it).  The LDS
// serves a 16-byte gather of 16 consecutive lanes in one pass when the 16 rows fall into
// different 16-byte bank groups, i.e. differ in (row mod 16).  So lane L wants, at step k,
// a row of class (L + k) mod 16: an id goes to the first free step of its class, ids whose
// class has no step left take any free step, and padding steps address the all-zero row
// of the wanted class (rows cbn .. cbn + 15 of the staged block are zero).
template <bool FILL>
__global__ __launch_bounds__(64) void tile_kernel(
    const uint64_t *__restrict__ svkeys, uint32_t V, const uint32_t *__restrict__ v_beg,
    const uint32_t *__restrict__ v_end, const uint64_t *__restrict__ skeys, int cbits, int cbn,
    const uint32_t *__restrict__ sl_cb, const uint32_t *__restrict__ sl_tile_base,
    uint32_t *__restrict__ tile_group, uint16_t *__restrict__ idx16)
{
    const uint32_t slice = blockIdx.x;
    const uint32_t lane = threadIdx.x;
    const uint32_t pos = slice * 64 + lane;
    const uint64_t mask = (1ull << cbits) - 1;
    uint32_t ptr = 0, e = 0;
    if (pos < V) {
        const uint32_t v = (uint32_t)svkeys[pos] & kVidMask;
        ptr = v_beg[v];
        e = v_end[v];
    }
    const uint32_t lo = sl_cb[slice] & 0xFFFFu, hi = sl_cb[slice] >> 16;
    const uint32_t t0 = sl_tile_base[slice];
    for (uint32_t cb = lo; cb <= hi; ++cb) {
        const uint64_t lim = (uint64_t)(cb + 1) * (uint32_t)cbn;
        const uint64_t cb0 = (uint64_t)cb * (uint32_t)cbn;
        const uint32_t first = ptr;
        while (ptr < e && (skeys[ptr] & mask) < lim)
            ++ptr;
        const uint32_t cnt = ptr - first;
        if (!FILL) {
            const uint32_t m = wave_max_u32(cnt);
            if (lane == 0)
                tile_group[t0 + cb - lo] = (m + kGroupSteps - 1) / kGroupSteps;
        } else {
            const uint32_t g0 = tile_group[t0 + cb - lo];
            const uint32_t steps = (tile_group[t0 + cb - lo + 1] - g0) * kGroupSteps;
            auto slot = [&](uint32_t k) -> uint16_t & {
                return idx16[((uint64_t)(g0 + k / kGroupSteps) * 64 + lane) * kGroupSteps +
                             (k % kGroupSteps)];
            };
            // steps of class c' = (id - lane) mod 16 are c', c' + 16, ...: how many ids of
            // every class find one
            cls16 used, run;
            for (uint32_t j = 0; j < cnt; ++j) {
                const uint32_t id = (uint32_t)((skeys[first + j] & mask) - cb0);
                const uint32_t c = (id - lane) & 15u;
                const uint32_t cap = c < steps ? (steps - c + 15u) >> 4 : 0u;
                const uint32_t u = used.get(c);
                if (u < cap)
                    used.set(c, u + 1);
            }
            for (uint32_t k = 0; k < steps; ++k)
                slot(k) = (uint16_t)((uint32_t)cbn + ((lane + k) & 15u));
            uint32_t kfree = 0;
            for (uint32_t j = 0; j < cnt; ++j) {
                const uint32_t id = (uint32_t)((skeys[first + j] & mask) - cb0);
                const uint32_t c = (id - lane) & 15u;
                const uint32_t m = run.get(c);
                uint32_t k;
                if (m < used.get(c)) {
                    run.set(c, m + 1);
                    k = c + 16u * m;
                } else { // no step of its class left: the next step no class claims
                    while ((kfree >> 4) < used.get(kfree & 15u))
                        ++kfree;
                    k = kfree++;
                }
                slot(k) = (uint16_t)id;
            }
        }
    }
}

// the padding group behind the last tile
__global__ void tail_group_kernel(uint16_t *__restrict__ idx16, uint32_t G, int cbn)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 64u * kGroupSteps)
        idx16[(uint64_t)G * 64 * kGroupSteps + i] = (uint16_t)cbn;
}

// per processing position: {part id (row-major: the parts of a row are consecutive ids)
// | bit 31 if it is the row's only part, node id of the row}
__global__ void part_info_kernel(const uint64_t *__restrict__ svkeys, uint32_t V,
                                 const uint32_t *__restrict__ v_slot,
                                 const int32_t *__restrict__ order, uint2 *__restrict__ part_info)
{
    const uint32_t pos = blockIdx.x * blockDim.x + threadIdx.x;
    if (pos < V) {
        const uint32_t v = (uint32_t)svkeys[pos] & kVidMask;
        const uint32_t sl = v_slot[v];
        part_info[pos] = make_uint2(v | (sl & 0x80000000u), (uint32_t)order[sl & 0x7FFFFFFFu]);
    }
}

__global__ void wg_range_kernel(const uint32_t *__restrict__ sl_cb, uint32_t S, uint32_t W,
                                uint32_t spw, uint32_t *__restrict__ wg_cb)
{
    const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W)
        return;
    uint32_t lo = 0xFFFFu, hi = 0;
    for (uint32_t s = w * spw; s < (w + 1) * spw && s < S; ++s) {
        lo = min(lo, sl_cb[s] & 0xFFFFu);
        hi = max(hi, sl_cb[s] >> 16);
    }
    wg_cb[w] = lo | (hi << 16);
}

// sort key of a workgroup: estimated time, complemented so that an ascending sort lists
// the heaviest first.  The wavefronts of a workgroup meet at every column block, so a
// block costs its refill plus the longest tile among the slices (measured on MI355X:
// about 1.56 us per refill of 8192 rows, 0.51 us per group of 8 steps on the critical
// path, 10 us per work item); the unit below is 10 ns.
__global__ void wg_cost_kernel(const uint32_t *__restrict__ wg_cb,
                               const uint32_t *__restrict__ sl_cb,
                               const uint32_t *__restrict__ sl_tile_base,
                               const uint32_t *__restrict__ tile_group, uint32_t S, uint32_t W,
                               uint32_t spw, int cbn, uint64_t *__restrict__ keys)
{
    const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W)
        return;
    const uint32_t s0 = w * spw, s1 = min(s0 + spw, S);
    const uint32_t wlo = wg_cb[w] & 0xFFFFu, whi = wg_cb[w] >> 16;
    uint64_t crit = 0;
    for (uint32_t cb = wlo; cb <= whi; ++cb) {
        uint32_t longest = 0;
        for (uint32_t sl = s0; sl < s1; ++sl) {
            const uint32_t lo = sl_cb[sl] & 0xFFFFu, hi = sl_cb[sl] >> 16;
            if (cb >= lo && cb <= hi) {
                const uint32_t t = sl_tile_base[sl] + cb - lo;
                longest = max(longest, tile_group[t + 1] - tile_group[t]);
            }
        }
        crit += longest;
    }
    const uint64_t fills = whi - wlo + 1;
    const uint64_t cost = crit * (51 * kGroupSteps / 8) + fills * (156ull * cbn / 8192) + 1000;
    keys[w] = ((0xFFFFFFFFull - min(cost, (uint64_t)0xFFFFFFFFull)) << 32) | w;
}

// What the aggregation kernel reads at its start, flattened so that it takes two
// dependent loads instead of five: per dispatch position {workgroup, its block range},
// per slice {its block range, first tile, first group}.
__global__ void wg_item_kernel(const uint64_t *__restrict__ keys, uint32_t W,
                               const uint32_t *__restrict__ wg_cb, uint2 *__restrict__ wg_item)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < W) {
        const uint32_t w = (uint32_t)keys[i];
        wg_item[i] = make_uint2(w, wg_cb[w]);
    }
}

__global__ void slice_desc_kernel(const uint32_t *__restrict__ sl_cb,
                                  const uint32_t *__restrict__ sl_tile_base,
                                  const uint32_t *__restrict__ tile_group, uint32_t S,
                                  uint4 *__restrict__ sl_desc)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < S)
        sl_desc[i] = make_uint4(sl_cb[i], sl_tile_base[i], tile_group[sl_tile_base[i]], 0u);
}

} // namespace

void bg_free_blocked(bitgnn_blocked *b)
{
    if (!b)
        return;
    (void)hipFree(b->wg_item);
    (void)hipFree(b->sl_desc);
    (void)hipFree(b->tile_group);
    (void)hipFree(b->idx16);
    (void)hipFree(b->row_vptr);
    (void)hipFree(b->part_info);
    free(b);
}

// Builds adj->blk from the CSR arrays of `adj` (already on the device).
int bg_build_blocked(bitgnn_ctx *ctx, hipStream_t s, bitgnn_adj *adj)
{
    const uint32_t n = (uint32_t)adj->n, nnz = (uint32_t)adj->nnz;
    const int cbn = ctx->cb_nodes, part_len = ctx->part_len;
    const int64_t ncb = (adj->n + cbn - 1) / cbn;
    if (ncb > 4095 || nnz == 0 || cbn > kMaxCbNodes)
        return BITGNN_OK; // stays on the CSR path
    int cbits = 1;
    while ((1ll << cbits) < adj->n)
        ++cbits;

    DevBuf rank, deg_sorted, nparts, keys_a, keys_b, hist, scan_ws, multi;
    const uint32_t sort_n = nnz > n ? nnz : n;
    const uint32_t sort_tiles = (sort_n + kSortTile - 1) / kSortTile;
    BG_HIP(ctx, rank.alloc((size_t)n * 4));
    BG_HIP(ctx, deg_sorted.alloc(((size_t)n + 1) * 4));
    BG_HIP(ctx, nparts.alloc(((size_t)n + 1) * 4));
    BG_HIP(ctx, keys_a.alloc((size_t)sort_n * 8));
    BG_HIP(ctx, keys_b.alloc((size_t)sort_n * 8));
    BG_HIP(ctx, hist.alloc((size_t)256 * sort_tiles * 4));
    // one workspace for the scans of the sort histograms, of the n + 1 row counters and of
    // the slice counters (S + 1 <= sort_n / 32 + 2); the tile scan gets its own below
    const uint64_t scan_max = (uint64_t)256 * sort_tiles > (uint64_t)n + 1
                                  ? (uint64_t)256 * sort_tiles
                                  : (uint64_t)n + 1;
    BG_HIP(ctx, scan_ws.alloc(scan_ws_words(scan_max) * 4));

    BG_HIP(ctx, multi.alloc(4));
    BG_HIP(ctx, hipMemsetAsync(multi.p, 0, 4, s));
    slot_kernel<<<blocks_for((int64_t)n + 1, 256), 256, 0, s>>>(
        adj->order, adj->deg, n, part_len, rank.as<int32_t>(), deg_sorted.as<uint32_t>(),
        nparts.as<uint32_t>(), multi.as<uint32_t>());
    // exclusive scans: rp2 = entry offsets by slot, vptr = first part by slot
    scan_inplace(deg_sorted.as<uint32_t>(), n + 1, scan_ws.as<uint32_t>(), s);
    scan_inplace(nparts.as<uint32_t>(), n + 1, scan_ws.as<uint32_t>(), s);
    const uint32_t *rp2 = deg_sorted.as<uint32_t>();
    uint32_t *vptr = nparts.as<uint32_t>();
    blocked_keys_kernel<<<blocks_for(n, 4), 256, 0, s>>>(adj->rowptr, adj->col, adj->order,
                                                        rank.as<int32_t>(), rp2, n, cbits,
                                                        keys_a.as<uint64_t>());
    BG_LAUNCH_CHECK(ctx, "blocked_keys");
    uint64_t *skeys = radix_sort(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), nnz, 2 * cbits,
                                 hist.as<uint32_t>(), scan_ws.as<uint32_t>(), s);
    BG_LAUNCH_CHECK(ctx, "blocked radix_sort");
    uint32_t V = 0, n_multi = 0;
    BG_HIP(ctx, hipMemcpyAsync(&V, vptr + n, 4, hipMemcpyDeviceToHost, s));
    BG_HIP(ctx, hipMemcpyAsync(&n_multi, multi.p, 4, hipMemcpyDeviceToHost, s));
    BG_HIP(ctx, hipStreamSynchronize(s));
    if (V >= kVidMask)
        return BITGNN_OK;

    // parts, sorted by (first block, last block, decreasing length)
    DevBuf v_beg, v_end, v_slot, vk_a, vk_b;
    BG_HIP(ctx, v_beg.alloc((size_t)V * 4));
    BG_HIP(ctx, v_end.alloc((size_t)V * 4));
    BG_HIP(ctx, v_slot.alloc((size_t)V * 4));
    BG_HIP(ctx, vk_a.alloc((size_t)V * 8));
    BG_HIP(ctx, vk_b.alloc((size_t)V * 8));
    vrow_kernel<<<blocks_for(n, 256), 256, 0, s>>>(skeys, rp2, vptr, n, cbits, cbn,
                                                  v_beg.as<uint32_t>(), v_end.as<uint32_t>(),
                                                  v_slot.as<uint32_t>(), vk_a.as<uint64_t>());
    BG_LAUNCH_CHECK(ctx, "vrow");
    // V <= nnz + n, so the histogram buffers sized for sort_n suffice when V <= sort_n;
    // V can exceed sort_n only if n > nnz, i.e. never on the graphs that get here
    if ((V + kSortTile - 1) / kSortTile > sort_tiles)
        return BITGNN_OK;
    uint64_t *svkeys = radix_sort(vk_a.as<uint64_t>(), vk_b.as<uint64_t>(), V, 64,
                                  hist.as<uint32_t>(), scan_ws.as<uint32_t>(), s);

    // work items of 16 slices, or of 8 or 4 on graphs with too few slices to give every
    // compute unit an item of 16 (measured on the 131 K-node R-MAT graph: 126 us per
    // aggregation with 135 items of 16 slices, 107 us with 270 items of 8)
    const uint32_t S = (V + 63) / 64;
    uint32_t spw = kSlicesPerWg;
    const uint32_t want = (uint32_t)(ctx->n_cus > 0 ? ctx->n_cus : 256);
    while (spw > 4 && (S + spw - 1) / spw < want)
        spw /= 2;
    const uint32_t W = (S + spw - 1) / spw;
    DevBuf sl_cb, sl_tile_base, wg_cb, part_info;
    BG_HIP(ctx, sl_cb.alloc((size_t)S * 4));
    BG_HIP(ctx, sl_tile_base.alloc(((size_t)S + 1) * 4));
    BG_HIP(ctx, wg_cb.alloc((size_t)W * 4));
    BG_HIP(ctx, part_info.alloc((size_t)V * 8));
    slice_range_kernel<<<S + 1, 64, 0, s>>>(svkeys, V, S, sl_cb.as<uint32_t>(),
                                            sl_tile_base.as<uint32_t>());
    scan_inplace(sl_tile_base.as<uint32_t>(), S + 1, scan_ws.as<uint32_t>(), s);
    uint32_t T = 0;
    BG_HIP(ctx, hipMemcpyAsync(&T, sl_tile_base.as<uint32_t>() + S, 4, hipMemcpyDeviceToHost, s));
    BG_HIP(ctx, hipStreamSynchronize(s));

    DevBuf tile_group;
    BG_HIP(ctx, tile_group.alloc(((size_t)T + 1) * 4));
    BG_HIP(ctx, hipMemsetAsync(tile_group.as<uint32_t>() + T, 0, 4, s));
    tile_kernel<false><<<S, 64, 0, s>>>(svkeys, V, v_beg.as<uint32_t>(), v_end.as<uint32_t>(),
                                        skeys, cbits, cbn, sl_cb.as<uint32_t>(),
                                        sl_tile_base.as<uint32_t>(), tile_group.as<uint32_t>(),
                                        nullptr);
    BG_LAUNCH_CHECK(ctx, "tile count");
    // the number of tiles is not bounded by the sizes above (sparse rows that span many
    // column blocks): size the workspace of this scan by itself
    DevBuf tile_scan_ws;
    BG_HIP(ctx, tile_scan_ws.alloc(scan_ws_words((uint64_t)T + 1) * 4));
    scan_inplace(tile_group.as<uint32_t>(), T + 1, tile_scan_ws.as<uint32_t>(), s);
    uint32_t G = 0;
    BG_HIP(ctx, hipMemcpyAsync(&G, tile_group.as<uint32_t>() + T, 4, hipMemcpyDeviceToHost, s));
    BG_HIP(ctx, hipStreamSynchronize(s));
    constexpr uint64_t kGroupIds = 64ull * kGroupSteps;
    if (((uint64_t)G + 1) * kGroupIds * 2 >= (1ull << 32)) // the kernel uses 32-bit byte offsets
        return BITGNN_OK;
    // Many column blocks with few neighbours each pad the tiles heavily: beyond 6 stored
    // ids per non-zero the plain CSR kernel is the better choice (a threshold of 0 stored
    // non-zeros per node forces the blocked form whatever the padding).
    if (ctx->min_avg_degree > 0 && (uint64_t)G * kGroupIds > 6ull * nnz)
        return BITGNN_OK;

    DevBuf idx16;
    BG_HIP(ctx, idx16.alloc(((size_t)G + 1) * kGroupIds * 2));
    tail_group_kernel<<<blocks_for((int64_t)kGroupIds, 256), 256, 0, s>>>(idx16.as<uint16_t>(), G,
                                                                         cbn);
    tile_kernel<true><<<S, 64, 0, s>>>(svkeys, V, v_beg.as<uint32_t>(), v_end.as<uint32_t>(), skeys,
                                       cbits, cbn, sl_cb.as<uint32_t>(),
                                       sl_tile_base.as<uint32_t>(), tile_group.as<uint32_t>(),
                                       idx16.as<uint16_t>());
    BG_LAUNCH_CHECK(ctx, "tile fill");
    part_info_kernel<<<blocks_for(V, 256), 256, 0, s>>>(svkeys, V, v_slot.as<uint32_t>(),
                                                       adj->order, part_info.as<uint2>());
    wg_range_kernel<<<blocks_for(W, 256), 256, 0, s>>>(sl_cb.as<uint32_t>(), S, W, spw,
                                                      wg_cb.as<uint32_t>());
    BG_LAUNCH_CHECK(ctx, "wg_range");
    // dispatch order: heaviest workgroups first (the key buffers of the parts are free again)
    DevBuf wg_item, sl_desc;
    BG_HIP(ctx, wg_item.alloc((size_t)W * 8));
    BG_HIP(ctx, sl_desc.alloc((size_t)S * 16));
    wg_cost_kernel<<<blocks_for(W, 64), 64, 0, s>>>(wg_cb.as<uint32_t>(), sl_cb.as<uint32_t>(),
                                                   sl_tile_base.as<uint32_t>(),
                                                   tile_group.as<uint32_t>(), S, W, spw, cbn,
                                                   vk_a.as<uint64_t>());
    uint64_t *wsorted = radix_sort(vk_a.as<uint64_t>(), vk_b.as<uint64_t>(), W, 64,
                                   hist.as<uint32_t>(), scan_ws.as<uint32_t>(), s);
    wg_item_kernel<<<blocks_for(W, 256), 256, 0, s>>>(wsorted, W, wg_cb.as<uint32_t>(),
                                                     wg_item.as<uint2>());
    slice_desc_kernel<<<blocks_for(S, 256), 256, 0, s>>>(sl_cb.as<uint32_t>(),
                                                        sl_tile_base.as<uint32_t>(),
                                                        tile_group.as<uint32_t>(), S,
                                                        sl_desc.as<uint4>());
    BG_LAUNCH_CHECK(ctx, "wg_item / slice_desc");
    BG_HIP(ctx, hipStreamSynchronize(s));

    bitgnn_blocked *b = (bitgnn_blocked *)calloc(1, sizeof(bitgnn_blocked));
    BG_REQUIRE(ctx, b, BITGNN_ERR_INVALID_ARG, "bitgnn_adj_build: out of host memory");
    b->cbn = cbn;
    b->n_multi = n_multi;
    b->ncb = (int32_t)ncb;
    b->part_len = part_len;
    b->forced = ctx->min_avg_degree == 0;
    b->n_vrows = V;
    b->n_slices = S;
    b->spw = (int32_t)spw;
    b->n_wgs = W;
    b->n_tiles = T;
    b->n_groups = G;
    b->device_bytes = ((size_t)G + 1) * kGroupIds * 2 + ((size_t)T + 1) * 4 + (size_t)S * 16 +
                      (size_t)W * 8 + ((size_t)n + 1) * 4 + (size_t)V * 8;
    b->wg_item = (uint2 *)wg_item.release();
    b->sl_desc = (uint4 *)sl_desc.release();
    b->tile_group = (uint32_t *)tile_group.release();
    b->idx16 = (uint16_t *)idx16.release();
    b->row_vptr = (uint32_t *)nparts.release();
    b->part_info = (uint2 *)part_info.release();
    adj->blk = b;
    adj->device_bytes += b->device_bytes;
    return BITGNN_OK;
}
