// Adjacency builder: edge list -> 0/1 aggregation matrix A_hat as a set of
// (row, col) pairs (Section 2.1: A_hat = A + I; Section 3.2.1: the sparse bit
// matrix only stores which entries are 1).
//
// Everything runs on the GPU with hand-written kernels:
//   1. one 64-bit key (row << cb | col) per directed pair (+ reversed pairs,
//      + diagonal), endpoints range-checked;
//   2. LSD radix sort of the keys, 8 bits per pass, one wavefront per tile of
//      2048 keys; the stable rank inside a wave comes from 8 wave votes
//      (lanes with the same digit find each other through the vote masks);
//   3. duplicates dropped with a flag-scan-compact;
//   4. row pointers by binary search of each row's first key, degrees, and a
//      degree-sorted row order (rows of similar length share a wavefront in
//      the aggregation kernel).
// The paper's 4x4 bit tiles are not used: at the densities of these graphs a
// tile holds one non-zero (Section 4.2 says the same of its own data), so the
// fine-grained format here is the sorted column list itself.
#include "prims.h"

#include <stdlib.h>

namespace {

// ---------------------------------------------------------------- keys
__global__ void make_keys_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                                 uint32_t E, uint32_t N, int symmetrize, int self_loops, int cb,
                                 uint64_t *__restrict__ keys, int *__restrict__ err)
{
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < E) {
        uint32_t i = (uint32_t)src[t], j = (uint32_t)dst[t];
        if (i >= N || j >= N) { // negative values wrap to >= 2^31 > N
            atomicOr(err, 1);
            i = 0;
            j = 0;
        }
        keys[t] = ((uint64_t)i << cb) | j;
        if (symmetrize)
            keys[(uint64_t)E + t] = ((uint64_t)j << cb) | i;
    }
    if (self_loops && t < N)
        keys[(uint64_t)E * (symmetrize ? 2 : 1) + t] = ((uint64_t)t << cb) | t;
}

// ---------------------------------------------------------------- unique
__global__ __launch_bounds__(kScanThreads) void uniq_count_kernel(const uint64_t *__restrict__ keys,
                                                                  uint32_t n,
                                                                  uint32_t *__restrict__ counts)
{
    const uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        const uint32_t i = base + k;
        if (i < n && (i == 0 || keys[i] != keys[i - 1]))
            ++s;
    }
    uint32_t total;
    (void)block_exclusive_scan(s, &total);
    if (threadIdx.x == 0)
        counts[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void uniq_compact_kernel(
    const uint64_t *__restrict__ keys, uint32_t n, const uint32_t *__restrict__ offs,
    uint64_t *__restrict__ out)
{
    const uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    bool f[kScanItems];
    uint64_t kv[kScanItems];
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        const uint32_t i = base + k;
        kv[k] = (i < n) ? keys[i] : 0;
        f[k] = i < n && (i == 0 || kv[k] != keys[i - 1]);
        s += f[k];
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan(s, &total) + offs[blockIdx.x];
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
        if (f[k])
            out[run++] = kv[k];
}

// ---------------------------------------------------------------- CSR
__global__ void split_keys_kernel(const uint64_t *__restrict__ ukeys, uint32_t nnz, int cb,
                                  int32_t *__restrict__ col)
{
    const uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u < nnz)
        col[u] = (int32_t)(ukeys[u] & ((1ull << cb) - 1));
}

// rowptr[r] = index of the first key whose row is >= r (r = 0..N).
__global__ void rowptr_kernel(const uint64_t *__restrict__ ukeys, uint32_t nnz, int cb, uint32_t N,
                              uint32_t *__restrict__ rowptr)
{
    const uint32_t r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r > N)
        return;
    const uint64_t want = (uint64_t)r << cb;
    uint32_t lo = 0, hi = nnz;
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if (ukeys[mid] < want)
            lo = mid + 1;
        else
            hi = mid;
    }
    rowptr[r] = lo;
}

__global__ void degree_kernel(const uint32_t *__restrict__ rowptr, uint32_t N,
                              int32_t *__restrict__ deg, uint64_t *__restrict__ order_keys,
                              int *__restrict__ max_deg)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N)
        return;
    const uint32_t d = rowptr[i + 1] - rowptr[i];
    deg[i] = (int32_t)d;
    // ascending sort of this key = decreasing degree, ties by row id
    order_keys[i] = ((uint64_t)(0xFFFFFFFFu - d) << 32) | i;
    atomicMax(max_deg, (int)d);
}

__global__ void rank_kernel(const int32_t *__restrict__ order, uint32_t N,
                            int32_t *__restrict__ rank)
{
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < N)
        rank[order[s]] = (int32_t)s;
}

// Segment counts of the rows in degree order (entry N is 0, so that the exclusive scan of
// N + 1 entries ends with the total), and the number of rows with more than one segment
// (they are the first ones of the order).
__global__ void seg_count_kernel(const int32_t *__restrict__ order, const int32_t *__restrict__ deg,
                                 uint32_t N, uint32_t seg_len, uint32_t *__restrict__ nseg,
                                 uint32_t *__restrict__ n_long)
{
    const uint32_t slot = blockIdx.x * blockDim.x + threadIdx.x;
    if (slot > N)
        return;
    uint32_t c = 0;
    if (slot < N) {
        const uint32_t d = (uint32_t)deg[order[slot]];
        c = d <= seg_len ? 1u : (d + seg_len - 1) / seg_len;
        if (c > 1)
            atomicMax(n_long, slot + 1);
    }
    nseg[slot] = c;
}

__global__ void seg_slot_kernel(const uint32_t *__restrict__ seg_ptr, uint32_t n_long,
                                uint32_t *__restrict__ seg_slot)
{
    const uint32_t slot = blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= n_long)
        return;
    for (uint32_t v = seg_ptr[slot]; v < seg_ptr[slot + 1]; ++v)
        seg_slot[v] = slot;
}

__global__ void col_slot_kernel(const int32_t *__restrict__ col, uint32_t nnz,
                                const int32_t *__restrict__ rank, int32_t *__restrict__ col_slot)
{
    const uint32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < nnz)
        col_slot[e] = rank[col[e]];
}

__global__ void order_from_keys_kernel(const uint64_t *__restrict__ keys, uint32_t N,
                                       int32_t *__restrict__ order)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N)
        order[i] = (int32_t)(uint32_t)keys[i];
}

} // namespace

// Second half of the build, on a handle that already owns the CSR arrays (the caller
// destroys the handle when this fails): degree-order column slots, row segments.
static int adj_finish(bitgnn_ctx *ctx, hipStream_t s, bitgnn_adj *adj)
{
    const int64_t N = adj->n;
    const uint32_t nnz = (uint32_t)adj->nnz;
    // CSR-only and larger than a cache: column ids in degree-order slots.  On a power-law
    // graph a few percent of the nodes take half of all gathers; in a degree-ordered copy of
    // the activations their rows are adjacent and stay in L2.
    if (!adj->blk && nnz > 0 && N >= 65536) {
        DevBuf rank, col_slot;
        BG_HIP(ctx, rank.alloc((size_t)N * 4));
        BG_HIP(ctx, col_slot.alloc((size_t)nnz * 4));
        rank_kernel<<<blocks_for(N, 256), 256, 0, s>>>(adj->order, (uint32_t)N, rank.as<int32_t>());
        col_slot_kernel<<<blocks_for(nnz, 256), 256, 0, s>>>(adj->col, nnz, rank.as<int32_t>(),
                                                            col_slot.as<int32_t>());
        BG_LAUNCH_CHECK(ctx, "col_slot");
        BG_HIP(ctx, hipStreamSynchronize(s));
        adj->col_slot = (int32_t *)col_slot.release();
        adj->device_bytes += (size_t)nnz * 4;
    }
    // segments of the long rows for the CSR bit-SpMM
    if (N > 0) {
        DevBuf nseg, seg_slot, cnt;
        BG_HIP(ctx, nseg.alloc(((size_t)N + 1) * 4));
        BG_HIP(ctx, cnt.alloc(4));
        BG_HIP(ctx, hipMemsetAsync(cnt.p, 0, 4, s));
        adj->seg_len = (int64_t)nnz >= kSegLargeNnz ? kSegLenLarge : kSegLenSmall;
        seg_count_kernel<<<blocks_for(N + 1, 256), 256, 0, s>>>(
            adj->order, adj->deg, (uint32_t)N, adj->seg_len, nseg.as<uint32_t>(),
            cnt.as<uint32_t>());
        BG_LAUNCH_CHECK(ctx, "seg_count");
        DevBuf sws;
        BG_HIP(ctx, sws.alloc(scan_ws_words((uint64_t)N + 1) * 4));
        scan_inplace(nseg.as<uint32_t>(), (uint32_t)N + 1, sws.as<uint32_t>(), s);
        uint32_t n_long = 0, n_long_segs = 0;
        BG_HIP(ctx, hipMemcpyAsync(&n_long, cnt.p, 4, hipMemcpyDeviceToHost, s));
        BG_HIP(ctx, hipStreamSynchronize(s));
        if (n_long > 0) {
            BG_HIP(ctx, hipMemcpyAsync(&n_long_segs, nseg.as<uint32_t>() + n_long, 4,
                                       hipMemcpyDeviceToHost, s));
            BG_HIP(ctx, hipStreamSynchronize(s));
            BG_HIP(ctx, seg_slot.alloc((size_t)n_long_segs * 4));
            seg_slot_kernel<<<blocks_for(n_long, 256), 256, 0, s>>>(nseg.as<uint32_t>(), n_long,
                                                                   seg_slot.as<uint32_t>());
            BG_LAUNCH_CHECK(ctx, "seg_slot");
            BG_HIP(ctx, hipStreamSynchronize(s));
            adj->seg_slot = (uint32_t *)seg_slot.release();
            adj->seg_ptr = (uint32_t *)nseg.release(); // the first n_long + 1 entries are used
            adj->device_bytes += ((size_t)N + 1) * 4 + (size_t)n_long_segs * 4;
        }
        adj->n_long = n_long;
        adj->n_long_segs = n_long_segs;
    }
    return BITGNN_OK;
}

extern "C" int bitgnn_adj_build(bitgnn_ctx *ctx, void *stream, const int32_t *src,
                                const int32_t *dst, int64_t E, int64_t N, uint32_t flags,
                                bitgnn_adj **out)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, out, BITGNN_ERR_INVALID_ARG, "bitgnn_adj_build: out is null");
    BG_REQUIRE(ctx, E >= 0 && N >= 1, BITGNN_ERR_INVALID_ARG, "bitgnn_adj_build: E=%lld N=%lld",
               (long long)E, (long long)N);
    BG_REQUIRE(ctx, (flags & ~3u) == 0, BITGNN_ERR_INVALID_ARG, "bitgnn_adj_build: flags=%u",
               flags);
    BG_REQUIRE(ctx, E == 0 || (src && dst), BITGNN_ERR_INVALID_ARG,
               "bitgnn_adj_build: null edge arrays");
    BG_REQUIRE(ctx, bg_aligned(src, 4) && bg_aligned(dst, 4), BITGNN_ERR_ALIGNMENT,
               "bitgnn_adj_build: misaligned edge arrays");
    const bool sym = flags & BITGNN_ADJ_SYMMETRIZE;
    const bool loops = flags & BITGNN_ADJ_ADD_SELF_LOOPS;
    const int64_t nkeys64 = E * (sym ? 2 : 1) + (loops ? N : 0);
    BG_REQUIRE(ctx, nkeys64 + N < (1ll << 31), BITGNN_ERR_RANGE,
               "bitgnn_adj_build: %lld stored pairs + N exceed 32-bit offsets", (long long)nkeys64);
    BG_NEED_DEVICE(ctx);

    hipStream_t s = (hipStream_t)stream;
    BG_HIP(ctx, hipSetDevice(ctx->device));
    const uint32_t nkeys = (uint32_t)nkeys64;
    int cb = 1;
    while ((1ll << cb) < N)
        ++cb;

    const uint32_t sort_n = nkeys > (uint32_t)N ? nkeys : (uint32_t)N;
    const uint32_t sort_tiles = (sort_n + kSortTile - 1) / kSortTile;
    const uint32_t uniq_tiles = (nkeys + kScanTile - 1) / kScanTile;
    DevBuf keys_a, keys_b, hist, scan_ws, counts, flag;
    BG_HIP(ctx, keys_a.alloc((size_t)sort_n * 8));
    BG_HIP(ctx, keys_b.alloc((size_t)sort_n * 8));
    BG_HIP(ctx, hist.alloc((size_t)256 * sort_tiles * 4));
    BG_HIP(ctx, scan_ws.alloc(scan_ws_words((uint64_t)256 * sort_tiles) * 4));
    BG_HIP(ctx, counts.alloc(((size_t)uniq_tiles + 1) * 4));
    BG_HIP(ctx, flag.alloc(2 * sizeof(int)));
    BG_HIP(ctx, hipMemsetAsync(flag.p, 0, 2 * sizeof(int), s));
    int *d_err = flag.as<int>();
    int *d_maxdeg = d_err + 1;

    uint64_t *sorted = keys_a.as<uint64_t>();
    uint32_t nnz = 0;
    if (nkeys > 0) {
        const uint32_t span = (uint32_t)(E > N ? E : N);
        make_keys_kernel<<<blocks_for(span, 256), 256, 0, s>>>(
            src, dst, (uint32_t)E, (uint32_t)N, sym, loops, cb, keys_a.as<uint64_t>(), d_err);
        BG_LAUNCH_CHECK(ctx, "make_keys");
        sorted = radix_sort(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), nkeys, 2 * cb,
                            hist.as<uint32_t>(), scan_ws.as<uint32_t>(), s);
        BG_LAUNCH_CHECK(ctx, "radix_sort");
        uint64_t *other = sorted == keys_a.as<uint64_t>() ? keys_b.as<uint64_t>()
                                                          : keys_a.as<uint64_t>();
        uniq_count_kernel<<<uniq_tiles, kScanThreads, 0, s>>>(sorted, nkeys, counts.as<uint32_t>());
        BG_HIP(ctx, hipMemsetAsync(counts.as<uint32_t>() + uniq_tiles, 0, 4, s));
        // hist is free again: use it as the scan workspace of the counts
        scan_inplace(counts.as<uint32_t>(), uniq_tiles + 1, hist.as<uint32_t>(), s);
        uniq_compact_kernel<<<uniq_tiles, kScanThreads, 0, s>>>(sorted, nkeys,
                                                                counts.as<uint32_t>(), other);
        BG_LAUNCH_CHECK(ctx, "unique");
        BG_HIP(ctx, hipMemcpyAsync(&nnz, counts.as<uint32_t>() + uniq_tiles, 4,
                                   hipMemcpyDeviceToHost, s));
        sorted = other;
    }
    int h_err = 0;
    BG_HIP(ctx, hipMemcpyAsync(&h_err, d_err, sizeof(int), hipMemcpyDeviceToHost, s));
    BG_HIP(ctx, hipStreamSynchronize(s));
    BG_REQUIRE(ctx, h_err == 0, BITGNN_ERR_INDEX_RANGE,
               "bitgnn_adj_build: an edge endpoint is outside [0, %lld)", (long long)N);

    DevBuf rowptr, col, deg, order;
    BG_HIP(ctx, rowptr.alloc(((size_t)N + 1) * 4));
    BG_HIP(ctx, col.alloc((size_t)nnz * 4));
    BG_HIP(ctx, deg.alloc((size_t)N * 4));
    BG_HIP(ctx, order.alloc((size_t)N * 4));
    if (nnz > 0)
        split_keys_kernel<<<blocks_for(nnz, 256), 256, 0, s>>>(sorted, nnz, cb, col.as<int32_t>());
    rowptr_kernel<<<blocks_for(N + 1, 256), 256, 0, s>>>(sorted, nnz, cb, (uint32_t)N,
                                                        rowptr.as<uint32_t>());
    // the sorted keys are consumed; reuse the two key buffers for the row order
    BG_HIP(ctx, hipStreamSynchronize(s));
    uint64_t *oa = keys_a.as<uint64_t>(), *ob = keys_b.as<uint64_t>();
    degree_kernel<<<blocks_for(N, 256), 256, 0, s>>>(rowptr.as<uint32_t>(), (uint32_t)N,
                                                    deg.as<int32_t>(), oa, d_maxdeg);
    BG_LAUNCH_CHECK(ctx, "degree");
    uint64_t *osorted =
        radix_sort(oa, ob, (uint32_t)N, 64, hist.as<uint32_t>(), scan_ws.as<uint32_t>(), s);
    order_from_keys_kernel<<<blocks_for(N, 256), 256, 0, s>>>(osorted, (uint32_t)N,
                                                             order.as<int32_t>());
    BG_LAUNCH_CHECK(ctx, "order");
    int h_maxdeg = 0;
    BG_HIP(ctx, hipMemcpyAsync(&h_maxdeg, d_maxdeg, sizeof(int), hipMemcpyDeviceToHost, s));
    BG_HIP(ctx, hipStreamSynchronize(s));

    bitgnn_adj *adj = (bitgnn_adj *)calloc(1, sizeof(bitgnn_adj));
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_adj_build: out of host memory");
    adj->device = ctx->device;
    adj->n = N;
    adj->nnz = nnz;
    adj->max_degree = h_maxdeg;
    adj->device_bytes = ((size_t)N + 1) * 4 + (size_t)nnz * 4 + (size_t)N * 8;
    adj->rowptr = (uint32_t *)rowptr.release();
    adj->col = (int32_t *)col.release();
    adj->deg = (int32_t *)deg.release();
    adj->order = (int32_t *)order.release();
    // dense enough: also build the column-blocked form for the LDS-staged bit-SpMM
    if ((int64_t)nnz >= (int64_t)ctx->min_avg_degree * N) {
        keys_a.reset();
        keys_b.reset();
        int rc = bg_build_blocked(ctx, s, adj);
        if (rc != BITGNN_OK) {
            bitgnn_adj_destroy(adj);
            return rc;
        }
    }
    int rc = adj_finish(ctx, s, adj);
    // the aggregation workspace for the default widths: compute calls never allocate
    if (rc == BITGNN_OK)
        rc = bitgnn_ctx_reserve(ctx, bg_adj_workspace_bytes(adj, kDefaultWsChannels,
                                                            kDefaultWsClasses));
    if (rc != BITGNN_OK) {
        bitgnn_adj_destroy(adj);
        return rc;
    }
    *out = adj;
    return BITGNN_OK;
}

extern "C" int bitgnn_adj_workspace_bytes(const bitgnn_adj *adj, int32_t C_max, int32_t M_max,
                                          size_t *bytes)
{
    if (!adj || !bytes || C_max < 1 || C_max > 2048 || M_max < 1)
        return BITGNN_ERR_INVALID_ARG;
    *bytes = bg_adj_workspace_bytes(adj, C_max, M_max);
    return BITGNN_OK;
}

extern "C" int bitgnn_adj_info(const bitgnn_adj *adj, int64_t *N, int64_t *nnz,
                               int64_t *max_degree, size_t *device_bytes)
{
    if (!adj)
        return BITGNN_ERR_INVALID_ARG;
    if (N)
        *N = adj->n;
    if (nnz)
        *nnz = adj->nnz;
    if (max_degree)
        *max_degree = adj->max_degree;
    if (device_bytes)
        *device_bytes = adj->device_bytes;
    return BITGNN_OK;
}

extern "C" int bitgnn_adj_csr(const bitgnn_adj *adj, const uint32_t **rowptr, const int32_t **col,
                              const int32_t **deg)
{
    if (!adj)
        return BITGNN_ERR_INVALID_ARG;
    if (rowptr)
        *rowptr = adj->rowptr;
    if (col)
        *col = adj->col;
    if (deg)
        *deg = adj->deg;
    return BITGNN_OK;
}

extern "C" int bitgnn_adj_blocked_info(const bitgnn_adj *adj, int64_t *parts, int64_t *slices,
                                       int64_t *workgroups, int64_t *tiles, int64_t *stored_ids,
                                       int64_t *cb_nodes)
{
    if (!adj)
        return BITGNN_ERR_INVALID_ARG;
    const bitgnn_blocked *b = adj->blk;
    if (parts)
        *parts = b ? b->n_vrows : 0;
    if (slices)
        *slices = b ? b->n_slices : 0;
    if (workgroups)
        *workgroups = b ? b->n_wgs : 0;
    if (tiles)
        *tiles = b ? b->n_tiles : 0;
    if (stored_ids)
        *stored_ids = b ? (int64_t)b->n_groups * 64 * kGroupSteps : 0;
    if (cb_nodes)
        *cb_nodes = b ? b->cbn : 0;
    return BITGNN_OK;
}

extern "C" void bitgnn_adj_destroy(bitgnn_adj *adj)
{
    if (!adj)
        return;
    (void)hipFree(adj->rowptr);
    (void)hipFree(adj->col);
    (void)hipFree(adj->deg);
    (void)hipFree(adj->order);
    (void)hipFree(adj->col_slot);
    (void)hipFree(adj->seg_ptr);
    (void)hipFree(adj->seg_slot);
    bg_free_blocked(adj->blk);
    free(adj);
}
