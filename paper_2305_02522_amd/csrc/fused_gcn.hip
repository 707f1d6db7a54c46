// Whole two-layer GCN in ONE kernel launch for small graphs (Section 3.3, the fused
// end-to-end kernel: every layer function runs inside one persistent grid and a
// grid-wide barrier stands where the un-fused model has a kernel boundary).
//
//   phase 1  h  = (bin(x) W1 >= T_mm)        BMM.FBB, float features voted into words
//   -- grid barrier --
//   phase 2  h1 = (A_hat h >= T_agg)         BSpMM.BBB, S = 2 cnt - deg
//   -- grid barrier --
//   phase 3  logits = alpha * ((A_hat h1) W2)   the output layer re-associated: the +-1
//                                               rows are summed first, the class
//                                               projection follows in the same wavefront
//
// On a citation-sized graph (thousands of nodes, a handful of neighbours per node) the
// three un-fused calls are each bound by launch latency, not by their work; here the
// whole model costs one launch and two barriers.
//
// gfx950 mapping: one workgroup of 1024 threads per compute unit at most, so that the
// whole grid is resident at once (the barrier needs that) and a barrier has few arrivals.
// The grid barrier is one arrival counter in device memory, advanced by the first lane of
// every workgroup (barrier k is passed at k x workgroups arrivals); the rows that cross it
// travel through device-scope accesses (see store_shared_word), which is what makes the
// rows written under one XCD's L2 visible to the workgroups under another's.  Every wait
// is bounded: a workgroup that gives up still arrives at the remaining barriers, raises the
// caller's status word and skips its work.  The counter is never reset: every launch adds
// exactly 2 x kParticipants to it (workgroup 0 also arrives for the workgroups the grid does
// not have), so each workgroup finds the launch's starting value by rounding what it reads
// at its start down to that multiple.  A launch therefore carries no state from the host:
// the call can be recorded into a HIP graph, and a launch that gave up leaves the counter
// in step.
// Measured, calls back to back: 17 us per model on the 2,708-node citation-shaped workload
// against 44 us for the layer calls (in the kernel: phase 1 ~7 us, each barrier ~3.3,
// phase 2 ~1, phase 3 ~2); 34 against 40 us at 19,717 nodes x 500 features; level with
// the layer calls at 65,536 nodes, behind them beyond (their kernels are the tuned ones).
#include "common.h"

namespace {

constexpr int kFusedBlock = 1024;
constexpr int kFusedWaves = kFusedBlock / 64;

constexpr uint32_t kParticipants = 1024; // arrivals per barrier (a power of two >= any grid)
constexpr uint32_t kBarriers = 2;

struct GridBarrier {
    uint32_t *counter; // device word, only ever incremented (wraps)
    uint32_t target;   // value that means "everyone arrived at the next barrier"
    uint32_t nblocks;
    uint32_t spin_limit; // polls of ~1 us each before a wait is abandoned
    bool alive;        // false once a wait was abandoned (block-uniform)
};

// The bit matrices that cross a barrier are written and read with device-scope accesses
// (relaxed atomics: the store is written through to memory before it is acknowledged, the
// load is served from there), so a barrier needs no cache write-back or invalidate -- those
// cost ~0.2 us each and serialize per L2, which with hundreds of workgroups is most of a
// barrier.  What it does need: every wavefront's stores acknowledged before its workgroup
// arrives, and no load of the next phase issued before the workgroup has left.
__device__ __forceinline__ void store_shared_word(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_shared_word(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All threads of the block call this.  Returns false if the wait timed out.
__device__ __forceinline__ bool grid_barrier(GridBarrier &b, int32_t *status)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this wavefront's rows are in memory
    __syncthreads();
    __shared__ int ok_flag;
    if (threadIdx.x == 0) {
        // workgroup 0 stands in for the participants the grid does not have
        __hip_atomic_fetch_add(b.counter, blockIdx.x == 0 ? kParticipants - b.nblocks + 1u : 1u,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int ok = b.alive ? 1 : 0;
        if (ok) {
            uint32_t spins = 0;
            while ((int32_t)(__hip_atomic_load(b.counter, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT) -
                             b.target) < 0) {
                __builtin_amdgcn_s_sleep(8);
                if (++spins > b.spin_limit) {
                    ok = 0;
                    if (status)
                        atomicAdd(status, 1);
                    break;
                }
            }
        }
        ok_flag = ok;
    }
    __syncthreads();
    b.alive = ok_flag != 0;
    b.target += kParticipants;
    return b.alive;
}

// Phase 1.  One wavefront finishes kRowsA node rows at a time (2, or 4 when every wavefront
// has several groups to do and more loads in flight pay): 64 lanes load 64 consecutive
// floats, the compare mask is the activation word; lane c owns output channel c of each
// tile and holds kChunkA 64-bit weight words of it per step.
template <int TILES, int kRowsA>
__device__ __forceinline__ void phase_bmm_f32(const float *__restrict__ x, int64_t n, int32_t K,
                                              int64_t ldx, const uint64_t *__restrict__ w,
                                              int64_t w_stride, int32_t M,
                                              const int32_t *__restrict__ T,
                                              uint64_t *__restrict__ out, int64_t out_stride,
                                              int64_t gwave, int64_t nwaves, int lane)
{
    constexpr int kChunkA = TILES == 4 ? 4 : 8;
    const int32_t kw = (K + 63) / 64;
    const uint64_t *wrow[TILES];
    bool c_ok[TILES];
    int32_t tc[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int c = t * 64 + lane;
        c_ok[t] = c < M;
        wrow[t] = w + (int64_t)(c_ok[t] ? c : 0) * w_stride;
        tc[t] = c_ok[t] ? T[c] : 0;
    }
    const int64_t ngroups = (n + kRowsA - 1) / kRowsA;
    for (int64_t g = gwave; g < ngroups; g += nwaves) {
        int acc[kRowsA][TILES];
#pragma unroll
        for (int r = 0; r < kRowsA; ++r)
#pragma unroll
            for (int t = 0; t < TILES; ++t)
                acc[r][t] = 0;
        const float *xr[kRowsA];
#pragma unroll
        for (int r = 0; r < kRowsA; ++r) {
            const int64_t row = g * kRowsA + r < n ? g * kRowsA + r : n - 1; // wave-uniform
            xr[r] = x + row * ldx;
        }
        for (int32_t k0 = 0; k0 < kw; k0 += kChunkA) {
            float v[kRowsA][kChunkA];
            uint64_t okmask[kChunkA];
#pragma unroll
            for (int j = 0; j < kChunkA; ++j) {
                const int32_t k = (k0 + j) * 64 + lane;
                okmask[j] = __ballot(k < K);
                const int32_t kk = k < K ? k : K - 1; // clamped: no load is conditional
#pragma unroll
                for (int r = 0; r < kRowsA; ++r)
                    v[r][j] = xr[r][kk];
            }
            uint64_t wv[TILES][kChunkA];
#pragma unroll
            for (int t = 0; t < TILES; ++t)
#pragma unroll
                for (int j = 0; j < kChunkA; ++j)
                    wv[t][j] = (k0 + j < kw && c_ok[t]) ? wrow[t][k0 + j] : 0ull;
#pragma unroll
            for (int j = 0; j < kChunkA; ++j)
#pragma unroll
                for (int r = 0; r < kRowsA; ++r) {
                    // beyond K the vote is 0 and so are the weight words
                    const uint64_t m = __ballot(v[r][j] >= 0.0f) & okmask[j];
#pragma unroll
                    for (int t = 0; t < TILES; ++t)
                        acc[r][t] += __popcll(m ^ wv[t][j]);
                }
        }
#pragma unroll
        for (int r = 0; r < kRowsA; ++r) {
            const int64_t row = g * kRowsA + r;
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                const uint64_t word = __ballot(c_ok[t] && K - 2 * acc[r][t] >= tc[t]);
                if (row < n && t * 64 < M && lane == 0)
                    store_shared_word(&out[row * out_stride + t], word);
            }
        }
    }
}

struct RowRange {
    uint32_t row, beg, end; // wave-uniform; beg == end == 0 past the last row
};

__device__ __forceinline__ RowRange fetch_row(const int32_t *__restrict__ order,
                                              const uint32_t *__restrict__ rowptr, int64_t slot,
                                              int64_t n)
{
    RowRange r{0u, 0u, 0u};
    if (slot < n) {
        r.row = (uint32_t)order[slot];
        r.beg = rowptr[r.row];
        r.end = rowptr[r.row + 1];
    }
    return r;
}

// column index of the lane's neighbour among the first 64 of the row
__device__ __forceinline__ int32_t fetch_first_cols(const int32_t *__restrict__ col,
                                                    const RowRange &r, int lane)
{
    return r.beg + (uint32_t)lane < r.end ? col[r.beg + lane] : 0;
}

// adds, for every tile, the bits of this lane's channel over the first m lanes' words
template <int TILES>
__device__ __forceinline__ void count_bits(const uint32_t (&lo)[TILES], const uint32_t (&hi)[TILES],
                                           uint32_t m, int (&cnt)[TILES])
{
    for (uint32_t l = 0; l < m; l += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) { // lanes past m hold zero words
            const int src_lane = (int)((l + u) & 63u);
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                const uint64_t word =
                    (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)lo[t], src_lane) |
                    ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi[t], src_lane) << 32);
                cnt[t] += __builtin_amdgcn_inverse_ballot_w64(word) ? 1 : 0;
            }
        }
    }
}

// Walks the wavefront's rows (slots gwave, gwave + nwaves, ... of the degree order), R rows
// at a time, and hands each row's counts -- the number of neighbours whose bit of channel
// (tile, lane) is set -- to `emit(row, degree, cnt)`.  64 neighbours of a row are taken at
// once: lane l fetches the words of neighbour l, then the words go round by lane broadcast
// and each lane picks its own bit.  A row costs four dependent memory latencies (order, row
// pointers, column indices, words); the R rows of a step go through them together.
template <int TILES, int R, class Emit>
__device__ __forceinline__ void for_each_row(const uint32_t *__restrict__ rowptr,
                                             const int32_t *__restrict__ col,
                                             const int32_t *__restrict__ order, int64_t n,
                                             int64_t gwave, int64_t nwaves, const uint64_t *src,
                                             int64_t src_stride, int mw, int lane, Emit &&emit)
{
    for (int64_t slot0 = gwave; slot0 < n; slot0 += R * nwaves) {
        RowRange r[R];
#pragma unroll
        for (int q = 0; q < R; ++q)
            r[q] = fetch_row(order, rowptr, slot0 + q * nwaves, n);
        int32_t j[R];
#pragma unroll
        for (int q = 0; q < R; ++q)
            j[q] = fetch_first_cols(col, r[q], lane);
        uint32_t lo[R][TILES], hi[R][TILES];
#pragma unroll
        for (int q = 0; q < R; ++q)
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                // lanes without a neighbour hold zero words: they count nothing
                const bool mine = r[q].beg + (uint32_t)lane < r[q].end;
                const uint64_t wd = (mine && t < mw)
                                        ? load_shared_word(&src[(int64_t)j[q] * src_stride + t])
                                        : 0ull;
                lo[q][t] = (uint32_t)wd;
                hi[q][t] = (uint32_t)(wd >> 32);
            }
#pragma unroll
        for (int q = 0; q < R; ++q) {
            int cnt[TILES];
#pragma unroll
            for (int t = 0; t < TILES; ++t)
                cnt[t] = 0;
            const uint32_t deg = r[q].end - r[q].beg;
            count_bits<TILES>(lo[q], hi[q], deg < 64u ? deg : 64u, cnt);
            for (uint32_t e0 = r[q].beg + 64; e0 < r[q].end; e0 += 64) { // long rows
                const uint32_t m = r[q].end - e0 < 64u ? r[q].end - e0 : 64u;
                const bool mine = (uint32_t)lane < m;
                const int32_t jj = mine ? col[e0 + lane] : 0;
                uint32_t l2[TILES], h2[TILES];
#pragma unroll
                for (int t = 0; t < TILES; ++t) {
                    const uint64_t wd = (mine && t < mw)
                                            ? load_shared_word(&src[(int64_t)jj * src_stride + t])
                                            : 0ull;
                    l2[t] = (uint32_t)wd;
                    h2[t] = (uint32_t)(wd >> 32);
                }
                count_bits<TILES>(l2, h2, m, cnt);
            }
            if (slot0 + q * nwaves < n)
                emit(r[q].row, deg, cnt);
        }
    }
}

template <int TILES, int ROWS_A>
__global__ __launch_bounds__(kFusedBlock) void gcn2_fused_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, int64_t n, const float *__restrict__ x, int32_t K0,
    int64_t ldx, const uint64_t *__restrict__ w1, int32_t C1, int64_t w1_stride,
    const int32_t *__restrict__ T_mm, const int32_t *__restrict__ T_agg,
    const uint64_t *__restrict__ w2, int32_t M, int64_t w2_stride,
    const float *__restrict__ alpha, uint64_t *tmp_bits, uint64_t *h_bits, int64_t h_stride,
    float *__restrict__ logits, int64_t ldo, uint32_t *bar_counter, uint32_t spin_limit,
    int32_t *status)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // consecutive work items go to different workgroups (rows come by decreasing degree)
    const int64_t gwave = (int64_t)wave * gridDim.x + blockIdx.x;
    const int64_t nwaves = (int64_t)gridDim.x * kFusedWaves;
    const int64_t mw = ((int64_t)C1 + 63) / 64;
    constexpr int kRowsB = TILES == 4 ? 2 : 4; // rows of an aggregation step in flight
    // Read before this workgroup's first arrival: the counter is then less than one launch's
    // worth (kBarriers x kParticipants) past the launch's starting value, a multiple of that.
    const uint32_t seen =
        __hip_atomic_load(bar_counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    GridBarrier bar{bar_counter, (seen & ~(kBarriers * kParticipants - 1u)) + kParticipants,
                    gridDim.x, spin_limit, true};

    phase_bmm_f32<TILES, ROWS_A>(x, n, K0, ldx, w1, w1_stride, C1, T_mm, tmp_bits, mw, gwave, nwaves,
                         lane);

    const bool go2 = grid_barrier(bar, status);
    if (go2) {
        int32_t ta[TILES];
        bool c_ok[TILES];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            c_ok[t] = t * 64 + lane < C1;
            ta[t] = c_ok[t] ? T_agg[t * 64 + lane] : 0;
        }
        for_each_row<TILES, kRowsB>(rowptr, col, order, n, gwave, nwaves, tmp_bits, mw, (int)mw, lane,
                            [&](uint32_t row, uint32_t deg, const int (&cnt)[TILES]) {
#pragma unroll
                                for (int t = 0; t < TILES; ++t) {
                                    const uint64_t word =
                                        __ballot(c_ok[t] && 2 * cnt[t] - (int)deg >= ta[t]);
                                    if (t * 64 < C1 && lane == 0)
                                        store_shared_word(&h_bits[(int64_t)row * h_stride + t],
                                                          word);
                                }
                            });
    }

    const bool go3 = grid_barrier(bar, status);
    if (go3) {
        // Lane m owns class m and keeps its weight words.  With the counts cnt_c of a row
        // (lane c) and w = 2 bit - 1:
        //   sum_c w_mc (2 cnt_c - deg) = 2 sum_c w_mc cnt_c - deg (2 popc(W_m) - C1),
        //   sum_c w_mc cnt_c = sum_b 2^b (2 popc(P_b & W_m) - popc(P_b)),
        // where P_b is the wave-wide vote "bit b of cnt_c is set": a handful of votes and
        // popcounts per row, whatever the number of classes.
        uint64_t wm[TILES];
        int wsum = -C1;
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            wm[t] = (lane < M && t < mw) ? w2[(int64_t)lane * w2_stride + t] : 0ull;
            wsum += 2 * __popcll(wm[t]);
        }
        const float al = lane < M ? alpha[lane] : 0.0f;
        for_each_row<TILES, kRowsB>(
            rowptr, col, order, n, gwave, nwaves, h_bits, h_stride, (int)mw, lane,
            [&](uint32_t row, uint32_t deg, const int (&cnt)[TILES]) {
                const int planes = 32 - __clz((int)deg); // cnt <= deg; wave-uniform
                int acc = 0;
#pragma unroll
                for (int t = 0; t < TILES; ++t)
                    for (int b = 0; b < planes; ++b) {
                        const uint64_t pb = __ballot((cnt[t] >> b) & 1);
                        acc += (2 * __popcll(pb & wm[t]) - __popcll(pb)) << b;
                    }
                const int res = 2 * acc - (int)deg * wsum;
                if (lane < M)
                    logits[(int64_t)row * ldo + lane] = al * (float)res;
            });
    }
}

} // namespace

extern "C" int bitgnn_ctx_set_fused_spin_limit(bitgnn_ctx *ctx, uint32_t polls)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, polls >= 1, BITGNN_ERR_INVALID_ARG,
               "bitgnn_ctx_set_fused_spin_limit: polls must be >= 1");
    ctx->fused_spin_limit = polls;
    return BITGNN_OK;
}

extern "C" int bitgnn_gcn2_fused(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                 const float *x, int32_t K0, int64_t ldx, const uint64_t *w1bits,
                                 int32_t C1, int64_t w1_stride, const int32_t *T_mm,
                                 const int32_t *T_agg, const uint64_t *w2bits, int32_t M,
                                 int64_t w2_stride, const float *alpha, uint64_t *tmp_bits,
                                 uint64_t *h_bits, int64_t h_stride, float *logits, int64_t ldo,
                                 int32_t *status)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn2_fused: adj is null");
    const int64_t n = adj->n;
    const int64_t mw = ((int64_t)C1 + 63) / 64;
    BG_REQUIRE(ctx, K0 >= 1 && C1 >= 1 && M >= 1, BITGNN_ERR_INVALID_ARG,
               "bitgnn_gcn2_fused: K0=%d C1=%d M=%d", K0, C1, M);
    BG_REQUIRE(ctx, x && w1bits && T_mm && T_agg && w2bits && alpha && tmp_bits && h_bits &&
                        logits,
               BITGNN_ERR_INVALID_ARG, "bitgnn_gcn2_fused: null pointer");
    BG_REQUIRE(ctx, ldx >= K0 && w1_stride >= ((int64_t)K0 + 63) / 64 && w2_stride >= mw &&
                        h_stride >= mw && ldo >= M,
               BITGNN_ERR_INVALID_ARG,
               "bitgnn_gcn2_fused: ldx=%lld w1_stride=%lld w2_stride=%lld h_stride=%lld ldo=%lld "
               "too small for K0=%d C1=%d M=%d",
               (long long)ldx, (long long)w1_stride, (long long)w2_stride, (long long)h_stride,
               (long long)ldo, K0, C1, M);
    BG_REQUIRE(ctx, bg_aligned(x, 4) && bg_aligned(T_mm, 4) && bg_aligned(T_agg, 4) &&
                        bg_aligned(alpha, 4) && bg_aligned(logits, 4) &&
                        bg_aligned(status, 4) && bg_aligned(w1bits, 8) && bg_aligned(w2bits, 8) &&
                        bg_aligned(tmp_bits, 8) && bg_aligned(h_bits, 8),
               BITGNN_ERR_ALIGNMENT, "bitgnn_gcn2_fused: misaligned pointer");
    BG_REQUIRE(ctx, n >= 1 && n <= BITGNN_FUSED_MAX_NODES &&
                        adj->max_degree <= BITGNN_FUSED_MAX_DEGREE &&
                        C1 <= BITGNN_FUSED_MAX_HIDDEN && M <= BITGNN_FUSED_MAX_CLASSES,
               BITGNN_ERR_RANGE,
               "bitgnn_gcn2_fused: n=%lld max_degree=%lld C1=%d M=%d outside the fused kernel's "
               "range (n <= %d, degree <= %d, C1 <= %d, M <= %d): use the layer calls",
               (long long)n, (long long)adj->max_degree, C1, M, BITGNN_FUSED_MAX_NODES,
               BITGNN_FUSED_MAX_DEGREE, BITGNN_FUSED_MAX_HIDDEN, BITGNN_FUSED_MAX_CLASSES);
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;

    const int tiles = mw <= 1 ? 1 : mw <= 2 ? 2 : 4;
    const void *kernel = (const void *)gcn2_fused_kernel<4, 4>; // the largest variant
    // the whole grid must be resident at once: at most what the occupancy query allows
    static int per_cu = 0; // asked once per process: the answer depends on the code object only
    if (per_cu == 0)
        BG_HIP(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kFusedBlock, 0));
    BG_REQUIRE(ctx, per_cu >= 1, BITGNN_ERR_HIP, "bitgnn_gcn2_fused: kernel does not fit a CU");
    BG_REQUIRE(ctx, ctx->n_cus <= (int)kParticipants, BITGNN_ERR_UNSUPPORTED,
               "bitgnn_gcn2_fused: %d compute units, at most %u supported", ctx->n_cus,
               kParticipants);
    int64_t blocks = ctx->n_cus; // one per compute unit: fewer arrivals per barrier
    const int64_t useful = (n + kFusedWaves - 1) / kFusedWaves; // one row per wavefront
    if (blocks > useful)
        blocks = useful;
    uint32_t *counter = ctx->own.queue + kFusedBarrierWord;
    // four rows per phase-1 step once a wavefront would otherwise walk more than two steps
    const bool rows4 = (n + 1) / 2 > 2 * blocks * kFusedWaves;
#define BG_FUSED2(TV, RV)                                                                         \
    gcn2_fused_kernel<TV, RV><<<(unsigned)blocks, kFusedBlock, 0, s>>>(                           \
        adj->rowptr, adj->col, adj->order, n, x, K0, ldx, w1bits, C1, w1_stride, T_mm, T_agg,     \
        w2bits, M, w2_stride, alpha, tmp_bits, h_bits, h_stride, logits, ldo, counter,            \
        ctx->fused_spin_limit, status)
#define BG_FUSED(TV)                                                                              \
    do {                                                                                          \
        if (rows4)                                                                                \
            BG_FUSED2(TV, 4);                                                                     \
        else                                                                                      \
            BG_FUSED2(TV, 2);                                                                     \
    } while (0)
    if (tiles == 1)
        BG_FUSED(1);
    else if (tiles == 2)
        BG_FUSED(2);
    else
        BG_FUSED(4);
#undef BG_FUSED
#undef BG_FUSED2
    BG_LAUNCH_CHECK(ctx, "gcn2_fused_kernel");
    return BITGNN_OK;
}
