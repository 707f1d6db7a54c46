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
// gfx950 mapping: 256 threads per workgroup, at most two workgroups per compute unit so
// that the whole grid is resident at once (the barrier needs that); the grid barrier is
// one monotonic counter in device memory, advanced by the first lane of every workgroup
// with agent-scope release / acquire, which is what makes the rows written by one XCD's
// workgroups visible through another XCD's L2.  Every wait is bounded: a workgroup that
// gives up still arrives at the remaining barriers (so the counter stays in step with the
// host's count of launches), raises the caller's status word and skips its work.
// Rows produced inside the kernel are read with per-lane (vector) loads only.
#include "common.h"

namespace {

constexpr int kFusedBlock = 256;
constexpr int kFusedWaves = kFusedBlock / 64;
constexpr int kRowsA = 4;         // node rows a wavefront carries through phase 1
constexpr int kChunkA = 8;        // 64-bit words of the feature axis per register chunk
constexpr uint32_t kSpinLimit = 1u << 22; // polls of ~1 us each before a wait is abandoned
constexpr int kBarriers = 2;

struct GridBarrier {
    uint32_t *counter; // device word, only ever incremented
    uint32_t target;   // value that means "everyone arrived at the next barrier"
    uint32_t nblocks;
    bool alive;        // false once a wait was abandoned (block-uniform)
};

// All threads of the block call this.  Returns false if the wait timed out.
__device__ __forceinline__ bool grid_barrier(GridBarrier &b, int32_t *status)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); // this wavefront's rows are out
    __syncthreads();
    __shared__ int ok_flag;
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(b.counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        int ok = b.alive ? 1 : 0;
        if (ok) {
            uint32_t spins = 0;
            while ((int32_t)(__hip_atomic_load(b.counter, __ATOMIC_ACQUIRE,
                                               __HIP_MEMORY_SCOPE_AGENT) -
                             b.target) < 0) {
                __builtin_amdgcn_s_sleep(4);
                if (++spins > kSpinLimit) {
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
    b.target += b.nblocks;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); // drop stale lines before reading
    return b.alive;
}

// Phase 1.  One wavefront finishes kRowsA node rows: 64 lanes load 64 consecutive floats,
// the compare mask is the activation word; lane c owns output channel c of each tile.
template <int TILES>
__device__ __forceinline__ void phase_bmm_f32(const float *__restrict__ x, int64_t n, int32_t K,
                                              int64_t ldx, const uint64_t *__restrict__ w,
                                              int64_t w_stride, int32_t M,
                                              const int32_t *__restrict__ T,
                                              uint64_t *__restrict__ out, int64_t out_stride,
                                              int64_t gwave, int64_t nwaves, int lane)
{
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
                    out[row * out_stride + t] = word;
            }
        }
    }
}

// Number of neighbours of `row` whose bit of channel (tile, lane) is set, for every tile.
// The wavefront takes 64 neighbours at a time: lane l fetches the words of neighbour l,
// then the words go round by lane broadcast and each lane picks its own bit.
template <int TILES>
__device__ __forceinline__ void row_counts(const uint32_t *__restrict__ rowptr,
                                           const int32_t *__restrict__ col, uint32_t row,
                                           const uint64_t *src, int64_t src_stride, int mw,
                                           int lane, int (&cnt)[TILES], uint32_t &deg)
{
    const uint32_t beg = rowptr[row], end = rowptr[row + 1];
    deg = end - beg;
#pragma unroll
    for (int t = 0; t < TILES; ++t)
        cnt[t] = 0;
    for (uint32_t e0 = beg; e0 < end; e0 += 64) {
        const uint32_t m = end - e0 < 64u ? end - e0 : 64u; // wave-uniform
        const bool mine = (uint32_t)lane < m;
        const int32_t j = mine ? col[e0 + lane] : 0;
        uint32_t lo[TILES], hi[TILES];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            // lanes without a neighbour hold zero words: they count nothing
            const uint64_t wd = (mine && t < mw) ? src[(int64_t)j * src_stride + t] : 0ull;
            lo[t] = (uint32_t)wd;
            hi[t] = (uint32_t)(wd >> 32);
        }
        for (uint32_t l = 0; l < m; l += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int src_lane = (int)((l + u) & 63u);
#pragma unroll
                for (int t = 0; t < TILES; ++t) {
                    const uint64_t word =
                        (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)lo[t], src_lane) |
                        ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi[t], src_lane)
                         << 32);
                    cnt[t] += __builtin_amdgcn_inverse_ballot_w64(word) ? 1 : 0;
                }
            }
        }
    }
}

template <int TILES>
__global__ __launch_bounds__(kFusedBlock, 2) void gcn2_fused_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, int64_t n, const float *__restrict__ x, int32_t K0,
    int64_t ldx, const uint64_t *__restrict__ w1, int32_t C1, int64_t w1_stride,
    const int32_t *__restrict__ T_mm, const int32_t *__restrict__ T_agg,
    const uint64_t *__restrict__ w2, int32_t M, int64_t w2_stride,
    const float *__restrict__ alpha, uint64_t *tmp_bits, uint64_t *h_bits, int64_t h_stride,
    float *__restrict__ logits, int64_t ldo, uint32_t *bar_counter, uint32_t bar_base,
    int32_t *status)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gwave = (int64_t)blockIdx.x * kFusedWaves + wave;
    const int64_t nwaves = (int64_t)gridDim.x * kFusedWaves;
    const int64_t mw = ((int64_t)C1 + 63) / 64;
    GridBarrier bar{bar_counter, bar_base + gridDim.x, gridDim.x, true};

    phase_bmm_f32<TILES>(x, n, K0, ldx, w1, w1_stride, C1, T_mm, tmp_bits, mw, gwave, nwaves,
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
        for (int64_t slot = gwave; slot < n; slot += nwaves) {
            const uint32_t row = (uint32_t)order[slot];
            int cnt[TILES];
            uint32_t deg;
            row_counts<TILES>(rowptr, col, row, tmp_bits, mw, (int)mw, lane, cnt, deg);
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                const uint64_t word = __ballot(c_ok[t] && 2 * cnt[t] - (int)deg >= ta[t]);
                if (t * 64 < C1 && lane == 0)
                    h_bits[(int64_t)row * h_stride + t] = word;
            }
        }
    }

    const bool go3 = grid_barrier(bar, status);
    if (go3) {
        // weight bits of class m for this lane's channels: bit m of wsel[t]
        uint64_t wsel[TILES];
        bool c_ok[TILES];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            c_ok[t] = t * 64 + lane < C1;
            wsel[t] = 0;
        }
        for (int m = 0; m < M; ++m)
#pragma unroll
            for (int t = 0; t < TILES; ++t)
                if (t < mw)
                    wsel[t] |= ((w2[(int64_t)m * w2_stride + t] >> lane) & 1ull) << m;
        const float al = lane < M ? alpha[lane] : 0.0f;
        for (int64_t slot = gwave; slot < n; slot += nwaves) {
            const uint32_t row = (uint32_t)order[slot];
            int cnt[TILES];
            uint32_t deg;
            row_counts<TILES>(rowptr, col, row, h_bits, h_stride, (int)mw, lane, cnt, deg);
            int s[TILES];
#pragma unroll
            for (int t = 0; t < TILES; ++t)
                s[t] = c_ok[t] ? 2 * cnt[t] - (int)deg : 0; // pad channels carry nothing
            int res = 0;
            for (int m = 0; m < M; ++m) {
                int v = 0;
#pragma unroll
                for (int t = 0; t < TILES; ++t)
                    v += ((wsel[t] >> m) & 1ull) ? s[t] : -s[t];
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1)
                    v += __shfl_xor(v, d);
                if (lane == m)
                    res = v;
            }
            if (lane < M)
                logits[(int64_t)row * ldo + lane] = al * (float)res;
        }
    }
}

} // namespace

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
    const void *kernel = tiles == 1   ? (const void *)gcn2_fused_kernel<1>
                         : tiles == 2 ? (const void *)gcn2_fused_kernel<2>
                                      : (const void *)gcn2_fused_kernel<4>;
    // the whole grid must be resident at once: at most what the occupancy query allows
    int per_cu = 0;
    BG_HIP(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kFusedBlock, 0));
    BG_REQUIRE(ctx, per_cu >= 1, BITGNN_ERR_HIP, "bitgnn_gcn2_fused: kernel does not fit a CU");
    int64_t blocks = (int64_t)ctx->n_cus * (per_cu < 2 ? per_cu : 2);
    const int64_t useful = (n + kFusedWaves - 1) / kFusedWaves; // one row per wavefront
    if (blocks > useful)
        blocks = useful;
    const uint32_t base = ctx->bar_base;
    uint32_t *counter = ctx->queue + kFusedBarrierWord;
#define BG_FUSED(TV)                                                                              \
    gcn2_fused_kernel<TV><<<(unsigned)blocks, kFusedBlock, 0, s>>>(                               \
        adj->rowptr, adj->col, adj->order, n, x, K0, ldx, w1bits, C1, w1_stride, T_mm, T_agg,     \
        w2bits, M, w2_stride, alpha, tmp_bits, h_bits, h_stride, logits, ldo, counter, base,      \
        status)
    if (tiles == 1)
        BG_FUSED(1);
    else if (tiles == 2)
        BG_FUSED(2);
    else
        BG_FUSED(4);
#undef BG_FUSED
    BG_LAUNCH_CHECK(ctx, "gcn2_fused_kernel");
    // every workgroup arrives at every barrier, whatever happens: the device counter
    // advances by exactly this much per launch
    ctx->bar_base = base + (uint32_t)(kBarriers * blocks);
    return BITGNN_OK;
}
