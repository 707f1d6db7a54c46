// BMM: XNOR-popcount product of bit-packed +-1 activations and weights
// (Section 2.2: c = n - 2 popc(a xor b)), with the re-binarization or the scale
// folded into the epilogue (Section 3.1.2, BMM variants).
//
// gfx950 mapping (plain VALU; CDNA4 has no 1-bit matrix instruction):
//  - a lane owns one output channel c; its weight words sit in VGPRs
//  - a wavefront walks 32 node rows; the activation words of a row are the
//    same for all 64 lanes, so they are fetched with wave-uniform (scalar)
//    loads and used as scalar operands of v_xor
//  - v_bcnt_u32_b32 accumulates the popcount for free (third operand)
//  - the thresholded output bit of 64 channels is the wave-wide compare mask,
//    i.e. already the packed output word: no shuffles or votes beyond it
// The kernel is bound by VALU issue (2 lane-ops per 32 bit-MACs), not by HBM.
#include "common.h"

namespace {

constexpr int kWaves = 4;  // wavefronts per workgroup
constexpr int kRows = 32;  // node rows per wavefront
constexpr int kChunk = 8;  // 32-bit words of the K axis held per step

template <int EPI>
__global__ __launch_bounds__(kWaves * 64) void bgemm_kernel(
    const uint32_t *__restrict__ x32, int64_t n, int64_t x_stride32, int32_t K, int32_t kw32,
    const uint32_t *__restrict__ w32, int32_t M, int64_t w_stride32,
    const int32_t *__restrict__ T, const float *__restrict__ alpha, void *__restrict__ out,
    int64_t out_stride)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row0 = ((int64_t)blockIdx.x * kWaves + wave) * kRows;
    if (row0 >= n)
        return;
    const int ct = blockIdx.y;
    const int c = ct * 64 + lane;
    const bool c_ok = c < M;
    const uint32_t *wrow = w32 + (int64_t)(c_ok ? c : 0) * w_stride32;

    int acc[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r)
        acc[r] = 0;

    for (int k0 = 0; k0 < kw32; k0 += kChunk) {
        uint32_t wv[kChunk];
        if (k0 + kChunk <= kw32) {
#pragma unroll
            for (int j = 0; j < kChunk; ++j)
                wv[j] = wrow[k0 + j];
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                const int64_t row = (row0 + r < n) ? row0 + r : n - 1; // wave-uniform
                const uint32_t *xr = x32 + row * x_stride32 + k0;
#pragma unroll
                for (int j = 0; j < kChunk; ++j)
                    acc[r] += __popc(xr[j] ^ wv[j]);
            }
        } else {
            const int rem = kw32 - k0; // 1..kChunk-1, wave-uniform
#pragma unroll
            for (int j = 0; j < kChunk; ++j)
                wv[j] = (j < rem) ? wrow[k0 + j] : 0u;
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                const int64_t row = (row0 + r < n) ? row0 + r : n - 1;
                const uint32_t *xr = x32 + row * x_stride32 + k0;
#pragma unroll
                for (int j = 0; j < kChunk; ++j)
                    if (j < rem)
                        acc[r] += __popc(xr[j] ^ wv[j]);
            }
        }
    }

    if (EPI == BITGNN_EPI_THRESH_BITS) {
        const int32_t tc = c_ok ? T[c] : 0;
        uint64_t mine = 0;
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int32_t z = K - 2 * acc[r];
            const uint64_t m = __ballot(c_ok && z >= tc);
            if (lane == r)
                mine = m;
        }
        if (lane < kRows && row0 + lane < n)
            ((uint64_t *)out)[(row0 + lane) * out_stride + ct] = mine;
    } else if (EPI == BITGNN_EPI_RAW_I32) {
#pragma unroll
        for (int r = 0; r < kRows; ++r)
            if (c_ok && row0 + r < n)
                ((int32_t *)out)[(row0 + r) * out_stride + c] = K - 2 * acc[r];
    } else {
        const float a = c_ok ? alpha[c] : 0.0f;
#pragma unroll
        for (int r = 0; r < kRows; ++r)
            if (c_ok && row0 + r < n)
                ((float *)out)[(row0 + r) * out_stride + c] = a * (float)(K - 2 * acc[r]);
    }
}


// BMM with full-precision activations (the paper's BMM.FBB / BMM.FBF, Section 3.1.2:
// BIN folded into the product).  The binarization costs no pass of its own: 64 lanes
// load 64 consecutive floats of a node row (one coalesced 256-byte access) and the
// wave-wide compare mask IS the 64-bit activation word, already in scalar registers,
// where the XOR with the lane's weight words wants it.  The packed activations are
// never written to memory.  A wavefront owns TILES x 64 output channels, so the float
// matrix is streamed from HBM exactly once when M <= 64 * TILES; the kernel is then
// bound by that stream.  To keep the stream sequential for the memory system, a
// wavefront holds the weight words of a whole K chunk in registers and walks its 16
// rows one after the other: its requests cover one contiguous span of the matrix
// (16 rows back to back when ldx == K), two rows in flight at a time.
constexpr int kRowsF = 16;

template <int TILES>
struct f32_chunk {
    // 32-bit weight words per K chunk held in registers (two per vote of 64 floats)
    // (four tiles: 16 words where the last chunk of a row would be mostly full, else 8)
    static constexpr int words = TILES <= 2 ? 20 : 8;
    static constexpr int words_long = TILES <= 2 ? 20 : 16;
};

template <int VOTES, bool HAS_TAU>
__device__ __forceinline__ void f32_load_row(const float *__restrict__ xrow,
                                             const int32_t (&kc)[VOTES], float (&v)[VOTES])
{
#pragma unroll
    for (int b = 0; b < VOTES; ++b)
        v[b] = xrow[kc[b]];
}

template <int VOTES, int TILES, bool HAS_TAU>
__device__ __forceinline__ void f32_consume_row(const float (&v)[VOTES], const float (&tv)[VOTES],
                                                const uint64_t (&okmask)[VOTES],
                                                const uint32_t (&wv)[TILES][2 * VOTES],
                                                int (&acc)[TILES])
{
#pragma unroll
    for (int b = 0; b < VOTES; ++b) {
        // beyond K the vote is 0 and so are the weight words: nothing is added
        const uint64_t m = __ballot(v[b] >= (HAS_TAU ? tv[b] : 0.0f)) & okmask[b];
        const uint32_t lo = (uint32_t)m, hi = (uint32_t)(m >> 32);
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            acc[t] += __popc(lo ^ wv[t][2 * b]) + __popc(hi ^ wv[t][2 * b + 1]);
    }
}

// Epilogue of one finished row: the thresholded bits of row r are parked in lane r
// (written after the last row), integers and logits are stored at once.
template <int EPI, int TILES>
__device__ __forceinline__ void f32_finish_row(int r, int64_t row, bool row_ok, int lane,
                                               const int (&acc)[TILES], int32_t K, int ct0,
                                               const bool (&c_ok)[TILES],
                                               const int32_t (&tc)[TILES],
                                               const float (&al)[TILES], uint64_t (&mine)[TILES],
                                               void *__restrict__ out, int64_t out_stride)
{
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int c = (ct0 + t) * 64 + lane;
        const int32_t z = K - 2 * acc[t];
        if (EPI == BITGNN_EPI_THRESH_BITS) {
            const uint64_t m = __ballot(c_ok[t] && z >= tc[t]);
            if (lane == r)
                mine[t] = m;
        } else if (EPI == BITGNN_EPI_RAW_I32) {
            if (c_ok[t] && row_ok)
                ((int32_t *)out)[row * out_stride + c] = z;
        } else {
            if (c_ok[t] && row_ok)
                ((float *)out)[row * out_stride + c] = al[t] * (float)z;
        }
    }
}

// SINGLE: all of K fits one register chunk, so a row is finished as soon as it has been
// read and no per-row accumulators are kept.
template <int EPI, int TILES, bool HAS_TAU, bool SINGLE, int kWords = f32_chunk<TILES>::words>
__global__ __launch_bounds__(kWaves * 64) void bgemm_f32_kernel(
    const float *__restrict__ x, int64_t n, int32_t K, int64_t ldx, const float *__restrict__ tau,
    int32_t kw32, const uint32_t *__restrict__ w32, int32_t M, int64_t w_stride32,
    const int32_t *__restrict__ T, const float *__restrict__ alpha, void *__restrict__ out,
    int64_t out_stride)
{
    constexpr int kVotes = kWords / 2;
    constexpr int kAccRows = SINGLE ? 2 : kRowsF;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row0 = ((int64_t)blockIdx.x * kWaves + wave) * kRowsF;
    if (row0 >= n)
        return;
    const int ct0 = blockIdx.y * TILES;
    const uint32_t *wrow[TILES];
    bool c_ok[TILES];
    int32_t tc[TILES];
    float al[TILES];
    uint64_t mine[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int c = (ct0 + t) * 64 + lane;
        c_ok[t] = c < M;
        wrow[t] = w32 + (int64_t)(c_ok[t] ? c : 0) * w_stride32;
        tc[t] = (EPI == BITGNN_EPI_THRESH_BITS && c_ok[t]) ? T[c] : 0;
        al[t] = (EPI == BITGNN_EPI_SCALE_F32 && c_ok[t]) ? alpha[c] : 0.0f;
        mine[t] = 0;
    }
    int acc[kAccRows][TILES];
#pragma unroll
    for (int r = 0; r < kAccRows; ++r)
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            acc[r][t] = 0;
    const int64_t last = n - 1;

    for (int k0 = 0; k0 < kw32; k0 += kWords) {
        // weight words of the chunk (the bound is wave-uniform: scalar branches, no waits)
        uint32_t wv[TILES][kWords];
#pragma unroll
        for (int t = 0; t < TILES; ++t)
#pragma unroll
            for (int j = 0; j < kWords; ++j)
                wv[t][j] = (k0 + j < kw32) ? wrow[t][k0 + j] : 0u;
        int32_t kc[kVotes];
        float tv[kVotes];
        uint64_t okmask[kVotes];
#pragma unroll
        for (int b = 0; b < kVotes; ++b) {
            const int32_t k = k0 * 32 + b * 64 + lane;
            okmask[b] = __ballot(k < K);
            kc[b] = k < K ? k : K - 1; // clamped: no load is conditional
            tv[b] = HAS_TAU ? tau[kc[b]] : 0.0f;
        }
        // rows one after the other, the next row requested before the current is consumed
        float va[kVotes], vb[kVotes];
        f32_load_row<kVotes, HAS_TAU>(x + (row0 < last ? row0 : last) * ldx, kc, va);
#pragma unroll
        for (int r = 0; r < kRowsF; r += 2) {
            const int ra = SINGLE ? 0 : r, rb = SINGLE ? 1 : r + 1;
            const int64_t r1 = row0 + r + 1 < last ? row0 + r + 1 : last; // wave-uniform
            f32_load_row<kVotes, HAS_TAU>(x + r1 * ldx, kc, vb);
            f32_consume_row<kVotes, TILES, HAS_TAU>(va, tv, okmask, wv, acc[ra]);
            if (r + 2 < kRowsF) {
                const int64_t r2 = row0 + r + 2 < last ? row0 + r + 2 : last;
                f32_load_row<kVotes, HAS_TAU>(x + r2 * ldx, kc, va);
            }
            f32_consume_row<kVotes, TILES, HAS_TAU>(vb, tv, okmask, wv, acc[rb]);
            if (SINGLE) {
                f32_finish_row<EPI, TILES>(r, row0 + r, row0 + r < n, lane, acc[0], K, ct0, c_ok,
                                           tc, al, mine, out, out_stride);
                f32_finish_row<EPI, TILES>(r + 1, row0 + r + 1, row0 + r + 1 < n, lane, acc[1], K,
                                           ct0, c_ok, tc, al, mine, out, out_stride);
#pragma unroll
                for (int t = 0; t < TILES; ++t)
                    acc[0][t] = acc[1][t] = 0;
            }
        }
    }
    if (!SINGLE) {
#pragma unroll
        for (int r = 0; r < kRowsF; ++r)
            f32_finish_row<EPI, TILES>(r, row0 + r, row0 + r < n, lane, acc[r], K, ct0, c_ok, tc,
                                       al, mine, out, out_stride);
    }
    if (EPI == BITGNN_EPI_THRESH_BITS) {
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            if ((ct0 + t) * 64 < M && lane < kRowsF && row0 + lane < n)
                ((uint64_t *)out)[(row0 + lane) * out_stride + ct0 + t] = mine[t];
    }
}

template <int EPI, int TILES>
void launch_bgemm_f32(hipStream_t s, dim3 grid, const float *x, int64_t n, int32_t K, int64_t ldx,
                      const float *tau, int32_t kw32, const uint32_t *w32, int32_t M,
                      int64_t w_stride32, const int32_t *T, const float *alpha, void *out,
                      int64_t out_stride)
{
    // chunk of the K axis: the long one if its last step over a row wastes under 8 words
    constexpr int kLong = f32_chunk<TILES>::words_long, kShort = f32_chunk<TILES>::words;
    const bool use_long = kLong != kShort && ((kw32 + kLong - 1) / kLong) * kLong - kw32 < 8;
#define BG_F32(TAU, SINGLE)                                                                       \
    do {                                                                                          \
        if (use_long)                                                                             \
            bgemm_f32_kernel<EPI, TILES, TAU, SINGLE, kLong><<<grid, kWaves * 64, 0, s>>>(        \
                x, n, K, ldx, tau, kw32, w32, M, w_stride32, T, alpha, out, out_stride);          \
        else                                                                                      \
            bgemm_f32_kernel<EPI, TILES, TAU, SINGLE, kShort><<<grid, kWaves * 64, 0, s>>>(       \
                x, n, K, ldx, tau, kw32, w32, M, w_stride32, T, alpha, out, out_stride);          \
    } while (0)
    const bool single = kw32 <= (use_long ? kLong : kShort);
    if (tau) {
        if (single)
            BG_F32(true, true);
        else
            BG_F32(true, false);
    } else {
        if (single)
            BG_F32(false, true);
        else
            BG_F32(false, false);
    }
#undef BG_F32
}

template <int EPI>
void launch_bgemm_f32_tiles(hipStream_t s, int64_t n, int32_t M, const float *x, int32_t K,
                            int64_t ldx, const float *tau, int32_t kw32, const uint32_t *w32,
                            int64_t w_stride32, const int32_t *T, const float *alpha, void *out,
                            int64_t out_stride)
{
    const int mt = (M + 63) / 64;
    const unsigned gx = (unsigned)((n + kWaves * kRowsF - 1) / (kWaves * kRowsF));
    if (mt == 1)
        launch_bgemm_f32<EPI, 1>(s, dim3(gx, 1), x, n, K, ldx, tau, kw32, w32, M, w_stride32, T,
                                 alpha, out, out_stride);
    else if (mt == 2)
        launch_bgemm_f32<EPI, 2>(s, dim3(gx, 1), x, n, K, ldx, tau, kw32, w32, M, w_stride32, T,
                                 alpha, out, out_stride);
    else
        launch_bgemm_f32<EPI, 4>(s, dim3(gx, (unsigned)((mt + 3) / 4)), x, n, K, ldx, tau, kw32,
                                 w32, M, w_stride32, T, alpha, out, out_stride);
}

} // namespace

int bg_check_bgemm(bitgnn_ctx *ctx, const uint64_t *xbits, int64_t n, int64_t x_stride, int32_t K,
                   int32_t kwords, const uint64_t *wbits, int32_t M, int64_t w_stride,
                   int epilogue, const int32_t *T, const float *alpha, const void *out,
                   int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, n >= 0 && K >= 1 && kwords >= 1 && M >= 1, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm: n=%lld K=%d kwords=%d M=%d", (long long)n, K, kwords, M);
    BG_REQUIRE(ctx, (int64_t)K <= (int64_t)kwords * 64, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm: K=%d logical bits do not fit kwords=%d words", K, kwords);
    BG_REQUIRE(ctx, x_stride >= kwords && w_stride >= kwords, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm: x_stride=%lld w_stride=%lld < kwords=%d", (long long)x_stride,
               (long long)w_stride, kwords);
    BG_REQUIRE(ctx,
               epilogue == BITGNN_EPI_RAW_I32 || epilogue == BITGNN_EPI_THRESH_BITS ||
                   epilogue == BITGNN_EPI_SCALE_F32,
               BITGNN_ERR_INVALID_ARG, "bitgnn_bgemm: epilogue=%d", epilogue);
    const int64_t need = epilogue == BITGNN_EPI_THRESH_BITS ? (M + 63) / 64 : M;
    BG_REQUIRE(ctx, out_stride >= need, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm: out_stride=%lld < %lld", (long long)out_stride, (long long)need);
    BG_REQUIRE(ctx, wbits && (n == 0 || (xbits && out)), BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm: null pointer");
    BG_REQUIRE(ctx, epilogue != BITGNN_EPI_THRESH_BITS || T, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm: THRESH_BITS needs T");
    BG_REQUIRE(ctx, epilogue != BITGNN_EPI_SCALE_F32 || alpha, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm: SCALE_F32 needs alpha");
    BG_REQUIRE(ctx,
               bg_aligned(xbits, 8) && bg_aligned(wbits, 8) && bg_aligned(T, 4) &&
                   bg_aligned(alpha, 4) &&
                   bg_aligned(out, epilogue == BITGNN_EPI_THRESH_BITS ? 8 : 4),
               BITGNN_ERR_ALIGNMENT, "bitgnn_bgemm: misaligned pointer");
    return BITGNN_OK;
}

int bg_launch_bgemm(bitgnn_ctx *ctx, hipStream_t s, const uint64_t *xbits, int64_t n,
                    int64_t x_stride, int32_t K, int32_t kwords, const uint64_t *wbits, int32_t M,
                    int64_t w_stride, int epilogue, const int32_t *T, const float *alpha,
                    void *out, int64_t out_stride)
{
    if (n == 0)
        return BITGNN_OK;
    if (bg_bgemm_mfma_applies(ctx, n, kwords, M))
        return bg_launch_bgemm_mfma(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                                    epilogue, T, alpha, out, out_stride);
    const int64_t gx = (n + kWaves * kRows - 1) / (kWaves * kRows);
    BG_REQUIRE(ctx, gx < (1ll << 31), BITGNN_ERR_UNSUPPORTED, "bitgnn_bgemm: n too large");
    dim3 grid((unsigned)gx, (unsigned)((M + 63) / 64));
    dim3 block(kWaves * 64);
    const uint32_t *x32 = (const uint32_t *)xbits;
    const uint32_t *w32 = (const uint32_t *)wbits;
    const int32_t kw32 = kwords * 2;
    switch (epilogue) {
    case BITGNN_EPI_THRESH_BITS:
        bgemm_kernel<BITGNN_EPI_THRESH_BITS><<<grid, block, 0, s>>>(
            x32, n, x_stride * 2, K, kw32, w32, M, w_stride * 2, T, alpha, out, out_stride);
        break;
    case BITGNN_EPI_RAW_I32:
        bgemm_kernel<BITGNN_EPI_RAW_I32><<<grid, block, 0, s>>>(
            x32, n, x_stride * 2, K, kw32, w32, M, w_stride * 2, T, alpha, out, out_stride);
        break;
    default:
        bgemm_kernel<BITGNN_EPI_SCALE_F32><<<grid, block, 0, s>>>(
            x32, n, x_stride * 2, K, kw32, w32, M, w_stride * 2, T, alpha, out, out_stride);
        break;
    }
    BG_LAUNCH_CHECK(ctx, "bitgnn_bgemm");
    return BITGNN_OK;
}

extern "C" int bitgnn_bgemm(bitgnn_ctx *ctx, void *stream, const uint64_t *xbits, int64_t n,
                            int64_t x_stride, int32_t K, int32_t kwords, const uint64_t *wbits,
                            int32_t M, int64_t w_stride, int epilogue, const int32_t *T,
                            const float *alpha, void *out, int64_t out_stride)
{
    int rc = bg_check_bgemm(ctx, xbits, n, x_stride, K, kwords, wbits, M, w_stride, epilogue, T,
                            alpha, out, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    return bg_launch_bgemm(ctx, (hipStream_t)stream, xbits, n, x_stride, K, kwords, wbits, M,
                           w_stride, epilogue, T, alpha, out, out_stride);
}

int bg_check_bgemm_f32(bitgnn_ctx *ctx, const float *x, int64_t n, int32_t K, int64_t ldx,
                       const float *tau, const uint64_t *wbits, int32_t M, int64_t w_stride,
                       int epilogue, const int32_t *T, const float *alpha, const void *out,
                       int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, n >= 0 && K >= 1 && M >= 1, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm_f32: n=%lld K=%d M=%d", (long long)n, K, M);
    const int64_t kwords = ((int64_t)K + 63) / 64;
    BG_REQUIRE(ctx, ldx >= K && w_stride >= kwords, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm_f32: ldx=%lld w_stride=%lld", (long long)ldx, (long long)w_stride);
    BG_REQUIRE(ctx,
               epilogue == BITGNN_EPI_RAW_I32 || epilogue == BITGNN_EPI_THRESH_BITS ||
                   epilogue == BITGNN_EPI_SCALE_F32,
               BITGNN_ERR_INVALID_ARG, "bitgnn_bgemm_f32: epilogue=%d", epilogue);
    const int64_t need = epilogue == BITGNN_EPI_THRESH_BITS ? (M + 63) / 64 : M;
    BG_REQUIRE(ctx, out_stride >= need, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm_f32: out_stride=%lld < %lld", (long long)out_stride, (long long)need);
    BG_REQUIRE(ctx, wbits && (n == 0 || (x && out)), BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm_f32: null pointer");
    BG_REQUIRE(ctx, epilogue != BITGNN_EPI_THRESH_BITS || T, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm_f32: THRESH_BITS needs T");
    BG_REQUIRE(ctx, epilogue != BITGNN_EPI_SCALE_F32 || alpha, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bgemm_f32: SCALE_F32 needs alpha");
    BG_REQUIRE(ctx,
               bg_aligned(x, 4) && bg_aligned(tau, 4) && bg_aligned(wbits, 8) && bg_aligned(T, 4) &&
                   bg_aligned(alpha, 4) &&
                   bg_aligned(out, epilogue == BITGNN_EPI_THRESH_BITS ? 8 : 4),
               BITGNN_ERR_ALIGNMENT, "bitgnn_bgemm_f32: misaligned pointer");
    return BITGNN_OK;
}

int bg_launch_bgemm_f32(bitgnn_ctx *ctx, hipStream_t s, const float *x, int64_t n, int32_t K,
                        int64_t ldx, const float *tau, const uint64_t *wbits, int32_t M,
                        int64_t w_stride, int epilogue, const int32_t *T, const float *alpha,
                        void *out, int64_t out_stride)
{
    if (n == 0)
        return BITGNN_OK;
    BG_REQUIRE(ctx, (n + kWaves * kRowsF - 1) / (kWaves * kRowsF) < (1ll << 31),
               BITGNN_ERR_UNSUPPORTED, "bitgnn_bgemm_f32: n too large");
    const int32_t kw32 = (int32_t)(((int64_t)K + 63) / 64) * 2;
    const uint32_t *w32 = (const uint32_t *)wbits;
    switch (epilogue) {
    case BITGNN_EPI_THRESH_BITS:
        launch_bgemm_f32_tiles<BITGNN_EPI_THRESH_BITS>(s, n, M, x, K, ldx, tau, kw32, w32,
                                                       w_stride * 2, T, alpha, out, out_stride);
        break;
    case BITGNN_EPI_RAW_I32:
        launch_bgemm_f32_tiles<BITGNN_EPI_RAW_I32>(s, n, M, x, K, ldx, tau, kw32, w32,
                                                   w_stride * 2, T, alpha, out, out_stride);
        break;
    default:
        launch_bgemm_f32_tiles<BITGNN_EPI_SCALE_F32>(s, n, M, x, K, ldx, tau, kw32, w32,
                                                     w_stride * 2, T, alpha, out, out_stride);
        break;
    }
    BG_LAUNCH_CHECK(ctx, "bitgnn_bgemm_f32");
    return BITGNN_OK;
}

extern "C" int bitgnn_bgemm_f32(bitgnn_ctx *ctx, void *stream, const float *x, int64_t n, int32_t K,
                                int64_t ldx, const float *tau, const uint64_t *wbits, int32_t M,
                                int64_t w_stride, int epilogue, const int32_t *T,
                                const float *alpha, void *out, int64_t out_stride)
{
    int rc = bg_check_bgemm_f32(ctx, x, n, K, ldx, tau, wbits, M, w_stride, epilogue, T, alpha,
                                out, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    return bg_launch_bgemm_f32(ctx, (hipStream_t)stream, x, n, K, ldx, tau, wbits, M, w_stride,
                               epilogue, T, alpha, out, out_stride);
}
