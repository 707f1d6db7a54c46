// BIN: binarize and bit-pack (Section 2.2 sign rule, Section 2.3 on packing
// with a wave vote).
//
// gfx950 mapping: a wavefront takes 64 consecutive (row, word) chunks, 16 per row of 16
// lanes.  For one chunk each of the 16 lanes loads 4 consecutive elements (16 bytes for
// f32: a 256-byte run per chunk), compares them into a nibble, shifts the nibble to its
// place in the 64-bit word, and four DPP OR steps (quad permutes, half-row and row mirror)
// leave the word in all 16 lanes; lane t of the wavefront keeps the word of chunk t and
// after 16 turns the wavefront stores 64 words (512 bytes) at once.  Bits are LSB-first, so
// no bit reversal is needed.  The kernel is bound by the HBM read of x.  (One element per
// lane and a wave vote per chunk - the paper's form - kept the VALU 97 % busy at half the
// HBM rate: ~20 instructions per 64 elements against ~10 per 256 here.)  Rows of fewer
// than 4 elements take the one-element-per-lane kernel.
#include "common.h"

namespace {

constexpr int kBlock = 256;
constexpr int kUnroll = 16;

template <typename T> __device__ __forceinline__ bool bin_pred(T v, float tau);
template <> __device__ __forceinline__ bool bin_pred<float>(float v, float tau) { return v >= tau; }
template <> __device__ __forceinline__ bool bin_pred<int8_t>(int8_t v, float) { return v >= 0; }

template <typename T, bool HAS_TAU>
__global__ __launch_bounds__(kBlock) void pack_rows_kernel(const T *__restrict__ x, int64_t n,
                                                           int32_t K, int64_t ldx,
                                                           const float *__restrict__ tau,
                                                           uint64_t *__restrict__ out,
                                                           int64_t out_stride, int32_t words)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    const int64_t total = n * (int64_t)words;
    const int64_t q0 = wave * 64; // first chunk of this wave
    if (q0 >= total)
        return;
    int64_t row = q0 / words;
    int32_t w = (int32_t)(q0 - row * words);

    uint64_t mine = 0;
    for (int t0 = 0; t0 < 64; t0 += kUnroll) {
        T v[kUnroll];
        float tv[kUnroll];
        bool ok[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int32_t k = w * 64 + lane;
            ok[u] = (q0 + t0 + u < total) && (k < K);
            // clamped, unconditional loads: all kUnroll of them are in flight together
            const int32_t kc = k < K ? k : K - 1;
            const int64_t rc = row < n ? row : n - 1;
            v[u] = x[rc * ldx + kc];
            tv[u] = HAS_TAU ? tau[kc] : 0.0f;
            if (++w == words) {
                w = 0;
                ++row;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t m = __ballot(ok[u] && bin_pred<T>(v[u], tv[u]));
            if (lane == t0 + u)
                mine = m;
        }
    }
    const int64_t q = q0 + lane;
    if (q < total) {
        const int64_t my_row = q / words;
        out[my_row * out_stride + (q - my_row * words)] = mine;
    }
}

// 4 elements per lane: see the head of the file.  K >= 4 (a lane's 16-byte load is moved back
// to end at the row's last element, and the nibble is shifted to match).
constexpr int kUnroll4 = 4;

__device__ __forceinline__ uint32_t or_row16(uint32_t v)
{
    // values become uniform over pairs, quads, half rows, rows of 16 lanes
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);  // quad [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);  // quad [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false); // half-row mirror
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false); // row mirror
    return v;
}

template <typename T, bool HAS_TAU>
__global__ __launch_bounds__(kBlock) void pack_rows4_kernel(const T *__restrict__ x, int64_t n,
                                                            int32_t K, int64_t ldx,
                                                            const float *__restrict__ tau,
                                                            uint64_t *__restrict__ out,
                                                            int64_t out_stride, int32_t words)
{
    const int lane = threadIdx.x & 63, sub = lane & 15, grp = lane >> 4;
    const int64_t wave = (int64_t)blockIdx.x * (kBlock / 64) +
                         __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t total = n * (int64_t)words;
    const int64_t q0 = wave * 64; // first chunk of this wavefront (wave-uniform)
    if (q0 >= total)
        return;
    // this row of 16 lanes walks the chunks q0 + 16 grp + (0 .. 15); its position is kept as
    // a row pointer and a word index that step along (a 64-bit multiply per load had made
    // the kernel VALU-bound; the one 64-bit division is wave-uniform)
    const int64_t rowb = q0 / words;
    const uint32_t offb = (uint32_t)(q0 - rowb * words) + 16u * (uint32_t)grp;
    const uint32_t drow = offb / (uint32_t)words;
    const int64_t row0 = rowb + drow;
    int32_t w = (int32_t)(offb - drow * (uint32_t)words);
    // rows left after the current one, clamped (a row of lanes steps over at most 16 rows);
    // negative = past the last row (the pointer then stays on the last row)
    const int64_t left0 = n - 1 - row0;
    int32_t rows_left = left0 > 64 ? 64 : (left0 < -64 ? -64 : (int32_t)left0);
    const T *rowp = x + (row0 < n ? row0 : n - 1) * ldx;
    uint32_t mine_lo = 0, mine_hi = 0;
    int32_t mine_w = 0, mine_drow = 0, stepped = 0; // where the kept chunk lies
    for (int t0 = 0; t0 < 16; t0 += kUnroll4) {
        T v[kUnroll4][4];
        float tv[kUnroll4][4];
        uint32_t shift[kUnroll4], okm[kUnroll4];
#pragma unroll
        for (int u = 0; u < kUnroll4; ++u) {
            const int32_t k = w * 64 + 4 * sub;
            // clamped, unconditional loads: all kUnroll4 of them are in flight together
            const int32_t kk = k < K - 4 ? k : K - 4;
            __builtin_memcpy(v[u], rowp + kk, 4 * sizeof(T));
            if (HAS_TAU)
                __builtin_memcpy(tv[u], tau + kk, 16);
            else
                tv[u][0] = tv[u][1] = tv[u][2] = tv[u][3] = 0.0f;
            shift[u] = (uint32_t)(k - kk) < 4u ? (uint32_t)(k - kk) : 4u;
            const int32_t left = K - k; // elements of this lane that exist
            okm[u] = (rows_left >= 0 && left > 0) ? (left >= 4 ? 0xFu : (1u << left) - 1u) : 0u;
            if (sub == t0 + u) {
                mine_w = w;
                mine_drow = stepped;
            }
            if (++w == words) {
                w = 0;
                if (rows_left > 0)
                    rowp += ldx;
                --rows_left;
                ++stepped;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll4; ++u) {
            uint32_t nib = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                nib |= bin_pred<T>(v[u][j], tv[u][j]) ? (1u << j) : 0u;
            nib = (nib >> shift[u]) & okm[u];
            const uint32_t placed = nib << (4 * (sub & 7));
            const uint32_t lo = or_row16(sub < 8 ? placed : 0u);
            const uint32_t hi = or_row16(sub < 8 ? 0u : placed);
            if (sub == t0 + u) {
                mine_lo = lo;
                mine_hi = hi;
            }
        }
    }
    // lane 16 grp + t holds chunk q0 + 16 grp + t
    if (q0 + lane < total)
        out[(row0 + mine_drow) * out_stride + mine_w] = ((uint64_t)mine_hi << 32) | mine_lo;
}

// Transposed weight packing: one thread per (output channel c, word).  Weights
// are small and packed once, off the inference path.
__global__ void pack_weights_kernel(const int8_t *__restrict__ w, int32_t K, int32_t M,
                                    int64_t ldw, uint64_t *__restrict__ out, int64_t out_stride,
                                    int32_t words)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)M * words)
        return;
    const int32_t c = (int32_t)(t / words);
    const int32_t wd = (int32_t)(t % words);
    uint64_t bits = 0;
    for (int b = 0; b < 64; ++b) {
        const int32_t k = wd * 64 + b;
        if (k < K && w[(int64_t)k * ldw + c] >= 0)
            bits |= 1ull << b;
    }
    out[(int64_t)c * out_stride + wd] = bits;
}

template <typename T>
int pack_common(bitgnn_ctx *ctx, void *stream, const T *x, int64_t n, int32_t K, int64_t ldx,
                const float *tau, uint64_t *out, int64_t out_stride, const char *name)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, n >= 0 && K >= 1, BITGNN_ERR_INVALID_ARG, "%s: n=%lld K=%d", name,
               (long long)n, K);
    const int32_t words = (K + 63) / 64;
    BG_REQUIRE(ctx, ldx >= K, BITGNN_ERR_INVALID_ARG, "%s: ldx=%lld < K=%d", name, (long long)ldx,
               K);
    BG_REQUIRE(ctx, out_stride >= words, BITGNN_ERR_INVALID_ARG,
               "%s: out_stride=%lld < ceil(K/64)=%d", name, (long long)out_stride, words);
    if (n == 0)
        return BITGNN_OK;
    BG_REQUIRE(ctx, x && out, BITGNN_ERR_INVALID_ARG, "%s: null pointer", name);
    BG_REQUIRE(ctx, bg_aligned(x, sizeof(T)) && bg_aligned(out, 8) && bg_aligned(tau, 4),
               BITGNN_ERR_ALIGNMENT, "%s: misaligned pointer", name);
    BG_REQUIRE(ctx, n * (int64_t)words < (1ll << 37), BITGNN_ERR_UNSUPPORTED,
               "%s: n*words too large for one launch", name);
    BG_NEED_DEVICE(ctx);
    const int64_t waves = (n * words + 63) / 64;
    const unsigned grid = (unsigned)((waves + kBlock / 64 - 1) / (kBlock / 64));
    hipStream_t s = (hipStream_t)stream;
    if (K >= 4) {
        if (tau)
            pack_rows4_kernel<T, true><<<grid, kBlock, 0, s>>>(x, n, K, ldx, tau, out, out_stride,
                                                               words);
        else
            pack_rows4_kernel<T, false><<<grid, kBlock, 0, s>>>(x, n, K, ldx, nullptr, out,
                                                                out_stride, words);
    } else if (tau) {
        pack_rows_kernel<T, true><<<grid, kBlock, 0, s>>>(x, n, K, ldx, tau, out, out_stride, words);
    } else {
        pack_rows_kernel<T, false><<<grid, kBlock, 0, s>>>(x, n, K, ldx, nullptr, out, out_stride,
                                                           words);
    }
    BG_LAUNCH_CHECK(ctx, name);
    return BITGNN_OK;
}

} // namespace

extern "C" int bitgnn_pack_f32(bitgnn_ctx *ctx, void *stream, const float *x, int64_t n, int32_t K,
                               int64_t ldx, const float *tau, uint64_t *out, int64_t out_stride)
{
    return pack_common<float>(ctx, stream, x, n, K, ldx, tau, out, out_stride, "bitgnn_pack_f32");
}

extern "C" int bitgnn_pack_i8(bitgnn_ctx *ctx, void *stream, const int8_t *x, int64_t n, int32_t K,
                              int64_t ldx, uint64_t *out, int64_t out_stride)
{
    return pack_common<int8_t>(ctx, stream, x, n, K, ldx, nullptr, out, out_stride,
                               "bitgnn_pack_i8");
}

extern "C" int bitgnn_pack_weights_i8(bitgnn_ctx *ctx, void *stream, const int8_t *w, int32_t K,
                                      int32_t M, int64_t ldw, uint64_t *out, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, K >= 1 && M >= 1, BITGNN_ERR_INVALID_ARG, "bitgnn_pack_weights_i8: K=%d M=%d",
               K, M);
    const int32_t words = (K + 63) / 64;
    BG_REQUIRE(ctx, ldw >= M && out_stride >= words, BITGNN_ERR_INVALID_ARG,
               "bitgnn_pack_weights_i8: ldw=%lld out_stride=%lld", (long long)ldw,
               (long long)out_stride);
    BG_REQUIRE(ctx, w && out, BITGNN_ERR_INVALID_ARG, "bitgnn_pack_weights_i8: null pointer");
    BG_REQUIRE(ctx, bg_aligned(out, 8), BITGNN_ERR_ALIGNMENT,
               "bitgnn_pack_weights_i8: misaligned out");
    BG_NEED_DEVICE(ctx);
    const int64_t total = (int64_t)M * words;
    const unsigned grid = (unsigned)((total + 255) / 256);
    pack_weights_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(w, K, M, ldw, out, out_stride,
                                                               words);
    BG_LAUNCH_CHECK(ctx, "bitgnn_pack_weights_i8");
    return BITGNN_OK;
}
