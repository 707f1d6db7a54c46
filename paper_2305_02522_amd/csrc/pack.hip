// BIN: binarize and bit-pack (Section 2.2 sign rule, Section 2.3 on packing
// with a wave vote).
//
// gfx950 mapping: a wavefront takes 64 consecutive (row, word) chunks.  For one
// chunk the 64 lanes load the 64 elements of that word (one coalesced 256-byte
// access for f32), and the wave-wide compare mask IS the packed 64-bit word, in
// LSB-first order, so no bit reversal and no shuffles are needed.  Lane t keeps
// the mask of chunk t; after 64 chunks the wave stores 64 words.  The kernel
// is bound by the HBM read of x.
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
    if (tau)
        pack_rows_kernel<T, true><<<grid, kBlock, 0, s>>>(x, n, K, ldx, tau, out, out_stride, words);
    else
        pack_rows_kernel<T, false><<<grid, kBlock, 0, s>>>(x, n, K, ldx, nullptr, out, out_stride,
                                                           words);
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
