// ADD: the auxiliary element-wise merge of two activation tensors (Section 3.1.2: the
// self-connectivity of GraphSAGE is merged with ADD.BBF or ADD.FFF), with the operands in
// packed +-1 bits or in floats, and the result in floats or binarized again (BIN folded in,
// as the other low-level functions do).
//
// gfx950 mapping: a wavefront takes one (row, 64-channel) tile: one coalesced 256-byte
// access per float operand, one broadcast 8-byte word per bit operand; the thresholded
// result of 64 channels is the wave-wide compare mask, already the packed word.  Bound by
// the HBM stream of the float operands / result.
#include "common.h"

namespace {

constexpr int kAddBlock = 256;

template <bool A_BITS, bool B_BITS, bool BITS_OUT>
__global__ __launch_bounds__(kAddBlock) void add_kernel(const void *__restrict__ a, int64_t lda,
                                                        const void *__restrict__ b, int64_t ldb,
                                                        int64_t n, int32_t C, int32_t tiles,
                                                        const float *__restrict__ tau,
                                                        void *__restrict__ out, int64_t ldo)
{
    const int lane = threadIdx.x & 63;
    const int64_t nwaves = (int64_t)gridDim.x * (kAddBlock / 64);
    const int64_t total = n * (int64_t)tiles;
    for (int64_t q = (int64_t)blockIdx.x * (kAddBlock / 64) + (threadIdx.x >> 6); q < total;
         q += nwaves) {
        const int64_t row = q / tiles;
        const int32_t t = (int32_t)(q - row * tiles);
        const int32_t c = t * 64 + lane;
        const bool ok = c < C;
        float va, vb;
        if (A_BITS)
            va = ((((const uint64_t *)a)[row * lda + t] >> lane) & 1ull) ? 1.0f : -1.0f;
        else
            va = ok ? ((const float *)a)[row * lda + c] : 0.0f;
        if (B_BITS)
            vb = ((((const uint64_t *)b)[row * ldb + t] >> lane) & 1ull) ? 1.0f : -1.0f;
        else
            vb = ok ? ((const float *)b)[row * ldb + c] : 0.0f;
        const float y = va + vb;
        if (BITS_OUT) {
            const uint64_t word = __ballot(ok && y >= tau[ok ? c : 0]);
            if (lane == 0)
                ((uint64_t *)out)[row * ldo + t] = word;
        } else if (ok) {
            ((float *)out)[row * ldo + c] = y;
        }
    }
}

} // namespace

extern "C" int bitgnn_add(bitgnn_ctx *ctx, void *stream, const void *a, int a_is_bits,
                          int64_t lda, const void *b, int b_is_bits, int64_t ldb, int64_t n,
                          int32_t C, int epilogue, const float *tau, void *out, int64_t ldo)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, n >= 0 && C >= 1, BITGNN_ERR_INVALID_ARG, "bitgnn_add: n=%lld C=%d",
               (long long)n, C);
    const int64_t words = ((int64_t)C + 63) / 64;
    const bool bits_out = epilogue == BITGNN_EPI_THRESH_BITS;
    BG_REQUIRE(ctx, bits_out || epilogue == BITGNN_EPI_SCALE_F32, BITGNN_ERR_INVALID_ARG,
               "bitgnn_add: epilogue %d (THRESH_BITS or SCALE_F32)", epilogue);
    BG_REQUIRE(ctx, !bits_out || tau, BITGNN_ERR_INVALID_ARG,
               "bitgnn_add: THRESH_BITS needs tau");
    BG_REQUIRE(ctx, lda >= (a_is_bits ? words : C) && ldb >= (b_is_bits ? words : C) &&
                        ldo >= (bits_out ? words : C),
               BITGNN_ERR_INVALID_ARG, "bitgnn_add: lda=%lld ldb=%lld ldo=%lld too small for C=%d",
               (long long)lda, (long long)ldb, (long long)ldo, C);
    if (n == 0)
        return BITGNN_OK;
    BG_REQUIRE(ctx, a && b && out, BITGNN_ERR_INVALID_ARG, "bitgnn_add: null pointer");
    BG_REQUIRE(ctx, bg_aligned(a, a_is_bits ? 8 : 4) && bg_aligned(b, b_is_bits ? 8 : 4) &&
                        bg_aligned(out, bits_out ? 8 : 4) && bg_aligned(tau, 4),
               BITGNN_ERR_ALIGNMENT, "bitgnn_add: misaligned pointer");
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    const int64_t total = n * words;
    int64_t blocks = (total + kAddBlock / 64 - 1) / (kAddBlock / 64);
    const int64_t cap = (int64_t)ctx->n_cus * 32;
    if (blocks > cap)
        blocks = cap;
#define BG_ADD(AB, BB, OB)                                                                        \
    add_kernel<AB, BB, OB><<<(unsigned)blocks, kAddBlock, 0, s>>>(a, lda, b, ldb, n, C,           \
                                                                  (int32_t)words, tau, out, ldo)
    const int sel = (a_is_bits ? 4 : 0) | (b_is_bits ? 2 : 0) | (bits_out ? 1 : 0);
    switch (sel) {
    case 0: BG_ADD(false, false, false); break;
    case 1: BG_ADD(false, false, true); break;
    case 2: BG_ADD(false, true, false); break;
    case 3: BG_ADD(false, true, true); break;
    case 4: BG_ADD(true, false, false); break;
    case 5: BG_ADD(true, false, true); break;
    case 6: BG_ADD(true, true, false); break;
    default: BG_ADD(true, true, true); break;
    }
#undef BG_ADD
    BG_LAUNCH_CHECK(ctx, "add_kernel");
    return BITGNN_OK;
}
