// BSpMM: 0/1 adjacency times bit-packed +-1 activations with integer
// accumulation and a fused threshold / re-pack epilogue (Section 3.2.2,
// trinary dot product, method 3: S = 2*cnt - deg; Algorithm 1's final
// "c >= 0" test with the BatchNorm threshold T_c in place of 0).
//
// gfx950 mapping.  The paper transposes the gathered activation words with
// wave votes so that a popcount can run along the neighbour axis; on CDNA a
// vote lands in scalar registers and would serialize on the one scalar unit
// of a CU.  Instead the count is kept BIT-SLICED: a lane owns one 32-bit
// activation word (32 channels) of one node and adds the gathered neighbour
// words into "vertical" counters whose plane p holds bit p of all 32 channel
// counts.  A carry-save adder on whole words (xor3 + majority, 2 VALU ops)
// adds three words at once, so a neighbour costs ~2.2 VALU ops per 32
// channels, and no cross-lane traffic at all.  Neighbours are consumed 16 at
// a time (Harley-Seal tree: planes 1,2,4,8 exact, one carry of weight 16);
// the carries of weight >= 16 climb a binary-counter cascade whose control
// flow depends only on the block index, so it is wave-uniform.
//
// Threshold without unpacking: bit = (2 cnt - deg >= T_c)  <=>
// cnt - t >= m with deg = 2m + e and t = floor((T_c + e + 1) / 2).  The
// counters start at BIAS - t (a per-channel constant, bit-sliced once per call
// into a small table for both parities e), so at the end one bit-sliced
// comparison against the per-node constant BIAS + m yields the 32 output bits
// of the lane: already packed.
//
// Rows are visited in decreasing-degree order (from the builder), so the
// lanes of a wavefront have similar trip counts.
#include "common.h"

namespace {

constexpr int kBlock = 256;
constexpr int kGroup = 16; // neighbours per counter block

// (acc, b, c) -> acc = sum bit, carry = majority
__device__ __forceinline__ void csa(uint32_t &acc, uint32_t b, uint32_t c, uint32_t &carry)
{
    const uint32_t u = acc ^ b;
    carry = (acc & b) | (u & c);
    acc = u ^ c;
}

// Seeds of the vertical counters: table[(e*P + p)*W32 + w] bit c' = bit p of
// (BIAS - t(e, c)), c = 32 w + c', BIAS = 2^(P-1), t clamped to +-2^(P-2).
__global__ void bspmm_seed_kernel(const int32_t *__restrict__ T, int32_t C, int32_t W32, int P,
                                  uint32_t *__restrict__ table)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= 2 * P * W32)
        return;
    const int w = idx % W32;
    const int p = (idx / W32) % P;
    const int e = idx / (W32 * P);
    const int64_t lim = 1ll << (P - 2);
    uint32_t word = 0;
    for (int b = 0; b < 32; ++b) {
        const int c = 32 * w + b;
        if (c >= C)
            break;
        int64_t t = ((int64_t)T[c] + e + 1) >> 1; // floor
        t = t > lim ? lim : (t < -lim ? -lim : t);
        const uint64_t off = (uint64_t)((1ll << (P - 1)) - t);
        word |= (uint32_t)((off >> p) & 1u) << b;
    }
    table[idx] = word;
}

template <int P, int EPI>
__global__ __launch_bounds__(kBlock) void bspmm_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, uint32_t N, const uint32_t *__restrict__ h32,
    int64_t h_stride32, int32_t C, int32_t W32, const uint32_t *__restrict__ seeds,
    void *__restrict__ out, int64_t out_stride)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t slot = t / (uint32_t)W32;
    const int w = (int)(t - slot * (uint32_t)W32);
    const bool active = slot < N;
    const uint32_t row = active ? (uint32_t)order[slot] : 0u;
    uint32_t e = active ? rowptr[row] : 0u;
    const uint32_t end = active ? rowptr[row + 1] : 0u;
    const uint32_t deg = end - e;

    uint32_t acc[P], pend[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        acc[p] = (EPI == BITGNN_EPI_THRESH_BITS) ? seeds[((deg & 1u) * P + p) * W32 + w] : 0u;
        pend[p] = 0u;
    }

    const uint32_t *hw = h32 + w;
    uint32_t blk = 0; // blocks of 16 neighbours consumed so far (wave-uniform)
    while (__ballot(e < end) != 0ull) {
        uint32_t x[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const bool ok = e + u < end;
            const int32_t j = ok ? col[e + u] : 0;
            x[u] = ok ? hw[(int64_t)j * h_stride32] : 0u;
        }
        e = (end - e > (uint32_t)kGroup) ? e + kGroup : end;

        // 16 words -> planes 0..3 plus one carry of weight 16
        uint32_t a2, b2, a4, b4, a8, b8, c16;
        csa(acc[0], x[0], x[1], a2);
        csa(acc[0], x[2], x[3], b2);
        csa(acc[1], a2, b2, a4);
        csa(acc[0], x[4], x[5], a2);
        csa(acc[0], x[6], x[7], b2);
        csa(acc[1], a2, b2, b4);
        csa(acc[2], a4, b4, a8);
        csa(acc[0], x[8], x[9], a2);
        csa(acc[0], x[10], x[11], b2);
        csa(acc[1], a2, b2, a4);
        csa(acc[0], x[12], x[13], a2);
        csa(acc[0], x[14], x[15], b2);
        csa(acc[1], a2, b2, b4);
        csa(acc[2], a4, b4, b8);
        csa(acc[3], a8, b8, c16);

        // binary-counter cascade: level p has a parked carry iff bit (p-4) of blk
        uint32_t carry = c16;
#pragma unroll
        for (int p = 4; p < P; ++p) {
            if (!((blk >> (p - 4)) & 1u)) {
                pend[p] = carry;
                break;
            }
            uint32_t nc;
            csa(acc[p], pend[p], carry, nc);
            carry = nc;
        }
        ++blk;
    }

    // fold the parked carries: planes become an ordinary binary number
    {
        uint32_t carry = 0;
#pragma unroll
        for (int p = 4; p < P; ++p) {
            const uint32_t pd = ((blk >> (p - 4)) & 1u) ? pend[p] : 0u;
            uint32_t nc;
            csa(acc[p], pd, carry, nc);
            carry = nc;
        }
    }

    if (!active)
        return;
    const uint32_t tail = (uint32_t)C - 32u * (uint32_t)w; // channels from this word on
    if (EPI == BITGNN_EPI_THRESH_BITS) {
        // bit-sliced (value >= R), R = BIAS + deg/2, scanned from the low plane up
        const uint32_t R = (1u << (P - 1)) + (deg >> 1);
        uint32_t ge = 0xFFFFFFFFu;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint32_t rbit = 0u - ((R >> p) & 1u); // all ones if bit p of R is set
            ge = (acc[p] & ge) | (~rbit & (acc[p] | ge));
        }
        if (tail < 32u)
            ge &= (1u << tail) - 1u;
        uint32_t *o = (uint32_t *)out + (int64_t)row * out_stride * 2;
        o[w] = ge;
        if (w == W32 - 1 && (W32 & 1))
            o[W32] = 0u; // upper half of the last 64-bit word
    } else {
        int32_t *o = (int32_t *)out + (int64_t)row * out_stride + 32 * w;
        const int nb = tail < 32u ? (int)tail : 32;
        for (int b = 0; b < nb; ++b) {
            uint32_t cnt = 0;
#pragma unroll
            for (int p = 0; p < P; ++p)
                cnt |= ((acc[p] >> b) & 1u) << p;
            o[b] = 2 * (int32_t)cnt - (int32_t)deg;
        }
    }
}

// Integer aggregation of the last GCN layer: a group of LPR lanes owns a node,
// lane li sums channel li of the neighbours' int32 rows (coalesced row reads).
template <bool SCALE>
__global__ __launch_bounds__(kBlock) void spmm_i32_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, uint32_t N, const int32_t *__restrict__ Z, int32_t M,
    int64_t z_stride, const float *__restrict__ alpha, void *__restrict__ out,
    int64_t out_stride, int lpr_log2)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t slot = t >> lpr_log2;
    const int li = (int)(t & ((1u << lpr_log2) - 1u));
    if (slot >= N)
        return;
    const uint32_t row = (uint32_t)order[slot];
    const uint32_t beg = rowptr[row], end = rowptr[row + 1];
    for (int c = li; c < M; c += (1 << lpr_log2)) {
        int32_t sum = 0;
        for (uint32_t e = beg; e < end; ++e)
            sum += Z[(int64_t)col[e] * z_stride + c];
        if (SCALE)
            ((float *)out)[(int64_t)row * out_stride + c] = alpha[c] * (float)sum;
        else
            ((int32_t *)out)[(int64_t)row * out_stride + c] = sum;
    }
}

template <int P>
void launch_bspmm_p(hipStream_t s, unsigned grid, int epilogue, const bitgnn_adj *adj,
                    const uint32_t *h32, int64_t h_stride32, int32_t C, int32_t W32,
                    const uint32_t *seeds, void *out, int64_t out_stride)
{
    if (epilogue == BITGNN_EPI_THRESH_BITS)
        bspmm_kernel<P, BITGNN_EPI_THRESH_BITS><<<grid, kBlock, 0, s>>>(
            adj->rowptr, adj->col, adj->order, (uint32_t)adj->n, h32, h_stride32, C, W32, seeds,
            out, out_stride);
    else
        bspmm_kernel<P, BITGNN_EPI_RAW_I32><<<grid, kBlock, 0, s>>>(
            adj->rowptr, adj->col, adj->order, (uint32_t)adj->n, h32, h_stride32, C, W32, seeds,
            out, out_stride);
}

} // namespace

int bg_check_bspmm(bitgnn_ctx *ctx, const bitgnn_adj *adj, const uint64_t *hbits, int32_t C,
                   int64_t h_stride, int epilogue, const int32_t *T, const void *out,
                   int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_bspmm: adj is null");
    BG_REQUIRE(ctx, C >= 1, BITGNN_ERR_INVALID_ARG, "bitgnn_bspmm: C=%d", C);
    BG_REQUIRE(ctx, C <= 2048, BITGNN_ERR_UNSUPPORTED, "bitgnn_bspmm: C=%d > 2048", C);
    const int64_t words = (C + 63) / 64;
    BG_REQUIRE(ctx, h_stride >= words, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bspmm: h_stride=%lld < %lld", (long long)h_stride, (long long)words);
    BG_REQUIRE(ctx, epilogue == BITGNN_EPI_RAW_I32 || epilogue == BITGNN_EPI_THRESH_BITS,
               BITGNN_ERR_INVALID_ARG, "bitgnn_bspmm: epilogue=%d", epilogue);
    const int64_t need = epilogue == BITGNN_EPI_THRESH_BITS ? words : C;
    BG_REQUIRE(ctx, out_stride >= need, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bspmm: out_stride=%lld < %lld", (long long)out_stride, (long long)need);
    BG_REQUIRE(ctx, hbits && out, BITGNN_ERR_INVALID_ARG, "bitgnn_bspmm: null pointer");
    BG_REQUIRE(ctx, epilogue != BITGNN_EPI_THRESH_BITS || T, BITGNN_ERR_INVALID_ARG,
               "bitgnn_bspmm: THRESH_BITS needs T");
    BG_REQUIRE(ctx,
               bg_aligned(hbits, 8) && bg_aligned(T, 4) &&
                   bg_aligned(out, epilogue == BITGNN_EPI_THRESH_BITS ? 8 : 4),
               BITGNN_ERR_ALIGNMENT, "bitgnn_bspmm: misaligned pointer");
    BG_REQUIRE(ctx, adj->max_degree < (1ll << 24), BITGNN_ERR_RANGE,
               "bitgnn_bspmm: max degree %lld >= 2^24", (long long)adj->max_degree);
    return BITGNN_OK;
}

int bg_launch_bspmm(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const uint64_t *hbits,
                    int32_t C, int64_t h_stride, int epilogue, const int32_t *T, void *out,
                    int64_t out_stride)
{
    const int32_t W32 = (C + 31) / 32;
    // planes: need max_degree < 2^(P-2)
    int P = 12;
    while ((1ll << (P - 2)) <= adj->max_degree)
        P += (P == 20) ? 6 : 4; // 12, 16, 20, 26
    const uint32_t *seeds = nullptr;
    if (epilogue == BITGNN_EPI_THRESH_BITS) {
        const int entries = 2 * P * W32;
        BG_REQUIRE(ctx, (size_t)entries <= ctx->seed_table_words, BITGNN_ERR_UNSUPPORTED,
                   "bitgnn_bspmm: seed table too small");
        bspmm_seed_kernel<<<(entries + 127) / 128, 128, 0, s>>>(T, C, W32, P, ctx->seed_table);
        BG_LAUNCH_CHECK(ctx, "bspmm_seed");
        seeds = ctx->seed_table;
    }
    const int64_t threads = adj->n * (int64_t)W32;
    const int64_t grid = (threads + kBlock - 1) / kBlock;
    BG_REQUIRE(ctx, grid < (1ll << 31), BITGNN_ERR_UNSUPPORTED, "bitgnn_bspmm: N*C too large");
    const uint32_t *h32 = (const uint32_t *)hbits;
    switch (P) {
    case 12:
        launch_bspmm_p<12>(s, (unsigned)grid, epilogue, adj, h32, h_stride * 2, C, W32, seeds, out,
                           out_stride);
        break;
    case 16:
        launch_bspmm_p<16>(s, (unsigned)grid, epilogue, adj, h32, h_stride * 2, C, W32, seeds, out,
                           out_stride);
        break;
    case 20:
        launch_bspmm_p<20>(s, (unsigned)grid, epilogue, adj, h32, h_stride * 2, C, W32, seeds, out,
                           out_stride);
        break;
    default:
        launch_bspmm_p<26>(s, (unsigned)grid, epilogue, adj, h32, h_stride * 2, C, W32, seeds, out,
                           out_stride);
        break;
    }
    BG_LAUNCH_CHECK(ctx, "bitgnn_bspmm");
    return BITGNN_OK;
}

extern "C" int bitgnn_bspmm(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                            const uint64_t *hbits, int32_t C, int64_t h_stride, int epilogue,
                            const int32_t *T, void *out, int64_t out_stride)
{
    int rc = bg_check_bspmm(ctx, adj, hbits, C, h_stride, epilogue, T, out, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    return bg_launch_bspmm(ctx, (hipStream_t)stream, adj, hbits, C, h_stride, epilogue, T, out,
                           out_stride);
}

int bg_check_spmm_i32(bitgnn_ctx *ctx, const bitgnn_adj *adj, const int32_t *Z, int32_t M,
                      int64_t z_stride, int64_t z_abs_bound, const void *out, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_spmm_i32: adj is null");
    BG_REQUIRE(ctx, M >= 1 && z_stride >= M && out_stride >= M && z_abs_bound >= 0,
               BITGNN_ERR_INVALID_ARG, "bitgnn_spmm_i32: M=%d z_stride=%lld out_stride=%lld", M,
               (long long)z_stride, (long long)out_stride);
    BG_REQUIRE(ctx, Z && out, BITGNN_ERR_INVALID_ARG, "bitgnn_spmm_i32: null pointer");
    BG_REQUIRE(ctx, bg_aligned(Z, 4) && bg_aligned(out, 4), BITGNN_ERR_ALIGNMENT,
               "bitgnn_spmm_i32: misaligned pointer");
    BG_REQUIRE(ctx,
               z_abs_bound < (1ll << 31) &&
                   (adj->max_degree == 0 || z_abs_bound < (1ll << 31) / adj->max_degree),
               BITGNN_ERR_RANGE, "bitgnn_spmm_i32: max_degree %lld * bound %lld >= 2^31",
               (long long)adj->max_degree, (long long)z_abs_bound);
    return BITGNN_OK;
}

int bg_launch_spmm_i32(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const int32_t *Z,
                       int32_t M, int64_t z_stride, const float *alpha, void *out,
                       int64_t out_stride)
{
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < M && lpr_log2 < 6)
        ++lpr_log2;
    const int64_t threads = adj->n << lpr_log2;
    const int64_t grid = (threads + kBlock - 1) / kBlock;
    BG_REQUIRE(ctx, grid < (1ll << 31), BITGNN_ERR_UNSUPPORTED, "bitgnn_spmm_i32: N too large");
    if (alpha)
        spmm_i32_kernel<true><<<(unsigned)grid, kBlock, 0, s>>>(
            adj->rowptr, adj->col, adj->order, (uint32_t)adj->n, Z, M, z_stride, alpha, out,
            out_stride, lpr_log2);
    else
        spmm_i32_kernel<false><<<(unsigned)grid, kBlock, 0, s>>>(
            adj->rowptr, adj->col, adj->order, (uint32_t)adj->n, Z, M, z_stride, alpha, out,
            out_stride, lpr_log2);
    BG_LAUNCH_CHECK(ctx, "bitgnn_spmm_i32");
    return BITGNN_OK;
}

extern "C" int bitgnn_spmm_i32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                               const int32_t *Z, int32_t M, int64_t z_stride, int64_t z_abs_bound,
                               const float *alpha, void *out, int64_t out_stride)
{
    int rc = bg_check_spmm_i32(ctx, adj, Z, M, z_stride, z_abs_bound, out, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_REQUIRE(ctx, bg_aligned(alpha, 4), BITGNN_ERR_ALIGNMENT, "bitgnn_spmm_i32: misaligned alpha");
    BG_NEED_DEVICE(ctx);
    return bg_launch_spmm_i32(ctx, (hipStream_t)stream, adj, Z, M, z_stride, alpha, out,
                              out_stride);
}
