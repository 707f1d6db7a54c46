// Weighted / full-precision aggregation: the BSpMM variants of Section 3.1.1 whose
// activation operand or output is full precision, and the weighted adjacency written as
// the 0/1 matrix times its factorisation vectors,
//   Y[i][c] = r[i] * sum_{j in N(i)} f[j] * x[j][c],
// with x in float or as packed +-1 bits, and Y stored as float or binarized again.
// D^-1/2 A D^-1/2 is r = f = deg^-1/2, the mean aggregator r = 1/deg.
//
// Arithmetic: fp32, one rounded multiply and one rounded add per neighbour in the stored
// (ascending column) order, then one multiply by r[i]; no fused multiply-add, no
// re-association.  A value is therefore reproducible bit for bit, which matters where it
// decides an output bit.
//
// One wavefront per row (rows by decreasing degree, so the long ones start first), lanes
// across channels: a neighbour's float row is read as whole 256-byte segments.  The column
// ids and factors of 64 neighbours (and, for bit rows, their words) are fetched with one
// load each and handed out by lane reads.  The kernel is bound by the gather traffic, nnz * 4 C bytes for float
// activations: this is the price of full-precision aggregation that the bit path avoids.
#include "common.h"

namespace {

// a * b rounded to float by itself: the empty asm makes the product a value of its own,
// so the compiler cannot contract it with the add that follows into a fused multiply-add
__device__ __forceinline__ float mul_rounded(float a, float b)
{
    float p = a * b;
    asm volatile("" : "+v"(p));
    return p;
}

constexpr int kTiles = 4; // 64-channel tiles a lane accumulates per walk of the row
constexpr int kAhead = 4; // neighbours whose rows are in flight together

template <bool XBITS, bool BITS_OUT>
__global__ __launch_bounds__(256) void spmm_f32_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, uint32_t n, const void *__restrict__ xv, int64_t ldx,
    int32_t C, const float *__restrict__ r, const float *__restrict__ f,
    const float *__restrict__ tau, void *__restrict__ outv, int64_t ldo)
{
    const uint32_t slot = blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    if (slot >= n) // wave-uniform
        return;
    const uint32_t i = (uint32_t)order[slot];
    const uint32_t beg = rowptr[i], end = rowptr[i + 1];
    const float ri = r ? r[i] : 1.0f;
    const float *xf = (const float *)xv;
    const uint64_t *xb = (const uint64_t *)xv;

    for (int32_t c0 = 0; c0 < C; c0 += 64 * kTiles) {
        float acc[kTiles];
        uint32_t cc[kTiles]; // this lane's channel of every tile, clamped into the row
        bool live[kTiles];
#pragma unroll
        for (int u = 0; u < kTiles; ++u) {
            acc[u] = 0.0f;
            const int32_t c = c0 + 64 * u + (int32_t)lane;
            live[u] = c < C;
            cc[u] = (uint32_t)(live[u] ? c : C - 1);
        }
        for (uint32_t k0 = beg; k0 < end; k0 += 64) {
            const uint32_t cnt = end - k0 < 64u ? end - k0 : 64u;
            const uint32_t jl = (uint32_t)col[k0 + (lane < cnt ? lane : cnt - 1)];
            const float fl = f ? f[jl] : 1.0f;
            if (XBITS) {
                // Bit rows: every lane fetches the words of its own neighbour (one gather
                // per tile for 64 neighbours); a neighbour's word is then read from its
                // lane and, being the same for all lanes, serves as a lane mask.
                uint32_t wlo[kTiles], whi[kTiles];
#pragma unroll
                for (int u = 0; u < kTiles; ++u) {
                    uint64_t w = 0;
                    if (c0 + 64 * u < C) // wave-uniform
                        w = xb[(int64_t)jl * ldx + (c0 / 64 + u)];
                    wlo[u] = (uint32_t)w;
                    whi[u] = (uint32_t)(w >> 32);
                }
                for (uint32_t t = 0; t < cnt; ++t) {
                    const float fj =
                        __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fl), (int)t));
#pragma unroll
                    for (int u = 0; u < kTiles; ++u) {
                        if (c0 + 64 * u >= C)
                            continue;
                        const uint64_t word =
                            (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)wlo[u], (int)t) |
                            ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)whi[u], (int)t)
                             << 32);
                        const float x = __builtin_amdgcn_inverse_ballot_w64(word) ? 1.0f : -1.0f;
                        acc[u] = acc[u] + mul_rounded(fj, x);
                    }
                }
                continue;
            }
            // kAhead neighbours per turn: their rows are requested together, then added in
            // order (a turn past the end repeats the last neighbour and drops it)
            for (uint32_t t = 0; t < cnt; t += kAhead) {
                float fq[kAhead], xq[kAhead][kTiles];
#pragma unroll
                for (int q = 0; q < kAhead; ++q) {
                    const uint32_t tt = t + q < cnt ? t + q : cnt - 1; // wave-uniform
                    const uint32_t j = (uint32_t)__builtin_amdgcn_readlane((int)jl, (int)tt);
                    fq[q] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fl), (int)tt));
#pragma unroll
                    for (int u = 0; u < kTiles; ++u) {
                        if (c0 + 64 * u >= C) { // wave-uniform: tile beyond the last channel
                            xq[q][u] = 0.0f;
                        } else {
                            xq[q][u] = xf[(int64_t)j * ldx + cc[u]];
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < kAhead; ++q) {
                    if (t + q < cnt) { // wave-uniform
#pragma unroll
                        for (int u = 0; u < kTiles; ++u)
                            acc[u] = acc[u] + mul_rounded(fq[q], xq[q][u]);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kTiles; ++u) {
            if (c0 + 64 * u >= C)
                continue;
            const float y = mul_rounded(ri, acc[u]);
            if (BITS_OUT) {
                const bool bit = live[u] && y >= tau[cc[u]];
                const uint64_t word = __ballot(bit);
                if (lane == 0)
                    ((uint64_t *)outv)[(int64_t)i * ldo + (c0 / 64 + u)] = word;
            } else if (live[u]) {
                ((float *)outv)[(int64_t)i * ldo + cc[u]] = y;
            }
        }
    }
}

} // namespace

int bg_check_spmm_f32(bitgnn_ctx *ctx, const bitgnn_adj *adj, const void *x, int x_is_bits,
                      int32_t C, int64_t ldx, const float *r, const float *f, int epilogue,
                      const float *tau, const void *out, int64_t ldo)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_spmm_f32: adj is null");
    BG_REQUIRE(ctx, epilogue == BITGNN_EPI_SCALE_F32 || epilogue == BITGNN_EPI_THRESH_BITS,
               BITGNN_ERR_INVALID_ARG, "bitgnn_spmm_f32: epilogue %d (SCALE_F32 or THRESH_BITS)",
               epilogue);
    const int64_t cw = ((int64_t)C + 63) / 64;
    const bool bits_out = epilogue == BITGNN_EPI_THRESH_BITS;
    BG_REQUIRE(ctx,
               C >= 1 && ldx >= (x_is_bits ? cw : (int64_t)C) &&
                   ldo >= (bits_out ? cw : (int64_t)C),
               BITGNN_ERR_INVALID_ARG, "bitgnn_spmm_f32: C=%d ldx=%lld ldo=%lld", C, (long long)ldx,
               (long long)ldo);
    BG_REQUIRE(ctx, x && out && (!bits_out || tau), BITGNN_ERR_INVALID_ARG,
               "bitgnn_spmm_f32: null pointer");
    BG_REQUIRE(ctx,
               bg_aligned(x, x_is_bits ? 8 : 4) && bg_aligned(out, bits_out ? 8 : 4) &&
                   bg_aligned(r, 4) && bg_aligned(f, 4) && bg_aligned(tau, 4),
               BITGNN_ERR_ALIGNMENT, "bitgnn_spmm_f32: misaligned pointer");
    BG_REQUIRE(ctx, adj->n < (1ll << 31), BITGNN_ERR_UNSUPPORTED, "bitgnn_spmm_f32: N too large");
    return BITGNN_OK;
}

int bg_launch_spmm_f32(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const void *x,
                       int x_is_bits, int32_t C, int64_t ldx, const float *r, const float *f,
                       int epilogue, const float *tau, void *out, int64_t ldo)
{
    if (adj->n == 0)
        return BITGNN_OK;
    const bool bits_out = epilogue == BITGNN_EPI_THRESH_BITS;
    const unsigned grid = (unsigned)((adj->n + 3) / 4);
#define BG_SPMM_F32(XB, BO)                                                                       \
    spmm_f32_kernel<XB, BO><<<grid, 256, 0, s>>>(adj->rowptr, adj->col, adj->order,              \
                                                 (uint32_t)adj->n, x, ldx, C, r, f, tau, out, ldo)
    bg_time_begin(ctx, s);
    if (x_is_bits) {
        if (bits_out)
            BG_SPMM_F32(true, true);
        else
            BG_SPMM_F32(true, false);
    } else {
        if (bits_out)
            BG_SPMM_F32(false, true);
        else
            BG_SPMM_F32(false, false);
    }
    bg_time_end(ctx, s);
#undef BG_SPMM_F32
    BG_LAUNCH_CHECK(ctx, "bitgnn_spmm_f32");
    return BITGNN_OK;
}

extern "C" int bitgnn_spmm_f32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const void *x,
                               int x_is_bits, int32_t C, int64_t ldx, const float *r,
                               const float *f, int epilogue, const float *tau, void *out,
                               int64_t ldo)
{
    int rc = bg_check_spmm_f32(ctx, adj, x, x_is_bits, C, ldx, r, f, epilogue, tau, out, ldo);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    return bg_launch_spmm_f32(ctx, (hipStream_t)stream, adj, x, x_is_bits, C, ldx, r, f, epilogue,
                              tau, out, ldo);
}
