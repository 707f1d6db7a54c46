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
// across channels: a neighbour's row is read as whole 256-byte segments.  The column ids
// and factors of 64 neighbours (and, for bit rows, their words) are fetched with one load
// each, two blocks / one block ahead, and handed out by lane reads; 16 neighbours' rows are
// in flight per wavefront.  What bounds it (232,965 nodes, 110.6 M non-zeros): wide float
// rows by the gathered bytes, nnz * 4 C, which the caches deliver at ~9.4 TB/s (C = 128:
// 6.0 ms) -- the price of full-precision aggregation that the bit path avoids; rows of 128
// bytes or less by the rate of gather requests (~1.7-2.0 ms whatever the width).  The output
// of a BMM is therefore aggregated from its raw integers in int16 (XKIND 2: half the bytes,
// C = 128: 3.2 ms) with the scale applied here.
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

// kTiles: 64-channel tiles a lane accumulates per walk of the row (1, 2 or 4: the smallest
// that covers C, so that no register waits for a tile the row does not have).
// kAhead: neighbours whose rows are in flight together.  The gathers are served by the
// caches at a latency of microseconds, so what a wavefront keeps in flight sets the rate:
// with 4 neighbours the kernel ran at the same speed on half the bytes.

// XKIND: 0 float rows, 1 packed +-1 rows, 2 int16 rows with a per-channel scale (the raw
// integers of a BMM and its SCL: the value alpha_c * (float)z is formed here, with the same
// single rounding as the BMM's own scale epilogue, from half the gathered bytes)
template <int XKIND, bool BITS_OUT, int kTiles>
__global__ __launch_bounds__(256) void spmm_f32_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, uint32_t n, const void *__restrict__ xv, int64_t ldx,
    const float *__restrict__ xscale, int32_t C, const float *__restrict__ r,
    const float *__restrict__ f, const float *__restrict__ tau, void *__restrict__ outv,
    int64_t ldo)
{
    constexpr bool XBITS = XKIND == 1;
    constexpr int kAhead = kTiles == 4 ? 8 : 16;
    // wave-uniform on purpose: row bounds, neighbour ids and row addresses then live in
    // scalar registers and the loads take a scalar base plus a 32-bit lane offset
    const uint32_t slot =
        blockIdx.x * 4 + (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t lane = threadIdx.x & 63;
    if (slot >= n) // wave-uniform
        return;
    const uint32_t i = (uint32_t)order[slot];
    const uint32_t beg = rowptr[i], end = rowptr[i + 1];
    const float ri = r ? r[i] : 1.0f;
    const uint64_t *xb = (const uint64_t *)xv;

    for (int32_t c0 = 0; c0 < C; c0 += 64 * kTiles) {
        float acc[kTiles], sc[kTiles];
        uint32_t cc[kTiles];  // this lane's channel of every tile, clamped into the row
        uint32_t off[kTiles]; // ... as a byte offset into a row of x
        bool live[kTiles];
#pragma unroll
        for (int u = 0; u < kTiles; ++u) {
            acc[u] = 0.0f;
            const int32_t c = c0 + 64 * u + (int32_t)lane;
            live[u] = c < C;
            cc[u] = (uint32_t)(live[u] ? c : C - 1);
            off[u] = cc[u] * (XKIND == 2 ? 2u : 4u);
            sc[u] = XKIND == 2 ? xscale[cc[u]] : 1.0f;
        }
        // The column ids of a block of 64 neighbours are requested two blocks ahead and
        // their factors one block ahead, so that a block waits for its rows only.
        auto ids_of = [&](uint32_t k) -> uint32_t { // lane's id in the block starting at k
            if (k >= end)
                return 0u;
            const uint32_t c = end - k < 64u ? end - k : 64u;
            return (uint32_t)col[k + (lane < c ? lane : c - 1)];
        };
        uint32_t jl = ids_of(beg);
        uint32_t jl_next = ids_of(beg + 64);
        float fl = f ? f[jl] : 1.0f;
        for (uint32_t k0 = beg; k0 < end; k0 += 64) {
            const uint32_t cnt = end - k0 < 64u ? end - k0 : 64u;
            const float fl_next = f ? f[jl_next] : 1.0f; // node 0 past the end: never used
            const uint32_t jl_after = ids_of(k0 + 128);
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
                // one neighbour: its factor and words are read from its lane; a word, being
                // the same for all lanes, serves as the lane mask that picks +f or -f (a
                // tile past the last channel sums zero words and is never stored)
                auto add_neighbour = [&](int t) {
                    const float fj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fl), t));
#pragma unroll
                    for (int u = 0; u < kTiles; ++u) {
                        const uint64_t word =
                            (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)wlo[u], t) |
                            ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)whi[u], t) << 32);
                        const float x = __builtin_amdgcn_inverse_ballot_w64(word) ? 1.0f : -1.0f;
                        acc[u] = acc[u] + mul_rounded(fj, x);
                    }
                };
                uint32_t t = 0;
                for (; t + 4 <= cnt; t += 4) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        add_neighbour((int)t + q);
                }
                for (; t < cnt; ++t)
                    add_neighbour((int)t);
            }
            // The scalar unit is what limits narrow rows, so a neighbour costs it as little
            // as possible: the 64-bit row offset is computed once per lane for the block's
            // 64 neighbours and handed out by lane reads (lanes past the block's end repeat
            // its last neighbour, so a turn needs no clamping), and a full turn adds its
            // neighbours without asking whether each exists.
            const uint64_t rofs = (uint64_t)jl * (uint64_t)(ldx * (XKIND == 2 ? 2 : 4));
            const uint32_t rlo = (uint32_t)rofs, rhi = (uint32_t)(rofs >> 32);
            for (uint32_t t = 0; !XBITS && t < cnt; t += kAhead) {
                float fq[kAhead], xq[kAhead][kTiles];
#pragma unroll
                for (int q = 0; q < kAhead; ++q) {
                    const int tt = (int)t + q; // < 64, wave-uniform
                    const uint64_t ro =
                        (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)rlo, tt) |
                        ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)rhi, tt) << 32);
                    fq[q] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fl), tt));
                    const char *rowp = (const char *)xv + ro; // scalar
#pragma unroll
                    for (int u = 0; u < kTiles; ++u) {
                        if (XKIND == 2)
                            xq[q][u] = (float)*(const int16_t *)(rowp + off[u]);
                        else
                            xq[q][u] = *(const float *)(rowp + off[u]);
                    }
                }
                if (cnt - t >= (uint32_t)kAhead) {
#pragma unroll
                    for (int q = 0; q < kAhead; ++q)
#pragma unroll
                        for (int u = 0; u < kTiles; ++u) {
                            const float x =
                                XKIND == 2 ? mul_rounded(sc[u], xq[q][u]) : xq[q][u];
                            acc[u] = acc[u] + mul_rounded(fq[q], x);
                        }
                } else {
#pragma unroll
                    for (int q = 0; q < kAhead; ++q) {
                        if (t + q < cnt) { // wave-uniform
#pragma unroll
                            for (int u = 0; u < kTiles; ++u) {
                                const float x =
                                    XKIND == 2 ? mul_rounded(sc[u], xq[q][u]) : xq[q][u];
                                acc[u] = acc[u] + mul_rounded(fq[q], x);
                            }
                        }
                    }
                }
            }
            jl = jl_next;
            jl_next = jl_after;
            fl = fl_next;
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
    BG_REQUIRE(ctx, adj->n < (1ll << 31) && C <= (1 << 29), BITGNN_ERR_UNSUPPORTED,
               "bitgnn_spmm_f32: N or C too large");
    return BITGNN_OK;
}

// `xscale` non-null: x holds int16 rows (ldx in int16 units) and a value is
// xscale[c] * (float)x; otherwise x_is_bits selects packed +-1 or float rows.
int bg_launch_spmm_f32(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const void *x,
                       int x_is_bits, int32_t C, int64_t ldx, const float *r, const float *f,
                       int epilogue, const float *tau, void *out, int64_t ldo,
                       const float *xscale)
{
    if (adj->n == 0)
        return BITGNN_OK;
    const bool bits_out = epilogue == BITGNN_EPI_THRESH_BITS;
    const unsigned grid = (unsigned)((adj->n + 3) / 4);
#define BG_SPMM_F32T(XK, BO, TL)                                                                  \
    spmm_f32_kernel<XK, BO, TL><<<grid, 256, 0, s>>>(adj->rowptr, adj->col, adj->order,          \
                                                     (uint32_t)adj->n, x, ldx, xscale, C, r, f,   \
                                                     tau, out, ldo)
#define BG_SPMM_F32(XK, BO)                                                                       \
    do {                                                                                          \
        if (C <= 64)                                                                              \
            BG_SPMM_F32T(XK, BO, 1);                                                              \
        else if (C <= 128)                                                                        \
            BG_SPMM_F32T(XK, BO, 2);                                                              \
        else                                                                                      \
            BG_SPMM_F32T(XK, BO, 4);                                                              \
    } while (0)
    bg_time_begin(ctx, s);
    if (xscale) {
        if (bits_out)
            BG_SPMM_F32(2, true);
        else
            BG_SPMM_F32(2, false);
    } else if (x_is_bits) {
        if (bits_out)
            BG_SPMM_F32(1, true);
        else
            BG_SPMM_F32(1, false);
    } else {
        if (bits_out)
            BG_SPMM_F32(0, true);
        else
            BG_SPMM_F32(0, false);
    }
    bg_time_end(ctx, s);
#undef BG_SPMM_F32
#undef BG_SPMM_F32T
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
                              tau, out, ldo, nullptr);
}

int bg_check_spmm_i16(bitgnn_ctx *ctx, const bitgnn_adj *adj, const int16_t *z, int32_t C,
                      int64_t ldz, const float *alpha, const float *r, const float *f,
                      int epilogue, const float *tau, const void *out, int64_t ldo)
{
    // same shape rules as float rows (ldz counts int16 elements; z is 4-byte aligned)
    int rc = bg_check_spmm_f32(ctx, adj, z, 0, C, ldz, r, f, epilogue, tau, out, ldo);
    if (rc != BITGNN_OK)
        return rc;
    BG_REQUIRE(ctx, alpha, BITGNN_ERR_INVALID_ARG, "bitgnn_spmm_i16: alpha is null");
    BG_REQUIRE(ctx, bg_aligned(alpha, 4), BITGNN_ERR_ALIGNMENT,
               "bitgnn_spmm_i16: misaligned alpha");
    return BITGNN_OK;
}

extern "C" int bitgnn_spmm_i16(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                               const int16_t *z, int32_t C, int64_t ldz, const float *alpha,
                               const float *r, const float *f, int epilogue, const float *tau,
                               void *out, int64_t ldo)
{
    int rc = bg_check_spmm_i16(ctx, adj, z, C, ldz, alpha, r, f, epilogue, tau, out, ldo);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    return bg_launch_spmm_f32(ctx, (hipStream_t)stream, adj, z, 0, C, ldz, r, f, epilogue, tau,
                              out, ldo, alpha);
}

namespace {

// int32 rows -> int16 rows in place (the int16 row starts where the int32 row did): one
// wavefront per row reads a 64-channel tile, then writes it; the bytes a tile's write
// covers belong to this tile's first half or to tiles already read.  The two views of the
// row alias on purpose: the destination type says so, and compiler barriers keep every
// tile's load in front of its store and the store in front of the next tile's load.
typedef int16_t __attribute__((may_alias)) i16_alias;
__global__ __launch_bounds__(256) void narrow_rows_kernel(int32_t *z, int64_t n, int32_t M,
                                                          int64_t ld32)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n)
        return;
    const volatile int32_t *src = z + row * ld32;
    i16_alias *dst = (i16_alias *)(z + row * ld32);
    for (int32_t c0 = 0; c0 < M; c0 += 64) {
        const int32_t c = c0 + lane;
        const int32_t v = c < M ? src[c] : 0;
        asm volatile("" ::: "memory"); // the whole tile is loaded (one instruction) ...
        if (c < M)
            dst[c] = (int16_t)v; // ... before any lane stores (the store waits for the load)
        asm volatile("" ::: "memory");
    }
}

} // namespace

// Raw BMM integers (|z| <= 32767) in int32 rows of stride ld32 -> int16 rows of stride
// 2 * ld32 (in int16 units) at the same addresses.
int bg_launch_narrow_rows(bitgnn_ctx *ctx, hipStream_t s, int32_t *z, int64_t n, int32_t M,
                          int64_t ld32)
{
    if (n == 0)
        return BITGNN_OK;
    narrow_rows_kernel<<<(unsigned)((n + 3) / 4), 256, 0, s>>>(z, n, M, ld32);
    BG_LAUNCH_CHECK(ctx, "narrow_rows_kernel");
    return BITGNN_OK;
}
