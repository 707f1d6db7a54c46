// BMM on the matrix cores (Section 2.2: c = n - 2 popc(a xor b); the paper runs it on
// 1-bit tensor cores, which CDNA4 does not have).  The product is a dense contraction, so
// the bits are widened to 0/1 bytes on the fly and fed to v_mfma_i32_16x16x64_i8:
//   D[i][c] = sum_k x_ik w_kc            (x, w in {0,1})
//   popc(x_i xor w_c) = px_i + pw_c - 2 D[i][c]
//   Z[i][c] = K - 2 px_i - 2 pw_c + 4 D[i][c]
// with px, pw the popcounts of the stored rows (pad bits are zero in both operands).
//
// gfx950 mapping
//  - the weights, widened once per call to bytes (row stride K' + 16 so that the 16-byte
//    operand reads of 16 columns fall into different LDS bank groups), stay in LDS for the
//    whole life of a persistent workgroup (M' (K' + 16) <= 144 KB: wider outputs run as
//    column chunks of whole 64-bit output words, one launch each);
//  - a wavefront owns 32 node rows (two operands, widened from their packed words with
//    three VALU ops per four bytes) and walks column groups of 128: 16 accumulators of
//    16x16, every weight operand read from LDS feeds two MFMAs;
//  - the weights are the MFMA's first operand, so a lane ends up with 4 consecutive columns
//    of one node row: integers and logits leave as runs of 4, thresholded bits are built
//    in-lane and OR-ed over the 4 lanes that share the row;
//  - the rows of the next panel are requested while the current one is computed.
// Against the VALU kernel (2 lane-ops per 32 bit-MACs: 629 T bit-MAC/s at peak, ~310
// reached) the int8 MFMA peak is 2,500 T MAC/s; this kernel reaches ~740 on 2.4 M x 512 x 256
// (widening and the epilogue share the issue slots with the MFMAs).  It is chosen when the
// weights fit in LDS and there are enough rows to repay the set-up.
#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kMfWaves = 8;            // wavefronts per workgroup
constexpr int kMfRows = 32;            // rows per wavefront (two 16-row operands)
constexpr int kMfPanel = kMfWaves * kMfRows;
constexpr int kMfGroup = 8;            // column tiles of 16 per pass (128 columns)
#ifndef BITGNN_MF_PAD
#define BITGNN_MF_PAD 16
#endif
constexpr int kMfPad = BITGNN_MF_PAD;  // bytes added to a weight row in LDS (bank spreading)
constexpr size_t kMfLdsLimit = 144 * 1024;

// w8[c * ldw + k] = stored bit k of weight row c (0 beyond the kbits stored bits or M);
// pw[c] = its popcount.  Every stored bit position counts, not only k < K: rows may hold
// pad bits in the middle (concatenated segments), which are zero in both operands.
__global__ __launch_bounds__(256) void bgemm_widen_w_kernel(const uint32_t *__restrict__ w32,
                                                            int64_t w_stride32, int32_t kbits,
                                                            int32_t M, int32_t ldw,
                                                            uint8_t *__restrict__ w8,
                                                            int32_t *__restrict__ pw)
{
    __shared__ int part[4];
    const int c = blockIdx.x, t = threadIdx.x;
    int cnt = 0;
    for (int k = t; k < ldw; k += 256) {
        int v = 0;
        if (c < M && k < kbits)
            v = (w32[(int64_t)c * w_stride32 + (k >> 5)] >> (k & 31)) & 1u;
        w8[(int64_t)c * ldw + k] = (uint8_t)v;
        cnt += v;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1)
        cnt += __shfl_xor(cnt, d, 64);
    if ((t & 63) == 0)
        part[t >> 6] = cnt;
    __syncthreads();
    if (t == 0)
        pw[c] = part[0] + part[1] + part[2] + part[3];
}

// 16 bits -> 16 bytes of 0/1 (one MFMA operand of a lane)
__device__ __forceinline__ v4i widen16(uint32_t bits)
{
    v4i r;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        r[i] = (int)((((bits >> (4 * i)) & 0xFu) * 0x00204081u) & 0x01010101u);
    return r;
}

// KS = 64-bit words of a packed row held in registers (K <= 64 KS; 2, 4, 8 or 16).
template <int EPI, int KS>
__global__ __launch_bounds__(kMfWaves * 64) void bgemm_mfma_kernel(
    const uint64_t *__restrict__ xbits, int64_t n, int64_t x_stride, int32_t K, int32_t ksteps,
    const uint4 *__restrict__ w8g, int32_t ldw, const int32_t *__restrict__ pw, int32_t M,
    int32_t Mp, const int32_t *__restrict__ T, const float *__restrict__ alpha,
    void *__restrict__ out, int64_t out_stride)
{
    extern __shared__ uint4 wl[]; // Mp rows of ldw bytes
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    for (int i = tid; i < Mp * (ldw / 16); i += kMfWaves * 64)
        wl[i] = w8g[i];
    char *wbytes = (char *)wl;
    const int64_t last = n - 1;
    // column constants behind the weights in LDS, fixed for the run:
    // THRESH: T - K + 2 pw (a column beyond M never passes); else K - 2 pw, and the scale
    int32_t *colk = (int32_t *)(wbytes + (size_t)Mp * ldw);
    float *colf = (float *)(colk + Mp);
    for (int c = tid; c < Mp; c += kMfWaves * 64) {
        const bool c_ok = c < M;
        const int pwc = c_ok ? pw[c] : 0;
        if (EPI == BITGNN_EPI_THRESH_BITS) {
            // |Z| <= K, so thresholds beyond +-(K + 1) decide nothing more: clamped first,
            // the folded constant cannot overflow
            int32_t tc = c_ok ? T[c] : 0;
            tc = tc > K + 1 ? K + 1 : (tc < -K - 1 ? -K - 1 : tc);
            colk[c] = c_ok ? tc - K + 2 * pwc : 0x7FFFFFFF;
        }
        else
            colk[c] = K - 2 * pwc;
        colf[c] = (EPI == BITGNN_EPI_SCALE_F32 && c_ok) ? alpha[c] : 0.0f;
    }
    __syncthreads(); // the last barrier: weights and constants are read-only from here on

    // the packed words of the wavefront's two 16-row operands (clamped row and word index:
    // no load is conditional, so all of them travel together)
    auto load_rows = [&](int64_t panel, uint64_t (&wa)[KS], uint64_t (&wb)[KS]) {
        const int64_t row0 = panel * kMfPanel + wave * kMfRows;
        const int64_t ra = row0 + r < last ? row0 + r : last;
        const int64_t rb = row0 + 16 + r < last ? row0 + 16 + r : last;
        const uint64_t *xa = xbits + ra * x_stride, *xb = xbits + rb * x_stride;
#pragma unroll
        for (int u = 0; u < KS; ++u) {
            const int sc = u < ksteps ? u : ksteps - 1;
            wa[u] = xa[sc];
            wb[u] = xb[sc];
        }
    };

    // The weights go in as the MFMA's A operand (its rows = weight columns) and the node
    // rows as B, so a lane ends up with 4 consecutive columns (4 g + j of every tile) of ONE
    // node row (r): its own popcount applies, integers and logits leave as 16-byte stores,
    // and the thresholded bits of a row are assembled in-lane and OR-ed over the 4 lanes
    // that share the row.
    auto compute = [&](int64_t panel, const uint64_t (&wa)[KS], const uint64_t (&wb)[KS]) {
        const int64_t row0 = panel * kMfPanel + wave * kMfRows;
        if (row0 >= n)
            return;
        int px2[2] = {0, 0}; // twice the popcount of the lane's row in either operand
#pragma unroll
        for (int u = 0; u < KS; ++u)
            if (u < ksteps) {
                px2[0] += 2 * __popcll(wa[u]);
                px2[1] += 2 * __popcll(wb[u]);
            }
        for (int c0 = 0; c0 < Mp; c0 += kMfGroup * 16) {
            const int ntile = (Mp - c0) / 16 < kMfGroup ? (Mp - c0) / 16 : kMfGroup;
            v4i acc[2][kMfGroup];
#pragma unroll
            for (int t = 0; t < kMfGroup; ++t)
                acc[0][t] = acc[1][t] = (v4i){0, 0, 0, 0};
            const char *wcol = wbytes + (size_t)(c0 + r) * ldw + 16 * g;
#pragma unroll
            for (int u = 0; u < KS; ++u) {
                if (u < ksteps) { // wave-uniform
                    const v4i a0 = widen16((uint32_t)(wa[u] >> (16 * g)) & 0xFFFFu);
                    const v4i a1 = widen16((uint32_t)(wb[u] >> (16 * g)) & 0xFFFFu);
                    const char *wk = wcol + 64 * u;
#pragma unroll
                    for (int t = 0; t < kMfGroup; ++t) {
                        if (t < ntile) { // wave-uniform
                            const v4i b = *(const v4i *)(wk + (size_t)t * 16 * ldw);
                            acc[0][t] =
                                __builtin_amdgcn_mfma_i32_16x16x64_i8(b, a0, acc[0][t], 0, 0, 0);
                            acc[1][t] =
                                __builtin_amdgcn_mfma_i32_16x16x64_i8(b, a1, acc[1][t], 0, 0, 0);
                        }
                    }
                }
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int64_t row = row0 + 16 * h + r;
                if (EPI == BITGNN_EPI_THRESH_BITS) {
                    // bit = (4 D - 2 px >= T - K + 2 pw), at position 16 t' + 4 g + j of the
                    // 64-column word t / 4
                    uint32_t wlo[kMfGroup / 4] = {}, whi[kMfGroup / 4] = {};
#pragma unroll
                    for (int t = 0; t < kMfGroup; ++t) {
                        if (t >= ntile) // wave-uniform; tiles beyond M' contribute no bits
                            continue;
                        const v4i ck = *(const v4i *)(colk + c0 + 16 * t + 4 * g);
                        uint32_t nib = 0;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            nib |= (4 * acc[h][t][j] - px2[h] >= ck[j]) ? (1u << j) : 0u;
                        if ((t & 2) == 0)
                            wlo[t / 4] |= nib << (16 * (t & 1));
                        else
                            whi[t / 4] |= nib << (16 * (t & 1));
                    }
#pragma unroll
                    for (int wi = 0; wi < kMfGroup / 4; ++wi) {
                        uint32_t lo = wlo[wi] << (4 * g), hi = whi[wi] << (4 * g);
                        lo |= __shfl_xor(lo, 16, 64);
                        hi |= __shfl_xor(hi, 16, 64);
                        lo |= __shfl_xor(lo, 32, 64);
                        hi |= __shfl_xor(hi, 32, 64);
                        const int wcolumn = c0 / 64 + wi;
                        if (g == 0 && row < n && wcolumn * 64 < M)
                            ((uint64_t *)out)[row * out_stride + wcolumn] =
                                ((uint64_t)hi << 32) | lo;
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < kMfGroup; ++t) {
                        const int c = c0 + 16 * t + 4 * g;
                        if (t < ntile && row < n) {
                            const v4i ck = *(const v4i *)(colk + c); // K - 2 pw here
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int32_t z = 4 * acc[h][t][j] - px2[h] + ck[j];
                                if (c + j < M) {
                                    if (EPI == BITGNN_EPI_RAW_I32)
                                        ((int32_t *)out)[row * out_stride + c + j] = z;
                                    else
                                        ((float *)out)[row * out_stride + c + j] =
                                            colf[c + j] * (float)z;
                                }
                            }
                        }
                    }
                }
            }
        }
    };

    int64_t panel = blockIdx.x;
    const int64_t step = gridDim.x;
    if (KS > 8) {
        // rows of 16 words: one register set (a second one would spill); a panel's products
        // take long enough here that the other wavefront of the SIMD covers the loads
        uint64_t a0[KS], a1[KS];
        for (; panel * kMfPanel < n; panel += step) { // uniform over the workgroup
            load_rows(panel, a0, a1);
            compute(panel, a0, a1);
        }
        return;
    }
    // two register sets: the rows of the next panel are requested before the current
    // panel is computed
    uint64_t a0[KS], a1[KS], b0[KS], b1[KS];
    load_rows(panel, a0, a1);
    for (;;) {
        load_rows(panel + step, b0, b1);
        compute(panel, a0, a1);
        panel += step;
        if (panel * kMfPanel >= n) // uniform over the workgroup
            break;
        load_rows(panel + step, a0, a1);
        compute(panel, b0, b1);
        panel += step;
        if (panel * kMfPanel >= n)
            break;
    }
}

} // namespace

// Output columns per launch: all of them when the widened weights fit in LDS, else the
// largest multiple of 64 (whole output words) that does; 0 = the shape does not fit at all.
static int32_t mf_chunk(int64_t Kp, int64_t Mp)
{
    const int64_t row = Kp + kMfPad + 8; // widened weights + column constants, per column
    if (Mp * row <= (int64_t)kMfLdsLimit)
        return (int32_t)Mp;
    return (int32_t)((int64_t)kMfLdsLimit / row / 64 * 64);
}

// Whether the matrix-core kernel takes this shape: weights (or a column chunk of them)
// resident in LDS, enough work to be compute-bound (small M or K leave the VALU kernel at the
// memory bound anyway).
bool bg_bgemm_mfma_applies(const bitgnn_ctx *ctx, int64_t n, int32_t kwords, int32_t M)
{
    if (ctx->bgemm_path == 1)
        return false;
    const int64_t Kp = (int64_t)kwords * 64, Mp = ((int64_t)M + 15) / 16 * 16;
    // rows are held in registers (up to 16 words); weights and column constants in LDS
    const int32_t chunk = mf_chunk(Kp, Mp);
    if (Kp > 1024 || (chunk < Mp && chunk < 64))
        return false;
    if (ctx->bgemm_path == 2)
        return true;
    // measured on MI355X: the fixed cost (widening the weights, one LDS copy of them per
    // workgroup: 11-22 us whatever n, once per column chunk) is repaid from 40-70 thousand
    // rows on, depending on the shape (K x M = 512 x 256: level at 70 K; 128 x 128: from
    // 20 K; 256 x 40: only beyond 100 K); 1.4x - 2.4x faster for large n.  Rows of more
    // than 8 words and outputs in column chunks pay that cost per chunk and load rows without
    // a second register set: level with the VALU kernel at 89 K rows (1000 x 256: 79 against
    // 83 us), 1.4x at 200 K, 1.9x at 500 K, 3x at 2.4 M rows
    return n >= ((Kp > 512 || chunk < Mp) ? 131072 : 65536);
}

int bg_launch_bgemm_mfma(bitgnn_ctx *ctx, hipStream_t s, const uint64_t *xbits, int64_t n,
                         int64_t x_stride, int32_t K, int32_t kwords, const uint64_t *wbits,
                         int32_t M, int64_t w_stride, int epilogue, const int32_t *T,
                         const float *alpha, void *out, int64_t out_stride)
{
    const int32_t ldw = kwords * 64 + kMfPad;
    const int32_t chunk = mf_chunk((int64_t)kwords * 64, ((int64_t)M + 15) / 16 * 16);
    BG_REQUIRE(ctx, chunk > 0 && (chunk >= 64 || chunk >= M) && kwords <= 16, BITGNN_ERR_UNSUPPORTED,
               "bitgnn_bgemm: shape too large for the matrix-core kernel");
    const int64_t panels = (n + kMfPanel - 1) / kMfPanel;
    const int64_t cus = ctx->n_cus > 0 ? ctx->n_cus : 256;
    const unsigned grid = (unsigned)(panels < cus ? panels : cus);
    // Column chunks run one after the other on the stream and share the widening scratch: a
    // chunk's launches are ordered behind the previous chunk's kernel, which has read it.
    for (int32_t c0 = 0; c0 < M; c0 += chunk) {
        const int32_t Mc = M - c0 < chunk ? M - c0 : chunk, Mp = (Mc + 15) / 16 * 16;
        const size_t w8_bytes = (size_t)Mp * ldw;
        const size_t lds_bytes = w8_bytes + (size_t)Mp * 8; // + column constants
        BG_REQUIRE(ctx, w8_bytes + (size_t)Mp * 4 <= kBgemmScratchBytes, BITGNN_ERR_UNSUPPORTED,
                   "bitgnn_bgemm: weights too large for the matrix-core kernel's scratch");
        uint8_t *w8 = (uint8_t *)ctx->bgemm_ws;
        int32_t *pw = (int32_t *)(w8 + w8_bytes);
        bgemm_widen_w_kernel<<<Mp, 256, 0, s>>>((const uint32_t *)(wbits + (int64_t)c0 * w_stride),
                                                w_stride * 2, kwords * 64, Mc, ldw, w8, pw);
        BG_LAUNCH_CHECK(ctx, "bgemm_widen_w");
        const int32_t *Tc = T ? T + c0 : nullptr;
        const float *ac = alpha ? alpha + c0 : nullptr;
        void *oc = epilogue == BITGNN_EPI_THRESH_BITS ? (void *)((uint64_t *)out + c0 / 64)
                                                      : (void *)((int32_t *)out + c0);
#define BG_MFMA_KS(E, KS)                                                                         \
    do {                                                                                          \
        BG_HIP(ctx, hipFuncSetAttribute((const void *)bgemm_mfma_kernel<E, KS>,                   \
                                        hipFuncAttributeMaxDynamicSharedMemorySize,               \
                                        (int)lds_bytes));                                         \
        bgemm_mfma_kernel<E, KS><<<grid, kMfWaves * 64, lds_bytes, s>>>(                          \
            xbits, n, x_stride, K, kwords, (const uint4 *)w8, ldw, pw, Mc, Mp, Tc, ac, oc,        \
            out_stride);                                                                          \
    } while (0)
#define BG_MFMA(E)                                                                                \
    do {                                                                                          \
        if (kwords <= 2)                                                                          \
            BG_MFMA_KS(E, 2);                                                                     \
        else if (kwords <= 4)                                                                     \
            BG_MFMA_KS(E, 4);                                                                     \
        else if (kwords <= 8)                                                                     \
            BG_MFMA_KS(E, 8);                                                                     \
        else                                                                                      \
            BG_MFMA_KS(E, 16);                                                                    \
    } while (0)
        switch (epilogue) {
        case BITGNN_EPI_THRESH_BITS: BG_MFMA(BITGNN_EPI_THRESH_BITS); break;
        case BITGNN_EPI_RAW_I32: BG_MFMA(BITGNN_EPI_RAW_I32); break;
        default: BG_MFMA(BITGNN_EPI_SCALE_F32); break;
        }
#undef BG_MFMA_KS
#undef BG_MFMA
        BG_LAUNCH_CHECK(ctx, "bgemm_mfma");
    }
    return BITGNN_OK;
}
