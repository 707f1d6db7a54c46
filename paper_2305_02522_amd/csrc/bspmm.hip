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
    // v_bitop3_b32: any 3-input boolean in one VALU op (0xE8 majority, 0x96 xor3)
    carry = __builtin_amdgcn_bitop3_b32(acc, b, c, 0xE8);
    acc = __builtin_amdgcn_bitop3_b32(acc, b, c, 0x96);
}

// Seeds of the vertical counters: table[(e*P + p)*W32 + w] bit c' = bit p of
// (BIAS - t(e, c)), c = 32 w + c', BIAS = 2^(P-1), t clamped to +-2^(P-2).
// One half wavefront per table word, one lane per channel: the word is the vote of the 32
// lanes (a thread per word walked its 32 thresholds one after the other: 6 us for a table
// of a few hundred words, a quarter of a small graph's aggregation).  Every lane of the
// wavefront must call; `t` is the thread's index among the threads that build the table.
__device__ __forceinline__ void seed_word_vote(int t, int n_words, const int32_t *__restrict__ T,
                                               int32_t C, int32_t W32, int P,
                                               uint32_t *__restrict__ table)
{
    const int idx = t >> 5, b = t & 31;
    const bool valid = t >= 0 && idx < n_words;
    const int w = valid ? idx % W32 : 0;
    const int p = valid ? (idx / W32) % P : 0;
    const int e = valid ? idx / (W32 * P) : 0;
    const int c = 32 * w + b;
    bool bit = false;
    if (valid && c < C) {
        const int64_t lim = 1ll << (P - 2);
        int64_t th = ((int64_t)T[c] + e + 1) >> 1; // floor
        th = th > lim ? lim : (th < -lim ? -lim : th);
        const uint64_t off = (uint64_t)((1ll << (P - 1)) - th);
        bit = (off >> p) & 1u;
    }
    const uint64_t vote = __ballot(bit);
    if (valid && b == 0)
        table[idx] = (uint32_t)((t & 32) ? vote >> 32 : vote);
}

__global__ __launch_bounds__(256) void bspmm_seed_kernel(const int32_t *__restrict__ T, int32_t C,
                                                         int32_t W32, int P,
                                                         uint32_t *__restrict__ table)
{
    seed_word_vote((int)(blockIdx.x * blockDim.x + threadIdx.x), 2 * P * W32, T, C, W32, P, table);
}

// Epilogue of one (node, 32-channel word): `acc` holds the bit-sliced count (plus
// the seed for THRESH_BITS) as an ordinary binary number in P planes.
template <int P, int EPI>
__device__ __forceinline__ void bspmm_epilogue(const uint32_t (&acc)[P], uint32_t deg, uint32_t row,
                                               int w, int32_t W32, int32_t C,
                                               void *__restrict__ out, int64_t out_stride)
{
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

// The segments of the rows with more than seg_len neighbours, as the kernels see them.
struct RowSegments {
    const uint32_t *seg_ptr;  // [n_long + 1] first segment of long row (by degree-order slot)
    const uint32_t *seg_slot; // [n_long_segs] slot of a segment's row
    uint32_t n_long, n_long_segs;
    uint32_t seg_len;  // neighbours per segment
    int planes;        // planes of a segment's count: seg_len < 2^planes (at most 12)
    uint32_t *partial; // [n_long_segs][planes][W32] bit-sliced counts of the segments
};
static_assert(kSegLenLarge < (1u << 12), "every kernel variant has at least 12 planes");

// A thread group of W32 lanes walks one "virtual row": a segment of at most seg_len
// neighbours of a long row (those come first, and leave their bit-sliced counts in
// `seg.partial` for bspmm_long_rows_kernel), or a whole row of at most seg_len neighbours,
// finished here.  Without the split the longest row of a power-law graph, walked serially at
// one memory latency per 16 neighbours, sets the time of the whole kernel.  (Separate launches
// for the segments and for the other rows were slower on every workload tried.)
template <int P, int EPI>
__global__ __launch_bounds__(kBlock) void bspmm_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, uint32_t N, const uint32_t *__restrict__ h32,
    int64_t h_stride32, int32_t C, int32_t W32, const uint32_t *__restrict__ seeds,
    void *__restrict__ out, int64_t out_stride, RowSegments seg)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t v = t / (uint32_t)W32; // virtual row
    const int w = (int)(t - v * (uint32_t)W32);
    const bool active = v < (uint64_t)seg.n_long_segs + (N - seg.n_long);
    const bool part = v < seg.n_long_segs; // wave-uniform except at one boundary
    uint32_t slot = 0, k = 0;
    if (active) {
        if (part) {
            slot = seg.seg_slot[v];
            k = (uint32_t)v - seg.seg_ptr[slot];
        } else {
            slot = seg.n_long + (uint32_t)(v - seg.n_long_segs);
        }
    }
    const uint32_t row = active ? (uint32_t)order[slot] : 0u;
    const uint32_t rbeg = active ? rowptr[row] : 0u, rend = active ? rowptr[row + 1] : 0u;
    uint32_t e = rbeg + k * seg.seg_len;
    const uint32_t end = part && rend - e > seg.seg_len ? e + seg.seg_len : rend;
    const uint32_t deg = rend - rbeg;

    uint32_t acc[P], pend[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        // the threshold seed of a long row is added when its segments are
        acc[p] = (EPI == BITGNN_EPI_THRESH_BITS && !part)
                     ? seeds[((deg & 1u) * P + p) * W32 + w]
                     : 0u;
        pend[p] = 0u;
    }

    const uint32_t *hw = h32 + w;
    uint32_t blk = 0; // blocks of 16 neighbours consumed so far (wave-uniform)
    // clamped, unconditional loads (masked afterwards): the 16 index loads and then the 16
    // gathers are in flight together instead of one at a time, and the indices of the next
    // 16 neighbours are requested before this block's gathers are waited for, so that a long
    // row pays one memory latency per block instead of two
    const uint32_t last = end > e ? end - 1 : 0u;
    int32_t j[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u)
        j[u] = col[e + u < end ? e + u : last];
    while (__ballot(e < end) != 0ull) {
        uint32_t x[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) // lanes past their row end gather node 0 (always valid)
            x[u] = hw[(int64_t)(e + u < end ? j[u] : 0) * h_stride32];
        const uint32_t e_next = (end - e > (uint32_t)kGroup) ? e + kGroup : end;
#pragma unroll
        for (int u = 0; u < kGroup; ++u)
            j[u] = col[e_next + u < end ? e_next + u : last];
#pragma unroll
        for (int u = 0; u < kGroup; ++u)
            x[u] = e + u < end ? x[u] : 0u;
        e = e_next;

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
    if (part) { // a segment counts at most seg_len: the planes above seg.planes are zero
#pragma unroll
        for (int p = 0; p < 12; ++p)
            if (p < seg.planes)
                seg.partial[((size_t)v * seg.planes + p) * W32 + w] = acc[p];
        return;
    }
    bspmm_epilogue<P, EPI>(acc, deg, row, w, W32, C, out, out_stride);
}

// Long rows: the bit-sliced counts of a row's segments (and the threshold seed) are added
// plane by plane with a carry, then the row is finished as any other.  kMergeLanes lanes
// share a (row, word): each adds every kMergeLanes-th segment (a hub has a hundred and more,
// and one lane would pay a memory latency for each), then the lanes' sums are added pairwise
// across the lanes.
constexpr int kMergeLanes = 16;

template <int P>
__device__ __forceinline__ void planes_add(uint32_t (&acc)[P], const uint32_t (&b)[P])
{
    uint32_t carry = 0;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        uint32_t nc;
        csa(acc[p], b[p], carry, nc);
        carry = nc;
    }
}

template <int P, int EPI>
__global__ __launch_bounds__(kBlock) void bspmm_long_rows_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ order, int32_t C, int32_t W32,
    const uint32_t *__restrict__ seeds, void *__restrict__ out, int64_t out_stride,
    RowSegments seg)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const int q = (int)(t % kMergeLanes);
    const uint64_t g = t / kMergeLanes; // (row, word); its lanes sit side by side in a wavefront
    const uint64_t slot = g / (uint32_t)W32;
    const int w = (int)(g - slot * (uint32_t)W32);
    const bool active = slot < seg.n_long; // the same for the kMergeLanes lanes of a group
    uint32_t acc[P];
#pragma unroll
    for (int p = 0; p < P; ++p)
        acc[p] = 0u;
    if (active) {
        const uint32_t vend = seg.seg_ptr[slot + 1];
        for (uint32_t v = seg.seg_ptr[slot] + (uint32_t)q; v < vend; v += kMergeLanes) {
            uint32_t b[P];
#pragma unroll
            for (int p = 0; p < P; ++p)
                b[p] = p < seg.planes ? seg.partial[((size_t)v * seg.planes + p) * W32 + w] : 0u;
            planes_add<P>(acc, b);
        }
    }
    // all lanes of the wavefront take part in the exchanges
#pragma unroll
    for (int d = kMergeLanes / 2; d >= 1; d >>= 1) {
        uint32_t b[P];
#pragma unroll
        for (int p = 0; p < P; ++p)
            b[p] = (uint32_t)__shfl_xor((int)acc[p], d);
        planes_add<P>(acc, b);
    }
    if (!active || q != 0)
        return;
    const uint32_t row = (uint32_t)order[slot];
    const uint32_t deg = rowptr[row + 1] - rowptr[row];
    if (EPI == BITGNN_EPI_THRESH_BITS) {
        uint32_t sd[P];
#pragma unroll
        for (int p = 0; p < P; ++p)
            sd[p] = seeds[((deg & 1u) * P + p) * W32 + w];
        planes_add<P>(acc, sd);
    }
    bspmm_epilogue<P, EPI>(acc, deg, row, w, W32, C, out, out_stride);
}

// Rows longer than a segment are split as in bspmm_kernel: a segment leaves its int32 sums
// in seg.partial ([segment][M]) and spmm_i32_long_rows_kernel adds a row's segments.
template <bool SCALE>
__global__ __launch_bounds__(kBlock) void spmm_i32_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, uint32_t N, const int32_t *__restrict__ Z, int32_t M,
    int64_t z_stride, const float *__restrict__ alpha, void *__restrict__ out,
    int64_t out_stride, int lpr_log2, RowSegments seg)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t v = t >> lpr_log2; // virtual row: a segment of a long row, or a whole row
    const int li = (int)(t & ((1u << lpr_log2) - 1u));
    if (v >= (uint64_t)seg.n_long_segs + (N - seg.n_long))
        return;
    const bool part = v < seg.n_long_segs;
    uint32_t slot, k = 0;
    if (part) {
        slot = seg.seg_slot[v];
        k = (uint32_t)v - seg.seg_ptr[slot];
    } else {
        slot = seg.n_long + (uint32_t)(v - seg.n_long_segs);
    }
    const uint32_t row = (uint32_t)order[slot];
    const uint32_t rend = rowptr[row + 1];
    const uint32_t beg = rowptr[row] + k * seg.seg_len;
    const uint32_t end = part && rend - beg > seg.seg_len ? beg + seg.seg_len : rend;
    for (int c = li; c < M; c += (1 << lpr_log2)) {
        int32_t sum = 0;
        // eight neighbours per turn: their indices, then their values, are in flight
        // together (clamped loads; integer sums do not depend on the order)
        for (uint32_t e = beg; e < end; e += 8) {
            int32_t j[8], z[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                j[u] = col[e + u < end ? e + u : end - 1];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                z[u] = Z[(int64_t)j[u] * z_stride + c];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                sum += e + u < end ? z[u] : 0;
        }
        if (part)
            ((int32_t *)seg.partial)[(size_t)v * M + c] = sum;
        else if (SCALE)
            ((float *)out)[(int64_t)row * out_stride + c] = alpha[c] * (float)sum;
        else
            ((int32_t *)out)[(int64_t)row * out_stride + c] = sum;
    }
}

// The same aggregation for wide rows (more than 32 channels) whose int32 rows can be read
// VW values per lane (16 or 8 bytes): one wavefront per virtual row, LR = M / VW lanes cover
// a neighbour's row, so one gather instruction fetches 64 / LR neighbours instead of one --
// the chip issues ~35 G wavefront-wide gathers per second whatever they carry, and a lane
// per channel spends one per neighbour.  The neighbour slots' sums are added across the
// lanes at the end (integer sums do not depend on the order).
template <bool SCALE, int VW>
__global__ __launch_bounds__(kBlock) void spmm_i32_wide_kernel(
    const uint32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ order, uint32_t N, const int32_t *__restrict__ Z, int32_t M,
    int64_t z_stride, const float *__restrict__ alpha, void *__restrict__ out,
    int64_t out_stride, RowSegments seg)
{
    typedef int32_t vec_t __attribute__((ext_vector_type(VW)));
    const int lane = threadIdx.x & 63;
    const uint64_t v = (uint64_t)blockIdx.x * (kBlock / 64) +
                       (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (v >= (uint64_t)seg.n_long_segs + (N - seg.n_long)) // wave-uniform
        return;
    const bool part = v < seg.n_long_segs;
    uint32_t slot, k = 0;
    if (part) {
        slot = seg.seg_slot[v];
        k = (uint32_t)v - seg.seg_ptr[slot];
    } else {
        slot = seg.n_long + (uint32_t)(v - seg.n_long_segs);
    }
    const uint32_t row = (uint32_t)order[slot];
    const uint32_t rend = rowptr[row + 1];
    const uint32_t beg = rowptr[row] + k * seg.seg_len;
    const uint32_t end = part && rend - beg > seg.seg_len ? beg + seg.seg_len : rend;
    const int LR = M / VW;  // lanes per neighbour row
    const int Q = 64 / LR;  // neighbour slots of the wavefront
    const int q = lane / LR, r = lane - q * LR;
    const bool has_slot = q < Q;
    vec_t acc = 0;
    for (uint32_t e0 = beg; e0 < end; e0 += 64) {
        const int cnt = end - e0 < 64u ? (int)(end - e0) : 64;
        const int32_t jl = col[e0 + (uint32_t)(lane < cnt ? lane : cnt - 1)];
        for (int t0 = 0; t0 < cnt; t0 += 4 * Q) {
            vec_t z[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { // clamped loads, masked below
                const int t = t0 + u * Q + q;
                const int32_t j = __shfl(jl, t < cnt ? t : cnt - 1, 64);
                z[u] = *(const vec_t *)(Z + (int64_t)j * z_stride + r * VW);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (has_slot && t0 + u * Q + q < cnt)
                    acc += z[u];
        }
    }
    // the slots' sums are folded in halves until slot 0 holds the total
    for (int active = Q; active > 1;) {
        const int half = (active + 1) / 2;
#pragma unroll
        for (int i = 0; i < VW; ++i) {
            const int32_t other = __shfl(acc[i], lane + half * LR, 64);
            if (q + half < active)
                acc[i] += other;
        }
        active = half;
    }
    if (q != 0)
        return;
#pragma unroll
    for (int i = 0; i < VW; ++i) {
        const int c = r * VW + i;
        if (part)
            ((int32_t *)seg.partial)[(size_t)v * M + c] = acc[i];
        else if (SCALE)
            ((float *)out)[(int64_t)row * out_stride + c] = alpha[c] * (float)acc[i];
        else
            ((int32_t *)out)[(int64_t)row * out_stride + c] = acc[i];
    }
}

template <bool SCALE>
__global__ __launch_bounds__(kBlock) void spmm_i32_long_rows_kernel(
    const int32_t *__restrict__ order, int32_t M, const float *__restrict__ alpha,
    void *__restrict__ out, int64_t out_stride, int lpr_log2, RowSegments seg)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t slot = t >> lpr_log2;
    const int li = (int)(t & ((1u << lpr_log2) - 1u));
    if (slot >= seg.n_long)
        return;
    const uint32_t row = (uint32_t)order[slot];
    for (int c = li; c < M; c += (1 << lpr_log2)) {
        int32_t sum = 0;
        const uint32_t vend = seg.seg_ptr[slot + 1];
        for (uint32_t v0 = seg.seg_ptr[slot]; v0 < vend; v0 += 8) { // eight loads in flight
            int32_t z[8];
#pragma unroll
            for (int q = 0; q < 8; ++q)
                z[q] = v0 + q < vend ? ((const int32_t *)seg.partial)[(size_t)(v0 + q) * M + c] : 0;
#pragma unroll
            for (int q = 0; q < 8; ++q)
                sum += z[q];
        }
        if (SCALE)
            ((float *)out)[(int64_t)row * out_stride + c] = alpha[c] * (float)sum;
        else
            ((int32_t *)out)[(int64_t)row * out_stride + c] = sum;
    }
}

// `col` and `h32` are either the caller's (node ids, node-ordered rows) or the slot ids
// and the degree-ordered compact copy of the rows.
template <int P>
void launch_bspmm_p(hipStream_t s, unsigned grid, int epilogue, const bitgnn_adj *adj,
                    const int32_t *col, const uint32_t *h32, int64_t h_stride32, int32_t C,
                    int32_t W32, const uint32_t *seeds, void *out, int64_t out_stride,
                    const RowSegments &seg)
{
    const unsigned grid_long =
        (unsigned)(((uint64_t)seg.n_long * (uint32_t)W32 * kMergeLanes + kBlock - 1) / kBlock);
    if (epilogue == BITGNN_EPI_THRESH_BITS) {
        bspmm_kernel<P, BITGNN_EPI_THRESH_BITS><<<grid, kBlock, 0, s>>>(
            adj->rowptr, col, adj->order, (uint32_t)adj->n, h32, h_stride32, C, W32, seeds, out,
            out_stride, seg);
        if (grid_long)
            bspmm_long_rows_kernel<P, BITGNN_EPI_THRESH_BITS><<<grid_long, kBlock, 0, s>>>(
                adj->rowptr, adj->order, C, W32, seeds, out, out_stride, seg);
    } else {
        bspmm_kernel<P, BITGNN_EPI_RAW_I32><<<grid, kBlock, 0, s>>>(
            adj->rowptr, col, adj->order, (uint32_t)adj->n, h32, h_stride32, C, W32, seeds, out,
            out_stride, seg);
        if (grid_long)
            bspmm_long_rows_kernel<P, BITGNN_EPI_RAW_I32><<<grid_long, kBlock, 0, s>>>(
                adj->rowptr, adj->order, C, W32, seeds, out, out_stride, seg);
    }
}

// rows in degree order, W32 words each, no padding
__global__ void csr_permute_kernel(const uint32_t *__restrict__ h32, int64_t h_stride32,
                                   const int32_t *__restrict__ order, uint32_t n, int32_t W32,
                                   uint32_t *__restrict__ hperm)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t slot = t / (uint32_t)W32;
    const int w = (int)(t - slot * (uint32_t)W32);
    if (slot < n)
        hperm[t] = h32[(int64_t)order[slot] * h_stride32 + w];
}


// ---------------------------------------------------------------------------
// LDS-staged variant for dense-enough graphs (format: adj_blocked.hip).
//
// A workgroup of 16 wavefronts walks the column blocks its slices touch.  For a
// block it copies the (degree-ordered) activation rows of the block's nodes into
// LDS with coalesced 16-byte accesses; then every lane streams the 16-bit local
// ids of ITS row part, lane-interleaved in memory (one 16-byte load = 8 ids),
// gathers the 16-byte rows from LDS and adds them into bit-sliced counters of
// 8 or 10 planes x 128 channels (parts never exceed 255 resp. 1023 entries).
// Each lane writes its partial planes; the merge kernel adds the parts of a
// node, applies the seed and the threshold (or unpacks the integers).

// Counter planes of a row part: 8 when parts have at most 255 entries (the partial
// planes of a part are then exactly one 128-byte line), else 10 (up to 1023 entries).
static int part_planes_for(const bitgnn_blocked *b) { return b->part_len <= 255 ? 8 : 10; }

constexpr int kPendLow = 3; // a block of 8 gathers produces one carry of weight 2^3
constexpr int kPendTop = 6; // levels 3..5 park a carry; above, carries ripple (rare)

// Adds a carry of weight 2^P0 into the counters.  Level p holds a parked carry iff
// bit (p - kPendLow) of blk (the number of 8-step blocks consumed so far): a binary
// counter, so the control flow is wave-uniform and every register index is static.
template <int P0, int PP>
__device__ __forceinline__ void blk_cascade(uint32_t (&acc)[PP][4], uint32_t (&pend)[PP][4],
                                            uint32_t (&carry)[4], uint32_t blk)
{
    if constexpr (P0 < kPendTop) {
        if (!((blk >> (P0 - kPendLow)) & 1u)) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                pend[P0][q] = carry[q];
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t nc;
                csa(acc[P0][q], pend[P0][q], carry[q], nc);
                carry[q] = nc;
            }
            blk_cascade<P0 + 1, PP>(acc, pend, carry, blk);
        }
    } else {
        // ripple the carry through the upper planes (once per 2^(kPendTop-kPendLow) blocks)
#pragma unroll
        for (int p = kPendTop; p < PP; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t nc = acc[p][q] & carry[q];
                acc[p][q] ^= carry[q];
                carry[q] = nc;
            }
    }
}

// Weights of the class projection as +-1 bytes, one 128-channel window of one class per
// call (threads t < 128 of a workgroup; all threads of the workgroup must call), and the
// column sums of the window.
__device__ __forceinline__ void project_weights_entry(int c, int win, int t,
                                                      const uint32_t *__restrict__ w32,
                                                      int64_t w_stride32, int32_t K, int32_t M,
                                                      int32_t Mpad, int8_t *__restrict__ w8,
                                                      int32_t *__restrict__ wsum)
{
    const int k = win * 128 + t;
    int v = 0;
    if (t < 128 && c < M && k < K)
        v = ((w32[(int64_t)c * w_stride32 + (k >> 5)] >> (k & 31)) & 1u) ? 1 : -1;
    if (t < 128)
        w8[((int64_t)win * Mpad + c) * 128 + t] = (int8_t)v;
    // column sum: two wavefronts, combined through LDS
    __shared__ int part[2];
    int sum = v;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1)
        sum += __shfl_xor(sum, d, 64);
    if (t < 128 && (t & 63) == 0)
        part[t >> 6] = sum;
    __syncthreads();
    if (t == 0)
        wsum[win * Mpad + c] = part[0] + part[1];
}

// Set-up work that rides along with the first permute launch of a call instead of taking
// a launch of its own: the threshold seeds of the merge, or the projection's weights.
struct PermuteAux {
    int kind; // 0 none, 1 seeds, 2 projection weights
    // seeds: of the merge (P planes) and of the rows the aggregation kernel finishes itself
    // (PF planes; 0: none)
    const int32_t *T;
    int32_t C, W32, P, PF;
    uint32_t *table, *table_fin;
    // projection weights
    const uint32_t *w32;
    int64_t w_stride32;
    int32_t K, M, Mpad, nwin;
    int8_t *w8;
    int32_t *wsum;
};

// Activation rows in degree order (one 128-channel window); also rewinds the work
// counter of the aggregation kernel that follows on the same stream.
__global__ __launch_bounds__(256) void blk_permute_kernel(
    const uint32_t *__restrict__ h32, int64_t h_stride32, const int32_t *__restrict__ order,
    uint32_t n, int w0, int W32, uint4 *__restrict__ hperm, uint32_t *__restrict__ queue,
    uint32_t permute_blocks, PermuteAux aux)
{
    if (blockIdx.x >= permute_blocks) { // workgroup-uniform: the set-up work's own workgroups
        const int vb = (int)(blockIdx.x - permute_blocks);
        if (aux.kind == 1) {
            // 32 threads per table word: first the merge's table, then (wavefronts of
            // their own: the word counts are even) the finished rows' table
            const int t = vb * 256 + (int)threadIdx.x, n_merge = 2 * aux.P * aux.W32;
            if (t < n_merge * 32) // uniform over a wavefront
                seed_word_vote(t, n_merge, aux.T, aux.C, aux.W32, aux.P, aux.table);
            else if (aux.PF)
                seed_word_vote(t - n_merge * 32, 2 * aux.PF * aux.W32, aux.T, aux.C, aux.W32,
                               aux.PF, aux.table_fin);
        } else if (aux.kind == 2)
            project_weights_entry(vb % aux.Mpad, vb / aux.Mpad, (int)threadIdx.x, aux.w32,
                                  aux.w_stride32, aux.K, aux.M, aux.Mpad, aux.w8, aux.wsum);
        return;
    }
    const uint32_t slot = blockIdx.x * blockDim.x + threadIdx.x;
    if (slot == 0)
        *queue = 0u;
    if (slot >= n)
        return;
    const uint32_t *r = h32 + (int64_t)order[slot] * h_stride32;
    uint4 v;
    v.x = w0 + 0 < W32 ? r[w0 + 0] : 0u;
    v.y = w0 + 1 < W32 ? r[w0 + 1] : 0u;
    v.z = w0 + 2 < W32 ? r[w0 + 2] : 0u;
    v.w = w0 + 3 < W32 ? r[w0 + 3] : 0u;
    hperm[slot] = v;
}

// One block of 8 steps: gathers of 16-byte rows from LDS, added into the bit-sliced
// counters through a carry-save tree (7 adders per 8 inputs and 32-channel word).
template <int PP>
__device__ __forceinline__ void blk_consume(const uint32_t (&id)[8], const uint4 *hblk,
                                            uint32_t (&acc)[PP][4], uint32_t (&pend)[PP][4],
                                            uint32_t blk)
{
    uint32_t x[8][4];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint4 v = hblk[id[k]];
        x[k][0] = v.x;
        x[k][1] = v.y;
        x[k][2] = v.z;
        x[k][3] = v.w;
    }
    uint32_t carry[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t t0, t1, t2, t3, f0, f1;
        csa(acc[0][q], x[0][q], x[1][q], t0);
        csa(acc[0][q], x[2][q], x[3][q], t1);
        csa(acc[0][q], x[4][q], x[5][q], t2);
        csa(acc[0][q], x[6][q], x[7][q], t3);
        csa(acc[1][q], t0, t1, f0);
        csa(acc[1][q], t2, t3, f1);
        csa(acc[2][q], f0, f1, carry[q]); // weight 8
    }
    blk_cascade<kPendLow, PP>(acc, pend, carry, blk);
}

#ifdef BITGNN_PROFILE
__device__ unsigned long long *g_blk_prof = nullptr; // per workgroup: start, end, fill, compute
#define BLK_PROF_T() ((tid == 0) ? clock64() : 0)
#endif

// The 16-bit ids of one lane for one group: kGroupSteps / 2 dwords, one vector load each.
struct blk_ids {
    uint32_t w[kGroupSteps / 2];
};
// The id array is smaller than 4 GiB (checked when the format is built), so a group
// is addressed as uniform base + 32-bit byte offset.
__device__ __forceinline__ blk_ids blk_load_ids(const uint32_t *__restrict__ idx, uint32_t g,
                                                int lane)
{
    const uint32_t byte = (g * 64u + (uint32_t)lane) * (uint32_t)(kGroupSteps * 2);
    const uint4 *p = (const uint4 *)((const char *)idx + byte);
    blk_ids r;
#pragma unroll
    for (int j = 0; j < kGroupSteps / 8; ++j) {
        // read once: marked non-temporal so that the stream does not push the
        // activation rows out of L2
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p + j);
        r.w[4 * j + 0] = v.x;
        r.w[4 * j + 1] = v.y;
        r.w[4 * j + 2] = v.z;
        r.w[4 * j + 3] = v.w;
    }
    return r;
}

// What a wavefront needs to know of a work item (all wave-uniform).
struct blk_item {
    uint32_t wlo, whi;   // column blocks the workgroup walks
    uint32_t mylo, myhi; // column blocks of this wavefront's slice (mylo > myhi: none)
    uint32_t t0, g;      // first tile, first group of the slice's id stream
    uint32_t slice;
    bool has;
};
__device__ __forceinline__ blk_item blk_item_of(uint2 it, uint4 d, uint32_t slice, bool has)
{
    blk_item r;
    r.wlo = it.y & 0xFFFFu;
    r.whi = it.y >> 16;
    r.mylo = has ? (d.x & 0xFFFFu) : 1u;
    r.myhi = has ? (d.x >> 16) : 0u;
    r.t0 = has ? d.y : 0u;
    r.g = has ? d.z : 0u;
    r.slice = slice;
    r.has = has;
    return r;
}

// A workgroup barrier that orders LDS accesses only (no wait for global loads or stores in
// flight).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// What the kernel needs to finish rows that consist of a single part itself (threshold
// epilogue only): such a row's count is complete in the lane, so it is compared and stored
// there and then (Algorithm 1's final test and store) and never travels as partial planes.
struct BlkFinish {
    int enabled;
    const int32_t *deg;     // [n] by node id
    const uint32_t *seeds;  // [2][PP + 2][W32] threshold seeds of the part counters
    void *out;              // packed output rows
    int64_t out_stride;     // in 64-bit words
    int32_t C, W32, win;
};

// Launched with one workgroup per compute unit (its LDS block leaves room for one
// only).  Every workgroup takes work items (kSlicesPerWg slices each, heaviest first)
// from an atomic counter until the list is exhausted: a compute unit that finishes
// early picks up more work whatever the hardware's dispatch order is, and no time is
// lost to launching workgroups in the middle of the kernel.  The next item is drawn
// while the last block of the current one is processed (late enough to go to whichever
// workgroup is about to be free), and its descriptors and first ids are requested
// step by step behind the barriers of that block, so the switch costs no round trip.
// SPW: slices (wavefronts) per work item and workgroup.
template <int PP, int SPW>
__global__ __launch_bounds__(64 * SPW) void bspmm_blk_kernel(
    const uint4 *__restrict__ hperm, uint32_t n, uint32_t cbn, const uint2 *__restrict__ wg_item,
    const uint4 *__restrict__ sl_desc, const uint32_t *__restrict__ tile_group,
    const uint32_t *__restrict__ idx, const uint2 *__restrict__ part_info, uint32_t S,
    uint32_t V, uint32_t n_items, uint32_t *__restrict__ queue, uint4 *__restrict__ partial,
    BlkFinish fin)
{
    extern __shared__ uint4 hblk[]; // cbn rows + 16 all-zero rows (one per bank group)
    __shared__ uint32_t s_next;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the block buffer (without its zero rows) can stage every wavefront's partial planes,
    // 64 x 8 x 16 bytes each
    const bool stage_ok = cbn >= (uint32_t)SPW * 64u * 8u;
    if (tid < 16)
        hblk[cbn + tid] = make_uint4(0u, 0u, 0u, 0u);
    if (tid == 0)
        s_next = atomicAdd(queue, 1u);
    __syncthreads();
    uint32_t cur = s_next;
    if (cur >= n_items) // uniform over the workgroup
        return;
    blk_item it;
    {
        const uint2 w = wg_item[cur];
        const uint32_t slice = w.x * SPW + wave;
        const bool has = slice < S;
        it = blk_item_of(w, sl_desc[has ? slice : 0u], slice, has);
    }
    // The groups of a slice are one contiguous stream: group g + 1 is requested
    // while group g is consumed, across tile boundaries and LDS refills alike.
    // Reading one group past the stream's end is in bounds (padding group).
    blk_ids nxt = blk_load_ids(idx, it.g, lane);

    for (;;) { // one work item per turn; every wavefront of the workgroup leaves together
        __syncthreads(); // everyone has read s_next
        uint32_t g = it.g;
        const uint32_t pos = it.slice * 64 + lane;
        const bool writes = it.has && pos < V;
        const uint2 pinfo = part_info[writes ? pos : 0u]; // needed at the end only
        const uint32_t vid = pinfo.x & 0x3FFFFFFFu;
        const bool single = fin.enabled && (pinfo.x >> 31);
        // degree of a row this lane finishes itself (requested now, used at the end)
        const uint32_t fdeg = (writes && single) ? (uint32_t)fin.deg[pinfo.y] : 0u;
        uint32_t acc[PP][4], pend[PP][4];
#pragma unroll
        for (int p = 0; p < PP; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[p][q] = 0u;
                pend[p][q] = 0u;
            }
        uint32_t blk = 0; // blocks of 8 steps consumed by this wavefront
        uint32_t nx = 0;  // the item after this one
        uint2 nw = make_uint2(0u, 0u);
        uint4 nd = make_uint4(0u, 0u, 0u, 0u);
        uint32_t nslice = 0;
        bool nhas = false;
#ifdef BITGNN_PROFILE
        const long long p_start = BLK_PROF_T();
        const unsigned long long p_wall0 = (tid == 0) ? wall_clock64() : 0;
        long long p_fill = 0, p_comp = 0, p_t0 = p_start;
#endif

        for (uint32_t cb = it.wlo; cb <= it.whi; ++cb) {
            // end of this tile's groups: requested before the refill so that the scalar
            // load's latency hides behind it
            const bool mine = cb >= it.mylo && cb <= it.myhi; // wave-uniform
            const bool last = cb == it.whi;
            const uint32_t g1 = tile_group[mine ? it.t0 + cb - it.mylo + 1 : 0u];
            if (last && tid == 0)
                s_next = atomicAdd(queue, 1u);
            __syncthreads(); // all wavefronts are done with the previous block
#ifdef BITGNN_PROFILE
            { const long long t = BLK_PROF_T(); p_comp += t - p_t0; p_t0 = t; }
#endif
            if (last) { // the drawn number is visible now: first descriptor of the next item
                nx = s_next;
                nw = wg_item[nx < n_items ? nx : n_items - 1];
            }
            const uint32_t base = cb * cbn;
            const uint32_t rows = n - base < cbn ? n - base : cbn;
            // A wavefront copies 64 consecutive rows per instruction, straight from L2 into
            // LDS (no register round trip); the ragged end of the last block goes row by row.
#pragma unroll
            for (int k = 0; k < (kMaxCbNodes + 64 * SPW - 1) / (64 * SPW); ++k) {
                const uint32_t w0 = (uint32_t)wave * 64u + (uint32_t)k * (64u * SPW); // uniform
                if (w0 + 64u <= rows) {
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(hperm + base + w0 + lane),
                        (__attribute__((address_space(3))) void *)(hblk + w0), 16, 0, 0);
                } else if (w0 + lane < rows) {
                    hblk[w0 + lane] = hperm[base + w0 + lane];
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // the copies have landed
            __syncthreads();
#ifdef BITGNN_PROFILE
            { const long long t = BLK_PROF_T(); p_fill += t - p_t0; p_t0 = t; }
#endif
            if (last) { // second descriptor of the next item
                nslice = nw.x * SPW + wave;
                nhas = nslice < S;
                nd = sl_desc[nhas ? nslice : 0u];
            }
            if (mine) {
                for (; g < g1; ++g) {
                    // Unpack the ids first and pin them in registers: after that
                    // `nxt` is dead, the next request reuses its registers without a copy,
                    // and the wait for it moves to the top of the next iteration.
                    uint32_t id[kGroupSteps / 8][8];
#pragma unroll
                    for (int j = 0; j < kGroupSteps / 2; ++j) {
                        id[j / 4][2 * (j % 4)] = nxt.w[j] & 0xFFFFu;
                        id[j / 4][2 * (j % 4) + 1] = nxt.w[j] >> 16;
                    }
#pragma unroll
                    for (int j = 0; j < kGroupSteps; ++j)
                        asm volatile("" : "+v"(id[j / 8][j % 8]) : : "memory");
                    nxt = blk_load_ids(idx, g + 1, lane);
#pragma unroll
                    for (int j = 0; j < kGroupSteps / 8; ++j) {
                        blk_consume<PP>(id[j], hblk, acc, pend, blk);
                        ++blk;
                    }
                }
            }
        }
        // first ids of the next item (the old `nxt` is one group past this item's stream)
        const blk_item nit = blk_item_of(nw, nd, nslice, nhas);
        nxt = blk_load_ids(idx, nit.g, lane);

#ifdef BITGNN_PROFILE
        __syncthreads();
        if (tid == 0 && g_blk_prof) {
            const long long t = clock64();
            p_comp += t - p_t0;
            unsigned long long *o = g_blk_prof + 8ull * cur;
            o[0] = p_start; o[1] = t; o[2] = p_fill; o[3] = p_comp;
            o[4] = p_wall0; o[5] = wall_clock64(); o[6] = __smid();
            o[7] = __builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (3 << 11)); /* XCC_ID */
        }
#endif
        // fold the parked carries: planes become an ordinary binary number
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t carry = 0;
#pragma unroll
            for (int p = kPendLow; p < PP; ++p) {
                const uint32_t pd =
                    (p < kPendTop && ((blk >> (p - kPendLow)) & 1u)) ? pend[p][q] : 0u;
                uint32_t nc;
                csa(acc[p][q], pd, carry, nc);
                carry = nc;
            }
        }
        // A row that is one part is complete here: add the threshold seed, compare, store
        // the packed bits (its count fits PP planes, the seeded count PP + 2).
        if (writes && single) {
            constexpr int PF = PP + 2;
            const uint32_t row = pinfo.y;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int w = fin.win * 4 + q;
                if (w < fin.W32) {
                    uint32_t a[PF], sd[PF];
#pragma unroll
                    for (int p = 0; p < PF; ++p) {
                        a[p] = p < PP ? acc[p < PP ? p : 0][q] : 0u;
                        sd[p] = fin.seeds[((fdeg & 1u) * PF + p) * fin.W32 + w];
                    }
                    planes_add<PF>(a, sd);
                    bspmm_epilogue<PF, BITGNN_EPI_THRESH_BITS>(a, fdeg, row, w, fin.W32, fin.C,
                                                               fin.out, fin.out_stride);
                }
            }
        }
        const bool stores = writes && !single;
        // Partial planes are filed under the part id, so that the merge reads the parts of
        // a row, and of consecutive rows, back to back.  A lane storing its own 8 planes
        // would touch 64 different 128-byte lines with every store instruction; instead the
        // wavefront turns its 64 x 8 planes around in LDS (the block buffer is free once
        // everyone is done gathering) so that 8 adjacent lanes store one part's whole line.
        if (PP == 8 && stage_ok) {
            lds_barrier();
            uint4 *stage = hblk + (uint32_t)wave * (64 * PP);
#pragma unroll
            for (int p = 0; p < PP; ++p)
                stage[lane * PP + p] = make_uint4(acc[p][0], acc[p][1], acc[p][2], acc[p][3]);
            // (a wavefront reads back only what it wrote itself: no barrier)
#pragma unroll 1
            for (int r = 0; r < 64 * PP / 64; ++r) {
                const int src = r * (64 / PP) + lane / PP; // the part whose line this lane helps store
                const uint4 v = stage[src * PP + lane % PP];
                const uint32_t svid = (uint32_t)__shfl((int)vid, src, 64);
                const int swr = __shfl((int)stores, src, 64);
                if (swr)
                    partial[(uint64_t)svid * PP + lane % PP] = v;
            }
        } else if (stores) {
#pragma unroll
            for (int p = 0; p < PP; ++p)
                partial[(uint64_t)vid * PP + p] =
                    make_uint4(acc[p][0], acc[p][1], acc[p][2], acc[p][3]);
        }
        cur = nx; // read behind the first barrier of the last block: uniform
        if (cur >= n_items)
            break;
        it = nit;
    }
}

// Adds the partial planes of the parts [v0, v1) of one node (word q) into acc.  Two parts
// are requested per turn (the second address is clamped, so no load is conditional):
// most nodes have at most a few parts, and the loads of a turn travel together.
template <int P, int PP>
__device__ __forceinline__ void add_parts(uint32_t (&acc)[P], const uint32_t *__restrict__ partial32,
                                          uint32_t v0, uint32_t v1, int q)
{
    constexpr int kAdd = P < PP ? P : PP; // planes a part can fill
    for (uint32_t v = v0; v < v1; v += 2) {
        const bool two = v + 1 < v1; // lane-varying: handled by masking, not by branching
        const uint32_t *pa = partial32 + ((uint64_t)v * PP) * 4 + q;
        const uint32_t *pb = partial32 + ((uint64_t)(two ? v + 1 : v) * PP) * 4 + q;
        uint32_t a[kAdd], b[kAdd];
#pragma unroll
        for (int p = 0; p < kAdd; ++p) {
            a[p] = pa[p * 4];
            b[p] = pb[p * 4];
        }
        const uint32_t keep = two ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int h = 0; h < 2; ++h) { // acc += a, then acc += b (or 0)
            uint32_t carry = 0;
#pragma unroll
            for (int p = 0; p < kAdd; ++p) {
                uint32_t nc;
                csa(acc[p], h == 0 ? a[p] : (b[p] & keep), carry, nc);
                carry = nc;
            }
#pragma unroll
            for (int p = kAdd; p < P; ++p) {
                const uint32_t nc = acc[p] & carry;
                acc[p] ^= carry;
                carry = nc;
            }
        }
    }
}

// 4 lanes per node (one per 32-channel word of the window): sum the node's parts.
template <int P, int EPI, int PP>
__global__ __launch_bounds__(kBlock) void bspmm_merge_kernel(
    const uint32_t *__restrict__ partial32, const uint32_t *__restrict__ row_vptr,
    const int32_t *__restrict__ order,
    const int32_t *__restrict__ deg, uint32_t n, int win, int32_t C, int32_t W32,
    const uint32_t *__restrict__ seeds, void *__restrict__ out, int64_t out_stride)
{
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t slot = t >> 2;
    const int q = t & 3;
    const int w = win * 4 + q;
    if (slot >= n || w >= W32)
        return;
    const uint32_t row = (uint32_t)order[slot];
    const uint32_t d = (uint32_t)deg[row];
    uint32_t acc[P];
#pragma unroll
    for (int p = 0; p < P; ++p)
        acc[p] = (EPI == BITGNN_EPI_THRESH_BITS) ? seeds[((d & 1u) * P + p) * W32 + w] : 0u;
    add_parts<P, PP>(acc, partial32, row_vptr[slot], row_vptr[slot + 1], q);
    bspmm_epilogue<P, EPI>(acc, d, row, w, W32, C, out, out_stride);
}

// Output layer in aggregate-then-transform order, fused with the merge:
//   logits[i][c] = alpha[c] * sum_k S[i][k] * w[k][c],  S = 2 cnt - deg  (K <= 128)
// which equals the paper's MM.BBF + BSpMM.FBF order exactly in integers because no
// non-linearity sits between the two products.  With wsum_c = sum_k w[k][c],
//   sum_k S_k w_kc = 2 sum_k cnt_k w_kc - deg wsum_c,
// and sum_k cnt_k w_kc is a small dense integer contraction (nodes x K x classes): it runs
// on the matrix cores.  The bit-sliced counts of a node are turned into 7-bit digits
// (base 128, so every digit is a non-negative int8) by 8x8 bit transposes, the weights
// are +-1 bytes (0 beyond K or M), and one v_mfma_i32_16x16x32_i8 per digit, class tile
// and 32-channel word accumulates 16 nodes x 16 classes.  The digits recombine by shifts.
//
// Lane roles in a wavefront of 16 nodes:
//   merge:  lane = node * 4 + word   (sums the node's parts, as the plain merge does)
//   digits: lane = node + 16 * g     (8 channels 8g..8g+7 of every word: the B operand)
//   result: lane = node + 16 * g     holds classes 16 tile + 4 g + (0..3)
typedef int v4i __attribute__((ext_vector_type(4)));

// 8x8 bit transpose of the 64-bit matrix (hi:lo), row r = byte r: three delta swaps.
__device__ __forceinline__ void transpose8x8(uint32_t &lo, uint32_t &hi)
{
    uint32_t t;
    t = (lo ^ (lo >> 7)) & 0x00AA00AAu;
    lo ^= t ^ (t << 7);
    t = (hi ^ (hi >> 7)) & 0x00AA00AAu;
    hi ^= t ^ (t << 7);
    t = (lo ^ (lo >> 14)) & 0x0000CCCCu;
    lo ^= t ^ (t << 14);
    t = (hi ^ (hi >> 14)) & 0x0000CCCCu;
    hi ^= t ^ (t << 14);
    t = (lo ^ ((lo >> 28) | (hi << 4))) & 0xF0F0F0F0u; // 64-bit shift by 28, low half
    lo ^= t;
    hi ^= t >> 4; // (t << 28) lands in the high half only: t has no bits below bit 4
}

constexpr int kProjWaves = 4;     // wavefronts per workgroup, 16 nodes each
constexpr int kProjTiles = 4;     // class tiles of 16 per pass (64 classes)

template <int NB, int PP> // digits of 7 bits: max degree < 2^(7 NB)
__global__ __launch_bounds__(kProjWaves * 64, NB <= 2 ? 8 : 4) void bspmm_merge_project_kernel(
    const uint32_t *__restrict__ partial32, const uint32_t *__restrict__ row_vptr,
    const int32_t *__restrict__ order,
    const int32_t *__restrict__ deg, uint32_t n, int32_t W32, const int8_t *__restrict__ w8,
    const int32_t *__restrict__ wsum, int32_t M, const float *__restrict__ alpha,
    float *__restrict__ out, int64_t ldo, int32_t *__restrict__ ysum, bool has_prev,
    bool is_last)
{
    // K > 128 comes in windows of 128 channels, one call each: the integer sums of the
    // windows are chained through ysum[n][M] (has_prev: add it; !is_last: store there),
    // the last call scales and writes the logits.
    constexpr int P = 7 * NB;
    // per wavefront: first the merged planes [node][word][plane], later (same memory, the
    // planes are consumed by then and the region is private to the wavefront) the logits
    // [node][class] on their way out
    constexpr int kPlaneWords = 16 * 4 * (P + 1), kOutWords = 16 * (kProjTiles * 16 + 1);
    __shared__ uint32_t s_buf[kProjWaves][kPlaneWords > kOutWords ? kPlaneWords : kOutWords];
    __shared__ int32_t s_deg[kProjWaves][16];
    __shared__ uint32_t s_row[kProjWaves][16];
    __shared__ int32_t s_wsum[kProjTiles * 16];
    __shared__ float s_alpha[kProjTiles * 16];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const uint32_t slot0 = (blockIdx.x * kProjWaves + wave) * 16;
    // per-class constants and weight operands of the first 64 classes: requested before the
    // parts are merged, so that their latency hides behind that
    if (threadIdx.x < kProjTiles * 16) {
        const int c = threadIdx.x;
        s_wsum[c] = c < M ? wsum[c] : 0;
        s_alpha[c] = c < M ? alpha[c] : 0.0f;
    }

    // --- merge the parts of 16 nodes (lane = node * 4 + word)
    {
        const int node = lane >> 2, q = lane & 3;
        const uint32_t slot_raw = slot0 + node;
        const bool live = slot_raw < n;
        const uint32_t slot = live ? slot_raw : 0u;
        const uint32_t row = (uint32_t)order[slot];
        uint32_t acc[P];
#pragma unroll
        for (int p = 0; p < P; ++p)
            acc[p] = 0u;
        if (live && q < W32)
            add_parts<P, PP>(acc, partial32, row_vptr[slot], row_vptr[slot + 1], q);
#pragma unroll
        for (int p = 0; p < P; ++p)
            s_buf[wave][(node * 4 + q) * (P + 1) + p] = acc[p];
        if (q == 0) {
            s_deg[wave][node] = live ? deg[row] : 0;
            s_row[wave][node] = live ? row : 0xFFFFFFFFu;
        }
    }
    __syncthreads();

    // --- digits (lane = node + 16 g): B operands, 8 channels x NB digits per word
    const int nd = lane & 15, g = lane >> 4;
    // weight operands of one class tile at a time (the next tile's are requested while this
    // one's products run): holding all four tiles cost 32 registers and half the occupancy
    long aop[4];
#pragma unroll
    for (int w = 0; w < 4; ++w)
        aop[w] = *(const long *)(w8 + (int64_t)nd * 128 + 8 * g + 32 * w);
    long bop[4][NB];
    {
        const uint32_t sel01 = (uint32_t)g | ((uint32_t)(4 + g) << 8) | 0x0C0C0000u;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint32_t *pl = &s_buf[wave][(nd * 4 + w) * (P + 1) + 7 * b];
                // byte g of planes 7b .. 7b+6: rows of an 8x8 bit matrix (row 7 is zero)
                const uint32_t h01 = __builtin_amdgcn_perm(pl[1], pl[0], sel01);
                const uint32_t h23 = __builtin_amdgcn_perm(pl[3], pl[2], sel01);
                const uint32_t h45 = __builtin_amdgcn_perm(pl[5], pl[4], sel01);
                const uint32_t h6 = (pl[6] >> (8 * g)) & 0xFFu;
                uint32_t lo = __builtin_amdgcn_perm(h23, h01, 0x05040100u);
                uint32_t hi = __builtin_amdgcn_perm(h6, h45, 0x05040100u);
                transpose8x8(lo, hi); // now byte j = the digit of channel 8g + j
                bop[w][b] = (long)(((uint64_t)hi << 32) | lo);
            }
    }
    const int32_t d_nd = s_deg[wave][nd];

    // --- contraction with the class weights, 64 classes per pass
    for (int c0 = 0; c0 < M; c0 += kProjTiles * 16) {
        if (c0 > 0) { // later passes: constants and first operands of these 64 classes
            __syncthreads(); // the previous pass has read s_wsum / s_alpha / s_out
            if (threadIdx.x < kProjTiles * 16) {
                const int c = c0 + threadIdx.x;
                s_wsum[threadIdx.x] = c < M ? wsum[c] : 0;
                s_alpha[threadIdx.x] = c < M ? alpha[c] : 0.0f;
            }
#pragma unroll
            for (int w = 0; w < 4; ++w)
                aop[w] = *(const long *)(w8 + (int64_t)(c0 + nd) * 128 + 8 * g + 32 * w);
            __syncthreads();
        }
#pragma unroll 1
        for (int t = 0; t < kProjTiles; ++t) {
            if (c0 + t * 16 >= M) // wave-uniform
                break;
            long nop[4];
            {
                // rows of w8 are padded to a multiple of 16 classes; past the last tile the
                // first tile is read again and not used
                const bool more = t + 1 < kProjTiles && c0 + (t + 1) * 16 < M;
                const int nrow = more ? c0 + (t + 1) * 16 + nd : nd;
#pragma unroll
                for (int w = 0; w < 4; ++w)
                    nop[w] = *(const long *)(w8 + (int64_t)nrow * 128 + 8 * g + 32 * w);
            }
            v4i acc[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b)
                acc[b] = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                if (w < W32) {
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        acc[b] = __builtin_amdgcn_mfma_i32_16x16x32_i8(aop[w], bop[w][b], acc[b], 0,
                                                                       0, 0);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int cl = t * 16 + 4 * g + j;
                int32_t val = 0;
#pragma unroll
                for (int b = NB - 1; b >= 0; --b)
                    val = (val << 7) + acc[b][j];
                s_buf[wave][nd * (kProjTiles * 16 + 1) + cl] =
                    (uint32_t)(2 * val - d_nd * s_wsum[cl]);
            }
#pragma unroll
            for (int w = 0; w < 4; ++w)
                aop[w] = nop[w];
        }
        __syncthreads();
        const int ncls = M - c0 < kProjTiles * 16 ? M - c0 : kProjTiles * 16;
        for (int node = 0; node < 16; ++node) {
            const uint32_t row = s_row[wave][node];
            if (row != 0xFFFFFFFFu && lane < ncls) {
                int32_t y = (int32_t)s_buf[wave][node * (kProjTiles * 16 + 1) + lane];
                if (has_prev)
                    y += ysum[(int64_t)row * M + c0 + lane];
                if (is_last)
                    out[(int64_t)row * ldo + c0 + lane] = s_alpha[lane] * (float)y;
                else
                    ysum[(int64_t)row * M + c0 + lane] = y;
            }
        }
    }
}

// Merges the parts of the first `rows` rows in degree order (all rows, or only those of
// several parts when the aggregation kernel finished the others itself).
template <int P, int PP>
void launch_merge_pp(hipStream_t s, int epilogue, const bitgnn_adj *adj, const uint32_t *partial32,
                     uint32_t rows, int win, int32_t C, int32_t W32, const uint32_t *seeds,
                     void *out, int64_t out_stride)
{
    const bitgnn_blocked *b = adj->blk;
    const unsigned grid = (unsigned)(((uint64_t)rows * 4 + kBlock - 1) / kBlock);
    if (grid == 0)
        return;
    if (epilogue == BITGNN_EPI_THRESH_BITS)
        bspmm_merge_kernel<P, BITGNN_EPI_THRESH_BITS, PP><<<grid, kBlock, 0, s>>>(
            partial32, b->row_vptr, adj->order, adj->deg, rows, win, C, W32, seeds, out,
            out_stride);
    else
        bspmm_merge_kernel<P, BITGNN_EPI_RAW_I32, PP><<<grid, kBlock, 0, s>>>(
            partial32, b->row_vptr, adj->order, adj->deg, rows, win, C, W32, seeds, out,
            out_stride);
}

template <int P>
void launch_merge_p(hipStream_t s, int epilogue, const bitgnn_adj *adj, const uint32_t *partial32,
                    uint32_t rows, int win, int32_t C, int32_t W32, const uint32_t *seeds,
                    void *out, int64_t out_stride)
{
    if (part_planes_for(adj->blk) == 8)
        launch_merge_pp<P, 8>(s, epilogue, adj, partial32, rows, win, C, W32, seeds, out,
                              out_stride);
    else
        launch_merge_pp<P, 10>(s, epilogue, adj, partial32, rows, win, C, W32, seeds, out,
                               out_stride);
}

// The aggregation kernel proper; `partial` receives PP planes of 16 bytes per part.
static int launch_blk(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const uint4 *hperm,
                      uint4 *partial, const BlkFinish &fin)
{
    const bitgnn_blocked *b = adj->blk;
    const size_t lds = ((size_t)b->cbn + 16) * 16;
    const uint32_t cus = ctx->n_cus > 0 ? (uint32_t)ctx->n_cus : 256u;
    const unsigned grid = b->n_wgs < cus ? b->n_wgs : cus;
#define BG_BLK(PPV, SPWV)                                                                         \
    do {                                                                                          \
        BG_HIP(ctx, hipFuncSetAttribute((const void *)bspmm_blk_kernel<PPV, SPWV>,                \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));   \
        bg_time_begin(ctx, s);                                                                    \
        bspmm_blk_kernel<PPV, SPWV><<<grid, 64 * SPWV, lds, s>>>(                                 \
            hperm, (uint32_t)adj->n, (uint32_t)b->cbn, b->wg_item, b->sl_desc, b->tile_group,     \
            (const uint32_t *)b->idx16, b->part_info, b->n_slices, b->n_vrows, b->n_wgs,          \
            ctx->sc->queue, partial, fin);                                                        \
        bg_time_end(ctx, s);                                                                      \
    } while (0)
#define BG_BLK_SPW(PPV)                                                                           \
    do {                                                                                          \
        if (b->spw == 16)                                                                         \
            BG_BLK(PPV, 16);                                                                      \
        else if (b->spw == 8)                                                                     \
            BG_BLK(PPV, 8);                                                                       \
        else                                                                                      \
            BG_BLK(PPV, 4);                                                                       \
    } while (0)
    if (part_planes_for(b) == 8)
        BG_BLK_SPW(8);
    else
        BG_BLK_SPW(10);
#undef BG_BLK_SPW
#undef BG_BLK
    BG_LAUNCH_CHECK(ctx, "bspmm_blk");
    return BITGNN_OK;
}

} // namespace

#ifdef BITGNN_PROFILE
extern "C" int bitgnn_debug_set_blk_profile(unsigned long long *buf)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_blk_prof), &buf, sizeof(buf));
}
#endif

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

// Counter planes: need max_degree < 2^(P-2).  One of 12, 16, 20, 26.
static int planes_for(const bitgnn_adj *adj)
{
    int P = 12;
    while ((1ll << (P - 2)) <= adj->max_degree)
        P += (P == 20) ? 6 : 4;
    return P;
}

// Permute launch of one 128-channel window; `aux` (first window only) adds the workgroups
// of the call's set-up work.
static void launch_permute(hipStream_t s, const bitgnn_adj *adj, const uint32_t *h32,
                           int64_t h_stride32, int w0, int W32, uint4 *hperm, uint32_t *queue,
                           const PermuteAux &aux)
{
    const unsigned pb = (unsigned)((adj->n + 255) / 256);
    unsigned extra = 0;
    if (aux.kind == 1)
        extra = (unsigned)((2 * (aux.P + aux.PF) * aux.W32 * 32 + 255) / 256);
    else if (aux.kind == 2)
        extra = (unsigned)(aux.Mpad * aux.nwin);
    blk_permute_kernel<<<pb + extra, 256, 0, s>>>(h32, h_stride32, adj->order, (uint32_t)adj->n, w0,
                                                  W32, hperm, queue, pb, aux);
}

static int launch_seeds(bitgnn_ctx *ctx, hipStream_t s, int epilogue, const int32_t *T, int32_t C,
                        int32_t W32, int P, const uint32_t **seeds)
{
    *seeds = nullptr;
    if (epilogue != BITGNN_EPI_THRESH_BITS)
        return BITGNN_OK;
    const int entries = 2 * P * W32;
    BG_REQUIRE(ctx, (size_t)entries <= ctx->sc->seed_table_words, BITGNN_ERR_UNSUPPORTED,
               "bitgnn_bspmm: seed table too small");
    bspmm_seed_kernel<<<(entries * 32 + 255) / 256, 256, 0, s>>>(T, C, W32, P,
                                                              ctx->sc->seed_table);
    BG_LAUNCH_CHECK(ctx, "bspmm_seed");
    *seeds = ctx->sc->seed_table;
    return BITGNN_OK;
}

int bg_launch_bspmm_blocked(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj,
                            const uint64_t *hbits, int32_t C, int64_t h_stride, int epilogue,
                            const int32_t *T, void *out, int64_t out_stride)
{
    const bitgnn_blocked *b = adj->blk;
    const int32_t W32 = (C + 31) / 32;
    const int P = planes_for(adj);
    const int PF = part_planes_for(b) + 2;
    // With the threshold epilogue the aggregation kernel finishes the rows that are a single
    // part itself; only the first n_multi rows (in degree order) have parts to merge.
    const bool finish = epilogue == BITGNN_EPI_THRESH_BITS;
    // the threshold seeds are computed by extra workgroups of the first permute launch
    PermuteAux aux{};
    const uint32_t *seeds = nullptr;
    uint32_t *seeds_fin = nullptr;
    if (finish) {
        BG_REQUIRE(ctx, (size_t)(2 * (P + PF) * W32) <= ctx->sc->seed_table_words,
                   BITGNN_ERR_UNSUPPORTED, "bitgnn_bspmm: seed table too small");
        seeds_fin = ctx->sc->seed_table + 2 * P * W32;
        aux.kind = 1;
        aux.T = T;
        aux.C = C;
        aux.W32 = W32;
        aux.P = P;
        aux.PF = PF;
        aux.table = ctx->sc->seed_table;
        aux.table_fin = seeds_fin;
        seeds = ctx->sc->seed_table;
    }
    const size_t hperm_bytes = (((size_t)adj->n * 16) + 255) & ~(size_t)255;
    const size_t part_bytes = (size_t)b->n_vrows * part_planes_for(b) * 16;
    int rc = bg_ws_need(ctx, hperm_bytes + part_bytes, "bitgnn_bspmm");
    if (rc != BITGNN_OK)
        return rc;
    uint4 *hperm = (uint4 *)ctx->sc->ws;
    uint4 *partial = (uint4 *)((char *)ctx->sc->ws + hperm_bytes);
    const uint32_t *h32 = (const uint32_t *)hbits;
    const uint32_t merge_rows = finish ? b->n_multi : (uint32_t)adj->n;
    for (int win = 0; win * 4 < W32; ++win) {
        launch_permute(s, adj, h32, h_stride * 2, win * 4, W32, hperm, ctx->sc->queue,
                       win == 0 ? aux : PermuteAux{});
        BlkFinish fin{};
        fin.enabled = finish ? 1 : 0;
        fin.deg = adj->deg;
        fin.seeds = seeds_fin;
        fin.out = out;
        fin.out_stride = out_stride;
        fin.C = C;
        fin.W32 = W32;
        fin.win = win;
        rc = launch_blk(ctx, s, adj, hperm, partial, fin);
        if (rc != BITGNN_OK)
            return rc;
        switch (P) {
        case 12:
            launch_merge_p<12>(s, epilogue, adj, (const uint32_t *)partial, merge_rows, win, C,
                               W32, seeds, out, out_stride);
            break;
        case 16:
            launch_merge_p<16>(s, epilogue, adj, (const uint32_t *)partial, merge_rows, win, C,
                               W32, seeds, out, out_stride);
            break;
        case 20:
            launch_merge_p<20>(s, epilogue, adj, (const uint32_t *)partial, merge_rows, win, C,
                               W32, seeds, out, out_stride);
            break;
        default:
            launch_merge_p<26>(s, epilogue, adj, (const uint32_t *)partial, merge_rows, win, C,
                               W32, seeds, out, out_stride);
            break;
        }
        BG_LAUNCH_CHECK(ctx, "bspmm_merge");
    }
    return BITGNN_OK;
}

// logits = alpha * ((A_hat v) W) through the blocked form, 128 channels of v per pass.
int bg_launch_agg_project_blocked(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj,
                                  const uint64_t *hbits, int32_t K, int64_t h_stride,
                                  const uint64_t *wbits, int32_t M, int64_t w_stride,
                                  const float *alpha, int32_t *ysum, float *logits, int64_t ldo)
{
    const bitgnn_blocked *b = adj->blk;
    const int32_t W32 = (K + 31) / 32;
    const int nwin = (W32 + 3) / 4;
    const size_t hperm_bytes = (((size_t)adj->n * 16) + 255) & ~(size_t)255;
    const size_t part_bytes =
        ((size_t)b->n_vrows * part_planes_for(b) * 16 + 255) & ~(size_t)255;
    const int32_t Mpad = (M + 15) / 16 * 16;
    const size_t w8_bytes = (size_t)nwin * Mpad * 128;
    int rc = bg_ws_need(ctx, hperm_bytes + part_bytes + w8_bytes + (size_t)nwin * Mpad * 4,
                        "bitgnn_gcn_out_layer");
    if (rc != BITGNN_OK)
        return rc;
    uint4 *hperm = (uint4 *)ctx->sc->ws;
    uint4 *partial = (uint4 *)((char *)ctx->sc->ws + hperm_bytes);
    int8_t *w8 = (int8_t *)ctx->sc->ws + hperm_bytes + part_bytes;
    int32_t *wsum = (int32_t *)(w8 + w8_bytes);
    // the projection's +-1 byte weights are produced by extra workgroups of the first
    // permute launch
    PermuteAux aux{};
    aux.kind = 2;
    aux.w32 = (const uint32_t *)wbits;
    aux.w_stride32 = w_stride * 2;
    aux.K = K;
    aux.M = M;
    aux.Mpad = Mpad;
    aux.nwin = nwin;
    aux.w8 = w8;
    aux.wsum = wsum;
    const unsigned grid = (unsigned)((adj->n + kProjWaves * 16 - 1) / (kProjWaves * 16));
    // digits of 7 bits: max_degree < 2^(7 NB)
    int NB = 1;
    while ((1ll << (7 * NB)) <= adj->max_degree)
        ++NB;
    for (int win = 0; win < nwin; ++win) {
        launch_permute(s, adj, (const uint32_t *)hbits, h_stride * 2, win * 4, W32, hperm,
                       ctx->sc->queue, win == 0 ? aux : PermuteAux{});
        rc = launch_blk(ctx, s, adj, hperm, partial, BlkFinish{});
        if (rc != BITGNN_OK)
            return rc;
        const int32_t w32w = W32 - win * 4 < 4 ? W32 - win * 4 : 4;
        const int8_t *w8w = w8 + (size_t)win * Mpad * 128;
        const int32_t *wsumw = wsum + (size_t)win * Mpad;
        const bool has_prev = win > 0, is_last = win == nwin - 1;
#define BG_PROJECT(NBV)                                                                           \
    do {                                                                                          \
        if (part_planes_for(b) == 8)                                                              \
            bspmm_merge_project_kernel<NBV, 8><<<grid, kProjWaves * 64, 0, s>>>(                  \
                (const uint32_t *)partial, b->row_vptr, adj->order, adj->deg, (uint32_t)adj->n,   \
                w32w, w8w, wsumw, M, alpha, logits, ldo, ysum, has_prev, is_last);                \
        else                                                                                      \
            bspmm_merge_project_kernel<NBV, 10><<<grid, kProjWaves * 64, 0, s>>>(                 \
                (const uint32_t *)partial, b->row_vptr, adj->order, adj->deg, (uint32_t)adj->n,   \
                w32w, w8w, wsumw, M, alpha, logits, ldo, ysum, has_prev, is_last);                \
    } while (0)
        switch (NB) {
        case 1: BG_PROJECT(1); break;
        case 2: BG_PROJECT(2); break;
        case 3: BG_PROJECT(3); break;
        default: BG_PROJECT(4); break;
        }
#undef BG_PROJECT
        BG_LAUNCH_CHECK(ctx, "bspmm_merge_project");
    }
    return BITGNN_OK;
}

// Context workspace the aggregations on this graph use at most, for up to C aggregated
// channels (bit rows) and M output classes (integer rows / class projection): the largest
// of what the four launchers below and above lay out.
size_t bg_adj_workspace_bytes(const bitgnn_adj *adj, int32_t C, int32_t M)
{
    const size_t W32 = ((size_t)C + 31) / 32;
    size_t need = 0;
    // CSR bit-SpMM: degree-ordered copy of the rows + bit-sliced counts of the segments
    {
        const size_t perm = adj->col_slot ? (((size_t)adj->n * W32 * 4 + 255) & ~(size_t)255) : 0;
        int seg_planes = 1;
        while ((1u << seg_planes) <= adj->seg_len)
            ++seg_planes;
        need = perm + (size_t)adj->n_long_segs * seg_planes * W32 * 4;
    }
    // integer aggregation: int32 sums of the segments
    const size_t i32 = (size_t)adj->n_long_segs * (size_t)M * 4;
    need = i32 > need ? i32 : need;
    if (adj->blk) { // blocked form: one 128-channel window of rows + partial planes (+ the
                    // class projection's byte weights and column sums)
        const size_t hperm = (((size_t)adj->n * 16) + 255) & ~(size_t)255;
        const size_t part =
            ((size_t)adj->blk->n_vrows * part_planes_for(adj->blk) * 16 + 255) & ~(size_t)255;
        const size_t nwin = (W32 + 3) / 4, Mpad = ((size_t)M + 15) / 16 * 16;
        const size_t blk = hperm + part + nwin * Mpad * 128 + nwin * Mpad * 4;
        need = blk > need ? blk : need;
    }
    return need;
}

// Rough time models (microseconds, fitted on MI355X) of the two aggregation paths.  The
// CSR kernel is bound by its gather traffic or by the serial walk of the longest row;
// the blocked kernel by its id stream or, on small graphs, by the chain of LDS refills a
// workgroup walks through, and it pays that once per 128-channel pass.
bool bg_prefer_blocked(const bitgnn_adj *adj, int passes, int64_t bytes_per_nnz,
                       double chain_us_per_nnz, int64_t longest_chain)
{
    const bitgnn_blocked *b = adj->blk;
    if (!b)
        return false;
    if (b->forced)
        return true;
    // a gathered row costs its cache line plus its bytes: ~11 us per million 32-byte rows
    // (config 5), ~27 us per million 160-byte rows (the integer rows of an output layer)
    const double csr_traffic = (double)adj->nnz * (8.0 + 0.12 * (double)bytes_per_nnz) / 1e6;
    const double csr_chain = (double)longest_chain * chain_us_per_nnz;
    const double csr = (csr_traffic > csr_chain ? csr_traffic : csr_chain) + 10.0;
    const double stream = (double)b->n_groups * 64 * kGroupSteps / 1.3e6;
    const double rounds = (double)((b->n_wgs + 255) / 256);
    const double walk = rounds * (double)b->ncb * 3.0;
    const double blk = passes * ((stream > walk ? stream : walk) + 30.0);
    return blk < csr;
}

// force: 0 = choose (a measured preference of bitgnn_adj_tune first, else the time model),
// 1 = CSR kernel, 2 = column-blocked kernel (the caller has checked that the form exists)
static int launch_bspmm_path(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj,
                             const uint64_t *hbits, int32_t C, int64_t h_stride, int epilogue,
                             const int32_t *T, void *out, int64_t out_stride, int force)
{
    const int passes = (C + 127) / 128;
    bool blocked;
    if (force)
        blocked = force == 2;
    else if (adj->blk && !adj->blk->forced && adj->pref[passes < 4 ? passes - 1 : 3])
        blocked = adj->pref[passes < 4 ? passes - 1 : 3] == 2;
    else
        blocked = bg_prefer_blocked(adj, passes, 4 * (int64_t)((C + 31) / 32), 0.06,
                                    adj->max_degree < (int64_t)adj->seg_len
                                        ? adj->max_degree
                                        : (int64_t)adj->seg_len);
    if (blocked)
        return bg_launch_bspmm_blocked(ctx, s, adj, hbits, C, h_stride, epilogue, T, out,
                                       out_stride);
    const int32_t W32 = (C + 31) / 32;
    const int P = planes_for(adj);
    const uint32_t *seeds;
    int rc0 = launch_seeds(ctx, s, epilogue, T, C, W32, P, &seeds);
    if (rc0 != BITGNN_OK)
        return rc0;
    const int64_t threads = adj->n * (int64_t)W32;
    const int64_t pgrid = (threads + kBlock - 1) / kBlock;
    // virtual rows: the segments of the long rows, then the other rows
    const int64_t vrows = (int64_t)adj->n_long_segs + (adj->n - adj->n_long);
    const int64_t grid = (vrows * W32 + kBlock - 1) / kBlock;
    BG_REQUIRE(ctx, grid < (1ll << 31) && pgrid < (1ll << 31), BITGNN_ERR_UNSUPPORTED,
               "bitgnn_bspmm: N*C too large");
    const uint32_t *h32 = (const uint32_t *)hbits;
    const int32_t *col = adj->col;
    int64_t hs32 = h_stride * 2;
    const size_t perm_bytes = adj->col_slot ? (((size_t)threads * 4 + 255) & ~(size_t)255) : 0;
    int seg_planes = 1;
    while ((1u << seg_planes) <= adj->seg_len)
        ++seg_planes;
    const size_t seg_bytes = (size_t)adj->n_long_segs * seg_planes * W32 * 4;
    if (perm_bytes + seg_bytes) {
        const int rc = bg_ws_need(ctx, perm_bytes + seg_bytes, "bitgnn_bspmm");
        if (rc != BITGNN_OK)
            return rc;
    }
    const RowSegments seg{adj->seg_ptr,  adj->seg_slot, adj->n_long, adj->n_long_segs,
                          adj->seg_len,  seg_planes,    (uint32_t *)((char *)ctx->sc->ws + perm_bytes)};
    if (adj->col_slot) { // gather from a degree-ordered copy of the rows
        csr_permute_kernel<<<(unsigned)pgrid, kBlock, 0, s>>>(h32, hs32, adj->order,
                                                              (uint32_t)adj->n, W32,
                                                              (uint32_t *)ctx->sc->ws);
        BG_LAUNCH_CHECK(ctx, "csr_permute");
        h32 = (const uint32_t *)ctx->sc->ws;
        hs32 = W32;
        col = adj->col_slot;
    }
    bg_time_begin(ctx, s);
    switch (P) {
    case 12:
        launch_bspmm_p<12>(s, (unsigned)grid, epilogue, adj, col, h32, hs32, C, W32, seeds, out,
                           out_stride, seg);
        break;
    case 16:
        launch_bspmm_p<16>(s, (unsigned)grid, epilogue, adj, col, h32, hs32, C, W32, seeds, out,
                           out_stride, seg);
        break;
    case 20:
        launch_bspmm_p<20>(s, (unsigned)grid, epilogue, adj, col, h32, hs32, C, W32, seeds, out,
                           out_stride, seg);
        break;
    default:
        launch_bspmm_p<26>(s, (unsigned)grid, epilogue, adj, col, h32, hs32, C, W32, seeds, out,
                           out_stride, seg);
        break;
    }
    bg_time_end(ctx, s);
    BG_LAUNCH_CHECK(ctx, "bitgnn_bspmm");
    return BITGNN_OK;
}

int bg_launch_bspmm(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const uint64_t *hbits,
                    int32_t C, int64_t h_stride, int epilogue, const int32_t *T, void *out,
                    int64_t out_stride)
{
    return launch_bspmm_path(ctx, s, adj, hbits, C, h_stride, epilogue, T, out, out_stride, 0);
}

namespace {
struct TuneBuf { // device scratch of the tuning run, released on every return path
    void *p = nullptr;
    ~TuneBuf()
    {
        if (p)
            (void)hipFree(p);
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 8); }
};
} // namespace

// Tuning utility (Section 3.4): times the two aggregation kernels on this graph for a given
// width and keeps the winner in the handle.
extern "C" int bitgnn_adj_tune(bitgnn_ctx *ctx, void *stream, bitgnn_adj *adj, int32_t C,
                               int32_t reps, float *csr_ms, float *blocked_ms)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_adj_tune: adj is null");
    BG_REQUIRE(ctx, C >= 1 && reps >= 1 && reps <= 1000, BITGNN_ERR_INVALID_ARG,
               "bitgnn_adj_tune: C=%d reps=%d (1..1000)", C, reps);
    BG_NEED_DEVICE(ctx);
    if (csr_ms)
        *csr_ms = -1.0f;
    if (blocked_ms)
        *blocked_ms = -1.0f;
    if (adj->n == 0 || adj->nnz == 0)
        return BITGNN_OK;
    hipStream_t s = (hipStream_t)stream;
    const int64_t cw = ((int64_t)C + 63) / 64;
    { // a set-up call: it may grow the workspace
        const int rc_ws = bitgnn_ctx_reserve(ctx, bg_adj_workspace_bytes(adj, C, 1));
        if (rc_ws != BITGNN_OK)
            return rc_ws;
    }
    TuneBuf h, out, T;
    BG_HIP(ctx, h.alloc((size_t)adj->n * cw * 8));
    BG_HIP(ctx, out.alloc((size_t)adj->n * cw * 8));
    BG_HIP(ctx, T.alloc((size_t)C * 4));
    BG_HIP(ctx, hipMemsetAsync(h.p, 0x5A, (size_t)adj->n * cw * 8, s));
    BG_HIP(ctx, hipMemsetAsync(T.p, 0, (size_t)C * 4, s));
    hipEvent_t e0, e1;
    BG_HIP(ctx, hipEventCreate(&e0));
    BG_HIP(ctx, hipEventCreate(&e1));
    float ms[3] = {0.0f, -1.0f, -1.0f};
    int rc = BITGNN_OK;
    for (int path = 1; path <= 2 && rc == BITGNN_OK; ++path) {
        if (path == 2 && !adj->blk)
            break;
        // one untimed call first (workspace growth, code upload)
        for (int i = 0; i <= reps && rc == BITGNN_OK; ++i) {
            if (i == 1)
                (void)hipEventRecord(e0, s);
            rc = launch_bspmm_path(ctx, s, adj, (const uint64_t *)h.p, C, cw, BITGNN_EPI_THRESH_BITS,
                                   (const int32_t *)T.p, out.p, cw, path);
        }
        if (rc != BITGNN_OK)
            break;
        (void)hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess) {
            rc = bitgnn_fail(ctx, BITGNN_ERR_HIP, "bitgnn_adj_tune: event synchronize failed");
            break;
        }
        (void)hipEventElapsedTime(&ms[path], e0, e1);
        ms[path] /= (float)reps;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipStreamSynchronize(s);
    if (rc != BITGNN_OK)
        return rc;
    if (csr_ms)
        *csr_ms = ms[1];
    if (blocked_ms)
        *blocked_ms = ms[2];
    if (adj->blk) {
        const int passes = (C + 127) / 128;
        adj->pref[passes < 4 ? passes - 1 : 3] = ms[2] < ms[1] ? 2 : 1;
    }
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

// ---------------------------------------------------------------------------
// The same aggregation for callers that cannot allocate (code under HIP graph capture,
// tight serving loops): every scratch buffer of the kernels -- work counter, threshold
// seeds, degree-ordered activation rows, partial counters of row parts and segments --
// lives in one static device array, so the call touches no allocator at all.  Each GPU
// holds its own copy of the array until the process ends; its address is looked up once
// per device and kept (the array's name itself is only a host-side stand-in).
namespace {
constexpr size_t kStaticQueueBytes = 256;
constexpr size_t kStaticSeedBytes = (kSeedTableWords * 4 + 255) & ~(size_t)255;
constexpr size_t kStaticHeadBytes = kStaticQueueBytes + kStaticSeedBytes;
constexpr size_t kStaticScratchBytes = BITGNN_STATIC_SCRATCH_BYTES;
static_assert(kStaticScratchBytes > kStaticHeadBytes && kStaticScratchBytes % 256 == 0, "layout");
constexpr int kMaxStaticDevices = 64;
} // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void *g_static_scratch[kMaxStaticDevices]; // device address of `scratch`, per device

// Set-up: called by bitgnn_ctx_create with the context's device current.
int bg_static_scratch_init(bitgnn_ctx *ctx)
{
    if (ctx->device < 0 || ctx->device >= kMaxStaticDevices || g_static_scratch[ctx->device])
        return BITGNN_OK;
    void *ptr = nullptr;
    BG_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    g_static_scratch[ctx->device] = ptr;
    return BITGNN_OK;
}

extern "C" int bitgnn_bspmm_static(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                   const uint64_t *hbits, int32_t C, int64_t h_stride,
                                   int epilogue, const int32_t *T, void *out, int64_t out_stride)
{
    int rc = bg_check_bspmm(ctx, adj, hbits, C, h_stride, epilogue, T, out, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    BG_REQUIRE(ctx, ctx->device < kMaxStaticDevices && g_static_scratch[ctx->device],
               BITGNN_ERR_UNSUPPORTED, "bitgnn_bspmm_static: no static scratch on device %d",
               ctx->device);
    const size_t avail = kStaticScratchBytes - kStaticHeadBytes;
    const size_t need = bg_adj_workspace_bytes(adj, C, 1);
    BG_REQUIRE(ctx, need <= avail, BITGNN_ERR_UNSUPPORTED,
               "bitgnn_bspmm_static: this graph needs %zu bytes of scratch, the static array "
               "holds %zu (use bitgnn_bspmm)",
               need, avail);
    unsigned char *base = (unsigned char *)g_static_scratch[ctx->device];
    bg_scratch st;
    st.queue = (uint32_t *)base;
    st.seed_table = (uint32_t *)(base + kStaticQueueBytes);
    st.seed_table_words = kSeedTableWords;
    st.ws = base + kStaticHeadBytes;
    st.ws_bytes = avail;
    ctx->sc = &st; // the kernels take these pointers exactly as they take the context's
    rc = bg_launch_bspmm(ctx, (hipStream_t)stream, adj, hbits, C, h_stride, epilogue, T, out,
                         out_stride);
    ctx->sc = &ctx->own;
    return rc;
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
    const int64_t vrows = (int64_t)adj->n_long_segs + (adj->n - adj->n_long);
    const int64_t grid = ((vrows << lpr_log2) + kBlock - 1) / kBlock;
    BG_REQUIRE(ctx, grid < (1ll << 31), BITGNN_ERR_UNSUPPORTED, "bitgnn_spmm_i32: N too large");
    if (adj->n_long_segs) {
        const int rc = bg_ws_need(ctx, (size_t)adj->n_long_segs * M * 4, "bitgnn_spmm_i32");
        if (rc != BITGNN_OK)
            return rc;
    }
    const RowSegments seg{adj->seg_ptr, adj->seg_slot, adj->n_long, adj->n_long_segs,
                          adj->seg_len, 0,             (uint32_t *)ctx->sc->ws};
    const unsigned grid_long =
        (unsigned)((((uint64_t)adj->n_long << lpr_log2) + kBlock - 1) / kBlock);
    // wide rows that can be read 4 or 2 values per lane: several neighbours per gather
    const int vw = (M > 32 && M % 4 == 0 && z_stride % 4 == 0 && bg_aligned(Z, 16) && M <= 128) ? 4
                   : (M > 32 && M % 2 == 0 && z_stride % 2 == 0 && bg_aligned(Z, 8) && M <= 64)
                       ? 2
                       : 1;
    const unsigned grid_wide = (unsigned)((vrows + kBlock / 64 - 1) / (kBlock / 64));
#define BG_SPMM_I32(SV)                                                                           \
    do {                                                                                          \
        if (vw == 4)                                                                              \
            spmm_i32_wide_kernel<SV, 4><<<grid_wide, kBlock, 0, s>>>(                             \
                adj->rowptr, adj->col, adj->order, (uint32_t)adj->n, Z, M, z_stride, alpha, out,  \
                out_stride, seg);                                                                 \
        else if (vw == 2)                                                                         \
            spmm_i32_wide_kernel<SV, 2><<<grid_wide, kBlock, 0, s>>>(                             \
                adj->rowptr, adj->col, adj->order, (uint32_t)adj->n, Z, M, z_stride, alpha, out,  \
                out_stride, seg);                                                                 \
        else                                                                                      \
            spmm_i32_kernel<SV><<<(unsigned)grid, kBlock, 0, s>>>(                                \
                adj->rowptr, adj->col, adj->order, (uint32_t)adj->n, Z, M, z_stride, alpha, out,  \
                out_stride, lpr_log2, seg);                                                       \
        if (grid_long)                                                                            \
            spmm_i32_long_rows_kernel<SV><<<grid_long, kBlock, 0, s>>>(                           \
                adj->order, M, alpha, out, out_stride, lpr_log2, seg);                            \
    } while (0)
    if (alpha)
        BG_SPMM_I32(true);
    else
        BG_SPMM_I32(false);
#undef BG_SPMM_I32
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
