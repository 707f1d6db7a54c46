// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/bitgnn.h"

#define BITGNN_WAVE 64

// Device scratch the aggregation kernels work in: the context's own (allocated by the
// set-up calls), or the library's static array for the entry point that allocates nothing.
struct bg_scratch {
    uint32_t *queue;      // device words: [0] work counter of the blocked bit-SpMM,
                          // [kFusedBarrierWord] arrival counter of the fused kernel's barriers
    uint32_t *seed_table; // bit-SpMM threshold seeds
    size_t seed_table_words;
    // degree-ordered activations, partial counters of row parts and segments; sized by
    // bitgnn_adj_workspace_bytes, allocated by bitgnn_ctx_reserve / bitgnn_adj_build only
    void *ws;
    size_t ws_bytes;
};

struct bitgnn_ctx {
    int device;           // -1: validation-only context
    int n_cus;            // compute units of the device
    int bgemm_path;       // BITGNN_BGEMM_AUTO / _VALU / _MFMA (bitgnn_ctx_set_bgemm_path)
    void *bgemm_ws;       // device scratch of the matrix-core BMM: widened weights and their
                          // popcounts (fixed size, allocated with the context)
    bg_scratch own;       // the context's scratch
    bg_scratch *sc;       // the scratch the current call uses (&own outside such a call)
    uint32_t fused_spin_limit; // polls of one barrier wait before it is abandoned
    char err[256];
    // tuning of the column-blocked aggregation format (bitgnn_ctx_set_tuning)
    int32_t cb_nodes;       // nodes per LDS-resident column block (<= kMaxCbNodes)
    int32_t part_len;       // longest run of neighbours one lane accumulates (<= 1023)
    int32_t min_avg_degree; // graphs sparser than this keep the plain CSR path only
    // optional HIP-event timing of the main aggregation kernel (bitgnn_ctx_kernel_timing)
    int timing;
    int n_timed;
    hipEvent_t tev[2 * 256];
};

// Largest seed tables the bit-SpMM may ask for: 2 parities x 64 words x (26 planes for the
// merge + 12 planes for the rows the blocked kernel finishes itself).
static const size_t kSeedTableWords = 2 * (26 + 12) * 64;
static const int kMaxTimed = 256;
// Scratch of the matrix-core BMM: at most 144 KB of widened weights (its LDS limit) plus
// one popcount per padded weight row.
static const size_t kBgemmScratchBytes = 144 * 1024 + 16 * 1024;
// Widths bitgnn_adj_build reserves workspace for.
static const int32_t kDefaultWsChannels = 256, kDefaultWsClasses = 64;
static const int kFusedBarrierWord = 16; // its own 64-byte line of ctx->queue
// Brackets one kernel launch with events when timing is on (no-ops otherwise).
static inline void bg_time_begin(bitgnn_ctx *ctx, hipStream_t s)
{
    if (ctx->timing && ctx->n_timed < kMaxTimed)
        (void)hipEventRecord(ctx->tev[2 * ctx->n_timed], s);
}
static inline void bg_time_end(bitgnn_ctx *ctx, hipStream_t s)
{
    if (ctx->timing && ctx->n_timed < kMaxTimed) {
        (void)hipEventRecord(ctx->tev[2 * ctx->n_timed + 1], s);
        ++ctx->n_timed;
    }
}

// Gather steps per group of the blocked format: one lane's ids of a group are
// kGroupSteps consecutive 16-bit words (one or two 16-byte loads).
#ifndef BITGNN_GROUP_STEPS
#define BITGNN_GROUP_STEPS 8
#endif
static const int kGroupSteps = BITGNN_GROUP_STEPS;
static_assert(kGroupSteps == 8 || kGroupSteps == 16, "groups of 8 or 16 steps");

// Slices (wavefronts) per workgroup of the blocked bit-SpMM: 16 on large graphs; 8 or 4
// where that is what it takes to give every compute unit a work item.
static const int kSlicesPerWg = 16;
// most rows of a column block: (rows + 16 zero rows) x 16 bytes fill the 160 KB of LDS
static const int kMaxCbNodes = 10208;

// Segment lengths of the CSR bit-SpMM (see bitgnn_adj::seg_len) and the non-zero count from
// which the long one is used.
static const uint32_t kSegLenSmall = 128, kSegLenLarge = 1024;
static const int64_t kSegLargeNnz = 1ll << 24;

// Column-blocked, length-balanced aggregation format (see adj_blocked.hip).
struct bitgnn_blocked {
    int32_t cbn;            // nodes per column block
    uint32_t n_multi;       // rows with more than one part (the first n_multi degree-order slots)
    int32_t ncb;            // column blocks
    int32_t part_len;       // longest row part (sets the planes of the partial counters)
    int32_t forced;         // built with a density threshold of 0: always preferred
    uint32_t n_vrows;       // V: row parts ("virtual rows")
    uint32_t n_slices;      // ceil(V / 64)
    int32_t spw;            // slices (wavefronts) per work item: 16, 8 or 4
    uint32_t n_wgs;         // ceil(slices / spw)
    uint32_t n_tiles;       // (slice, column block) tiles
    uint32_t n_groups;      // groups of kGroupSteps gather steps over all tiles
    uint2 *wg_item;         // [n_wgs] by decreasing estimated work: {workgroup,
                            //         first column block | last << 16}
    uint4 *sl_desc;         // [n_slices] {first block | last << 16, first tile, first group, 0}
    uint32_t *tile_group;   // [n_tiles + 1] prefix of group counts
    uint16_t *idx16;        // [(n_groups + 1) * 64 * kGroupSteps] column ids inside the block;
                            // cbn = "none"; the last group is padding that a prefetch may read
    uint32_t *row_vptr;     // [n + 1] by degree-order slot: first part of the row
    uint2 *part_info;       // [V] by processing position: {part id (a row's parts are consecutive
                            // ids) | bit 31: the row's only part, node id of the row}
    size_t device_bytes;
};

struct bitgnn_adj {
    int device;
    int64_t n;
    int64_t nnz;
    int64_t max_degree;
    uint32_t *rowptr; // [n+1]
    int32_t *col;     // [nnz]
    int32_t *deg;     // [n]
    int32_t *order;   // [n] rows by decreasing degree
    int32_t *col_slot; // [nnz] column indices as degree-order slots (large CSR-only graphs:
                       // gathers from a degree-ordered copy keep the hubs' rows together)
    // Row segments of the CSR bit-SpMM: a row longer than seg_len neighbours is walked by
    // several thread groups, seg_len neighbours each (such rows come first in `order`).
    uint32_t seg_len;   // 128 on small graphs, where the longest row's serial walk is what
                        // the kernel waits for; 1024 on large ones, where only true hubs are
                        // worth the segments' extra pass (a power of two, at most 1024)
    uint32_t *seg_ptr;  // [n_long + 1] by degree-order slot: first segment of the long row
    uint32_t *seg_slot; // [n_long_segs] segment -> degree-order slot of its row
    uint32_t n_long;      // rows with more than seg_len neighbours
    uint32_t n_long_segs; // their segments
    size_t device_bytes;
    bitgnn_blocked *blk; // null when the graph is too sparse for the blocked path
    // bitgnn_adj_tune's verdict for bit aggregations of 1, 2, 3, >= 4 passes of 128 channels:
    // 0 = not measured (the time model decides), 1 = CSR kernel, 2 = column-blocked kernel
    int8_t pref[4];
};

static inline int bitgnn_fail(bitgnn_ctx *ctx, int code, const char *fmt, ...)
    __attribute__((format(printf, 3, 4)));
static inline int bitgnn_fail(bitgnn_ctx *ctx, int code, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

#define BG_REQUIRE(ctx, cond, code, ...)                                                          \
    do {                                                                                          \
        if (!(cond))                                                                              \
            return bitgnn_fail((ctx), (code), __VA_ARGS__);                                       \
    } while (0)

#define BG_HIP(ctx, call)                                                                         \
    do {                                                                                          \
        hipError_t e_ = (call);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return bitgnn_fail((ctx), BITGNN_ERR_HIP, "%s failed: %s (%d)", #call,                \
                               hipGetErrorString(e_), (int)e_);                                   \
    } while (0)

// After a kernel launch: report launch-time errors (bad configuration etc.).
#define BG_LAUNCH_CHECK(ctx, name)                                                                \
    do {                                                                                          \
        hipError_t e_ = hipGetLastError();                                                        \
        if (e_ != hipSuccess)                                                                     \
            return bitgnn_fail((ctx), BITGNN_ERR_HIP, "launch of %s failed: %s (%d)", name,       \
                               hipGetErrorString(e_), (int)e_);                                   \
    } while (0)

static inline bool bg_aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Calls with a validation-only context stop here, after all argument checks.
#define BG_NEED_DEVICE(ctx)                                                                       \
    do {                                                                                          \
        if ((ctx)->device < 0)                                                                    \
            return bitgnn_fail((ctx), BITGNN_ERR_NO_DEVICE,                                       \
                               "arguments valid; context has no GPU");                            \
    } while (0)

// Internal launchers shared across translation units (arguments already validated).
int bg_launch_bgemm(bitgnn_ctx *ctx, hipStream_t s, const uint64_t *xbits, int64_t n,
                    int64_t x_stride, int32_t K, int32_t kwords, const uint64_t *wbits, int32_t M,
                    int64_t w_stride, int epilogue, const int32_t *T, const float *alpha,
                    void *out, int64_t out_stride);
int bg_launch_bspmm(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const uint64_t *hbits,
                    int32_t C, int64_t h_stride, int epilogue, const int32_t *T, void *out,
                    int64_t out_stride);
int bg_launch_spmm_i32(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const int32_t *Z,
                       int32_t M, int64_t z_stride, const float *alpha, void *out,
                       int64_t out_stride);

bool bg_bgemm_mfma_applies(const bitgnn_ctx *ctx, int64_t n, int32_t kwords, int32_t M);
int bg_launch_bgemm_mfma(bitgnn_ctx *ctx, hipStream_t s, const uint64_t *xbits, int64_t n,
                         int64_t x_stride, int32_t K, int32_t kwords, const uint64_t *wbits,
                         int32_t M, int64_t w_stride, int epilogue, const int32_t *T,
                         const float *alpha, void *out, int64_t out_stride);
int bg_build_blocked(bitgnn_ctx *ctx, hipStream_t s, bitgnn_adj *adj);
void bg_free_blocked(bitgnn_blocked *b);
int bg_launch_bspmm_blocked(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj,
                            const uint64_t *hbits, int32_t C, int64_t h_stride, int epilogue,
                            const int32_t *T, void *out, int64_t out_stride);
int bg_ws_need(bitgnn_ctx *ctx, size_t bytes, const char *who);
int bg_static_scratch_init(bitgnn_ctx *ctx);
// Bytes of context workspace the aggregations on `adj` need for up to C aggregated
// channels and M output classes.
size_t bg_adj_workspace_bytes(const bitgnn_adj *adj, int32_t C, int32_t M);
// Whether the blocked form is expected to beat the CSR kernel for rows of `bytes_per_nnz`
// gathered bytes per non-zero, handled in `passes` passes of the blocked kernel.
// `longest_chain`: neighbours the CSR kernel in question walks serially at most.
bool bg_prefer_blocked(const bitgnn_adj *adj, int passes, int64_t bytes_per_nnz,
                       double chain_us_per_nnz, int64_t longest_chain);
int bg_launch_agg_project_blocked(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj,
                                  const uint64_t *hbits, int32_t K, int64_t h_stride,
                                  const uint64_t *wbits, int32_t M, int64_t w_stride,
                                  const float *alpha, int32_t *ysum, float *logits, int64_t ldo);

int bg_check_bgemm_f32(bitgnn_ctx *ctx, const float *x, int64_t n, int32_t K, int64_t ldx,
                       const float *tau, const uint64_t *wbits, int32_t M, int64_t w_stride,
                       int epilogue, const int32_t *T, const float *alpha, const void *out,
                       int64_t out_stride);
int bg_launch_bgemm_f32(bitgnn_ctx *ctx, hipStream_t s, const float *x, int64_t n, int32_t K,
                        int64_t ldx, const float *tau, const uint64_t *wbits, int32_t M,
                        int64_t w_stride, int epilogue, const int32_t *T, const float *alpha,
                        void *out, int64_t out_stride);

// Argument validation of the public calls, shared with the layer drivers.
int bg_check_bgemm(bitgnn_ctx *ctx, const uint64_t *xbits, int64_t n, int64_t x_stride, int32_t K,
                   int32_t kwords, const uint64_t *wbits, int32_t M, int64_t w_stride,
                   int epilogue, const int32_t *T, const float *alpha, const void *out,
                   int64_t out_stride);
int bg_check_spmm_f32(bitgnn_ctx *ctx, const bitgnn_adj *adj, const void *x, int x_is_bits,
                      int32_t C, int64_t ldx, const float *r, const float *f, int epilogue,
                      const float *tau, const void *out, int64_t ldo);
int bg_launch_spmm_f32(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj, const void *x,
                       int x_is_bits, int32_t C, int64_t ldx, const float *r, const float *f,
                       int epilogue, const float *tau, void *out, int64_t ldo,
                       const float *xscale);
int bg_launch_narrow_rows(bitgnn_ctx *ctx, hipStream_t s, int32_t *z, int64_t n, int32_t M,
                          int64_t ld32);
int bg_check_bspmm(bitgnn_ctx *ctx, const bitgnn_adj *adj, const uint64_t *hbits, int32_t C,
                   int64_t h_stride, int epilogue, const int32_t *T, const void *out,
                   int64_t out_stride);
int bg_check_spmm_i32(bitgnn_ctx *ctx, const bitgnn_adj *adj, const int32_t *Z, int32_t M,
                      int64_t z_stride, int64_t z_abs_bound, const void *out, int64_t out_stride);
