/*
 * bitgnn.h - C ABI of the MI355X (gfx950) binary-GNN inference library.
 *
 * The calls follow the problem statement of BitGNN (ICS '23): binarize and
 * bit-pack node features, build the adjacency, run binary GCN / GraphSAGE
 * layers (bit matrix product for the feature transformation, bit sparse
 * product for the neighbour aggregation, re-binarization fused into both),
 * return float logits.
 *
 * Conventions for every entry point
 *  - returns BITGNN_OK (0) or a negative BITGNN_ERR_* code; nothing throws.
 *    A message for the last failure of a context is kept in the context
 *    (bitgnn_last_error).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Compute calls only enqueue work on it and return: they never allocate,
 *    free or synchronize, so they may be recorded into a HIP graph.  The set-up
 *    calls (bitgnn_ctx_create, bitgnn_ctx_reserve, bitgnn_adj_build and the
 *    *_tune utilities) allocate and synchronize.  A context serves ONE stream at
 *    a time: it owns device scratch that concurrent calls would race on.
 *  - every data pointer is a DEVICE pointer owned by the caller and must stay
 *    valid until the enqueued work has run.  The library allocates device
 *    memory only inside a bitgnn_adj and inside a context: a few hundred KB of
 *    fixed scratch, plus the aggregation workspace (degree-ordered activation
 *    rows, partial counters of row parts and segments).  bitgnn_adj_build
 *    reserves that workspace for aggregations of up to
 *    BITGNN_DEFAULT_WS_CHANNELS channels and BITGNN_DEFAULT_WS_CLASSES classes
 *    on the graph it builds; wider calls need bitgnn_adj_workspace_bytes +
 *    bitgnn_ctx_reserve first and fail with BITGNN_ERR_WORKSPACE otherwise.
 *  - packed bit layout (part of the ABI): a packed matrix is row-major
 *    uint64 words, little endian; logical bit k of a row is bit (k % 64) of
 *    word (k / 64); bit 1 encodes +1 and bit 0 encodes -1.  Rows are addressed
 *    as (pointer, row stride in words), so a caller can place a packed block at
 *    any word offset inside a wider row (GraphSAGE's [self | neighbour] rows).
 *    Bits past the logical width in the last word are ZERO in every output and
 *    must be zero in every input.
 *  - a context created with device = -1 has no GPU: every call still validates
 *    its arguments and then returns BITGNN_ERR_NO_DEVICE instead of launching.
 *    There is no CPU implementation behind this library.
 */
#ifndef BITGNN_H
#define BITGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bitgnn_ctx bitgnn_ctx; /* opaque, library-owned */
typedef struct bitgnn_adj bitgnn_adj; /* opaque, library-owned, immutable once built */

enum {
    BITGNN_OK = 0,
    BITGNN_ERR_INVALID_ARG = -1, /* null pointer, negative or inconsistent size, bad enum */
    BITGNN_ERR_ALIGNMENT = -2,   /* pointer not aligned to its element type */
    BITGNN_ERR_INDEX_RANGE = -3, /* an edge endpoint is outside [0, N) */
    BITGNN_ERR_RANGE = -4,       /* an int32 accumulator or a 32-bit offset could overflow */
    BITGNN_ERR_HIP = -5,         /* a HIP runtime call failed (code in the message) */
    BITGNN_ERR_UNSUPPORTED = -6, /* size beyond what the kernels are built for */
    BITGNN_ERR_NO_DEVICE = -7,   /* arguments are valid but the context has no GPU */
    BITGNN_ERR_WORKSPACE = -8    /* the context workspace is too small for this call:
                                    bitgnn_adj_workspace_bytes + bitgnn_ctx_reserve */
};

/* Widths for which bitgnn_adj_build reserves the context workspace by itself. */
#define BITGNN_DEFAULT_WS_CHANNELS 256
#define BITGNN_DEFAULT_WS_CLASSES 64

enum { /* kernels of the BMM (Section 2.2), bitgnn_ctx_set_bgemm_path */
    BITGNN_BGEMM_AUTO = 0, /* chosen per shape from measured crossovers */
    BITGNN_BGEMM_VALU = 1, /* xor + popcount on the vector ALUs */
    BITGNN_BGEMM_MFMA = 2  /* bits widened to bytes, int8 matrix cores */
};

enum {
    BITGNN_ADJ_SYMMETRIZE = 1,    /* also store (j, i) for every (i, j) */
    BITGNN_ADJ_ADD_SELF_LOOPS = 2 /* A_hat = A + I (Section 2.1, GCNConv) */
};

enum {
    BITGNN_EPI_RAW_I32 = 0,     /* int32 accumulators */
    BITGNN_EPI_THRESH_BITS = 1, /* bit = (acc >= T[c]), packed */
    BITGNN_EPI_SCALE_F32 = 2    /* float = alpha[c] * (float)acc */
};

/* ---- context ------------------------------------------------------------ */

/* Creates a context on HIP device `device` (>= 0), or a GPU-less validation
 * context (device == -1).  *out is set only on success. */
int bitgnn_ctx_create(bitgnn_ctx **out, int device);
void bitgnn_ctx_destroy(bitgnn_ctx *ctx);
/* Message of the most recent failing call on `ctx` ("" if none).  The string
 * is owned by the context and valid until the next call on it. */
const char *bitgnn_last_error(const bitgnn_ctx *ctx);

/* Tuning of the aggregation format built by later bitgnn_adj_build calls (the
 * counterpart of the paper's tuning utilities, Section 3.4).  A graph with at
 * least min_avg_degree stored non-zeros per node also gets a column-blocked form
 * (unless its tiles would pad to more than 6 stored ids per non-zero; 0 forces it)
 * whose activation blocks of cb_nodes nodes (64..10208) are staged in LDS and
 * whose rows are cut into parts of at most part_len (4..1023) neighbours (up to
 * 255 the per-part partial counters are one 128-byte line, above it they take
 * 160 bytes); sparser graphs use plain CSR with global-memory gathers.  Results do
 * not depend on these values.  Defaults: 10208 (with 16 zero rows beside it a block
 * then fills the 160 KB of LDS), 255, 8. */
int bitgnn_ctx_set_tuning(bitgnn_ctx *ctx, int32_t cb_nodes, int32_t part_len,
                          int32_t min_avg_degree);

/* Forces one of the two BMM kernels (tests, A/B measurements); BITGNN_BGEMM_MFMA still
 * falls back to the VALU kernel for shapes the matrix-core kernel does not take (rows of
 * more than 16 words; it runs wide outputs in column chunks whose widened weights fit its
 * LDS).  Results never depend on the choice.  Default: BITGNN_BGEMM_AUTO. */
int bitgnn_ctx_set_bgemm_path(bitgnn_ctx *ctx, int path);
/* Which kernel bitgnn_bgemm launches for n rows of kwords 64-bit words against M weight
 * rows under the context's current setting: *kernel <- BITGNN_BGEMM_VALU or _MFMA.  Host
 * only; works on any context. */
int bitgnn_ctx_bgemm_kernel(const bitgnn_ctx *ctx, int64_t n, int32_t kwords, int32_t M,
                            int *kernel);

/* Grows the context's aggregation workspace to at least `bytes` (never shrinks it).  A
 * set-up call: it allocates, and synchronizes the device when it replaces a smaller
 * workspace, so no work of this context may be in flight or being captured.
 * bitgnn_ctx_workspace reports the current size. */
int bitgnn_ctx_reserve(bitgnn_ctx *ctx, size_t bytes);
int bitgnn_ctx_workspace(const bitgnn_ctx *ctx, size_t *bytes);

/* Optional timing of the main aggregation kernel of every bit-SpMM call (the
 * LDS-staged kernel, or the CSR kernel on sparse graphs; the small permute / merge
 * kernels around it are not included).  While enabled, each launch is bracketed by
 * HIP events on the call's stream; up to 256 launches are kept.
 * bitgnn_ctx_kernel_times waits for the recorded launches, writes their durations
 * in milliseconds (launch order) to ms[0..*count) and empties the list. */
int bitgnn_ctx_kernel_timing(bitgnn_ctx *ctx, int enable);
int bitgnn_ctx_kernel_times(bitgnn_ctx *ctx, float *ms, int32_t capacity, int32_t *count);

/* ---- BIN: binarize and pack (Section 2.2 sign rule; Section 2.3) --------- */

/* out[i][k/64] bit k%64 = (x[i*ldx + k] >= tau[k]) for k < K; tau == NULL means
 * tau = 0, the paper's sign function (x >= 0 -> +1, so -0.0 -> +1; NaN -> -1).
 * A per-column tau is BatchNorm folded into the comparison.
 * x: float [n][ldx] (ldx >= K); out: uint64 [n][out_stride], the call writes
 * ceil(K/64) words of every row and leaves the rest of the row untouched. */
int bitgnn_pack_f32(bitgnn_ctx *ctx, void *stream, const float *x, int64_t n, int32_t K,
                    int64_t ldx, const float *tau, uint64_t *out, int64_t out_stride);
/* Same for int8 input with the fixed rule x >= 0 -> bit 1. */
int bitgnn_pack_i8(bitgnn_ctx *ctx, void *stream, const int8_t *x, int64_t n, int32_t K,
                   int64_t ldx, uint64_t *out, int64_t out_stride);
/* Packs a weight matrix transposed, as the BGEMM wants it (weights are
 * binarized offline, Section 3.1.1): out[c][k/64] bit k%64 = (w[k*ldw + c] >= 0)
 * for k < K, c < M.  w: int8 [K][ldw]; out: uint64 [M][out_stride]. */
int bitgnn_pack_weights_i8(bitgnn_ctx *ctx, void *stream, const int8_t *w, int32_t K, int32_t M,
                           int64_t ldw, uint64_t *out, int64_t out_stride);

/* ---- adjacency (Section 2.1 A_hat; Section 3.2.1 sparse bit representation) */

/* Builds the 0/1 aggregation matrix from an edge list: A_hat[i][j] = 1 iff
 * (src, dst) = (i, j) occurs (or (j, i) with SYMMETRIZE, or i == j with
 * ADD_SELF_LOOPS).  Duplicates collapse (set semantics).  Row i of the result
 * lists N(i) = { j : A_hat[i][j] = 1 } in increasing j.
 * src, dst: int32 [E] device arrays, left unchanged.  Requires
 * E*(1 + symmetrize) + N < 2^31.  Synchronizes `stream`.  Temporary sort
 * buffers are freed before returning; the handle keeps the CSR arrays, the
 * degrees and a degree-sorted row order.  Also grows the context's aggregation
 * workspace (bitgnn_ctx_reserve) to what this graph needs at the default widths.
 * Errors: BITGNN_ERR_INDEX_RANGE if an endpoint is outside [0, N). */
int bitgnn_adj_build(bitgnn_ctx *ctx, void *stream, const int32_t *src, const int32_t *dst,
                     int64_t E, int64_t N, uint32_t flags, bitgnn_adj **out);
/* Context workspace (bytes) that compute calls on `adj` use at most when they aggregate
 * up to C_max channels (bit or float rows; 1..2048) and produce up to M_max classes
 * (bitgnn_spmm_i32, output layers).  Pass the result to bitgnn_ctx_reserve before the
 * first such call when C_max or M_max exceed the defaults bitgnn_adj_build reserves for. */
int bitgnn_adj_workspace_bytes(const bitgnn_adj *adj, int32_t C_max, int32_t M_max,
                               size_t *bytes);
/* Any output pointer may be NULL. */
int bitgnn_adj_info(const bitgnn_adj *adj, int64_t *N, int64_t *nnz, int64_t *max_degree,
                    size_t *device_bytes);
/* Device views of the handle's arrays (owned by the handle): rowptr uint32
 * [N+1], col int32 [nnz] (sorted inside each row), deg int32 [N]. */
int bitgnn_adj_csr(const bitgnn_adj *adj, const uint32_t **rowptr, const int32_t **col,
                   const int32_t **deg);
/* Shape of the column-blocked form, if the handle has one (else every output is
 * 0): row parts, slices of 64 parts, workgroups, (slice, block) tiles, stored ids
 * including padding, and nodes per column block.  Any pointer may be NULL. */
int bitgnn_adj_blocked_info(const bitgnn_adj *adj, int64_t *parts, int64_t *slices,
                            int64_t *workgroups, int64_t *tiles, int64_t *stored_ids,
                            int64_t *cb_nodes);
void bitgnn_adj_destroy(bitgnn_adj *adj);

/* Tuning utility (the paper's Section 3.4, per graph): runs bitgnn_bspmm's two kernels
 * (CSR with global-memory gathers, column-blocked with LDS-staged gathers) `reps` times
 * each on this graph for C channels, on scratch activations the call allocates and frees,
 * and records the faster one in the handle: later bit aggregations of the same number of
 * 128-channel passes take it instead of asking the built-in time model.  Results never
 * depend on the choice.  csr_ms / blocked_ms (host pointers, may be NULL) receive the
 * average time of a call in milliseconds, -1 for a form the handle does not have.
 * Synchronises the stream.  The handle must not be in use by other calls meanwhile. */
int bitgnn_adj_tune(bitgnn_ctx *ctx, void *stream, bitgnn_adj *adj, int32_t C, int32_t reps,
                    float *csr_ms, float *blocked_ms);

/* ---- BMM: XNOR-popcount product (Section 2.2, +-1 bit-dot-product) ------- */

/* Z[i][c] = sum_k vx[i][k]*vw[k][c] = K - 2*popc(xbits_i xor wbits_c), where the
 * xor runs over `kwords` words of both operands and K is the number of logical
 * (non-pad) bits among them (pad bits are zero in both, so they cancel).
 * xbits: uint64 [n][x_stride]; wbits: uint64 [M][w_stride] (K along the bits).
 * epilogue RAW_I32:     out = int32 [n][out_stride] <- Z
 *          THRESH_BITS: out = uint64 [n][out_stride], ceil(M/64) words per row
 *                       <- bit c = (Z >= T[c]); needs T (int32 [M])
 *          SCALE_F32:   out = float [n][out_stride] <- alpha[c]*(float)Z; needs
 *                       alpha (float [M])
 * Covers the BMM.BBB / BMM.BBF variants of Section 3.1.2 (BIN and SCL folded
 * in; a scale before a re-binarization is dropped because it is positive). */
int bitgnn_bgemm(bitgnn_ctx *ctx, void *stream, const uint64_t *xbits, int64_t n,
                 int64_t x_stride, int32_t K, int32_t kwords, const uint64_t *wbits, int32_t M,
                 int64_t w_stride, int epilogue, const int32_t *T, const float *alpha, void *out,
                 int64_t out_stride);

/* The same product with full-precision activations, BIN folded in (the paper's
 * BMM.FBB / BMM.FBF): vx[i][k] = +1 if x[i*ldx + k] >= tau[k] (tau NULL = 0) else -1,
 * k < K; the packed activations are never materialized.  x: float [n][ldx];
 * wbits: uint64 [M][w_stride], ceil(K/64) words used.  Epilogues as bitgnn_bgemm. */
int bitgnn_bgemm_f32(bitgnn_ctx *ctx, void *stream, const float *x, int64_t n, int32_t K,
                     int64_t ldx, const float *tau, const uint64_t *wbits, int32_t M,
                     int64_t w_stride, int epilogue, const int32_t *T, const float *alpha,
                     void *out, int64_t out_stride);

/* ---- BSpMM: bit sparse product (Section 3.2.2; Algorithm 1) -------------- */

/* S[i][c] = sum_{j in N(i)} v[j][c] = 2*#{j in N(i) : bit c of hbits_j} - deg(i)
 * (trinary 0/1 x +-1 dot product, method 3) for c < C.
 * hbits: uint64 [N][h_stride].
 * epilogue RAW_I32:     out = int32 [N][out_stride] <- S
 *          THRESH_BITS: out = uint64 [N][out_stride], ceil(C/64) words per row
 *                       <- bit c = (S >= T[c]) (Algorithm 1's c >= 0 with the
 *                       BatchNorm threshold in place of 0); needs T (int32 [C]).
 * `out` may lie in the same rows as hbits as long as the words do not overlap. */
int bitgnn_bspmm(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const uint64_t *hbits,
                 int32_t C, int64_t h_stride, int epilogue, const int32_t *T, void *out,
                 int64_t out_stride);

/* bitgnn_bspmm for callers that cannot allocate device memory at all: code recorded under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as bitgnn_bspmm, but every scratch buffer of the kernels
 * (work counter, threshold seeds, degree-ordered activation rows, partial counters) lies
 * in a static device array of BITGNN_STATIC_SCRATCH_BYTES that each GPU the library runs
 * on holds until the process ends; neither this call nor anything it launches allocates,
 * frees or synchronizes, and the context's own workspace is not used.
 * Limit: bitgnn_adj_workspace_bytes(adj, C, 1) must fit in the array minus 16 KB of fixed
 * tables, else BITGNN_ERR_UNSUPPORTED (message gives both sizes).
 * All calls on one GPU, from any context, share that GPU's array: calls that overlap in
 * time on one GPU race; run them one after the other on a stream. */
#define BITGNN_STATIC_SCRATCH_BYTES (32u << 20)
int bitgnn_bspmm_static(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                        const uint64_t *hbits, int32_t C, int64_t h_stride, int epilogue,
                        const int32_t *T, void *out, int64_t out_stride);

/* Aggregation of integer activations over the 0/1 adjacency (the last layer's
 * BSpMM.FBF of the binary-aggregation model, kept in exact integers):
 * Y[i][c] = sum_{j in N(i)} Z[j][c], c < M.  Z: int32 [N][z_stride].
 * alpha != NULL: out = float [N][out_stride] <- alpha[c]*(float)Y
 * alpha == NULL: out = int32 [N][out_stride] <- Y
 * z_abs_bound: the caller's bound on |Z| (e.g. K); the call fails with
 * BITGNN_ERR_RANGE if max_degree * z_abs_bound >= 2^31. */
int bitgnn_spmm_i32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const int32_t *Z,
                    int32_t M, int64_t z_stride, int64_t z_abs_bound, const float *alpha,
                    void *out, int64_t out_stride);

/* Weighted / full-precision aggregation: the BSpMM variants of Section 3.1.1 whose
 * activation operand or output is full precision, and the weighted adjacency as the
 * 0/1 matrix times its factorisation vectors:
 *   Y[i][c] = r[i] * sum_{j in N(i)} f[j] * x[j][c],  c < C.
 * x: x_is_bits == 0: float [N][ldx];  x_is_bits != 0: packed +-1 rows, uint64 [N][ldx]
 *    (pad bits zero).  r, f: float [N] or NULL (= 1): D^-1/2 A D^-1/2 is
 *    r = f = deg^-1/2, the mean aggregator is r = 1/deg.
 * epilogue SCALE_F32:   out = float [N][ldo] <- Y
 *          THRESH_BITS: out = uint64 [N][ldo], ceil(C/64) words per row,
 *                       bit c = (Y >= tau[c]); needs tau (float [C]); pad bits zero.
 * Arithmetic: float, one rounded multiply and one rounded add per neighbour in the
 * order of bitgnn_adj_csr's column indices, then one multiply by r[i]; no fused
 * multiply-add.  Results are therefore bit-reproducible.  x and out must not overlap.
 * All pointers are device pointers owned by the caller; asynchronous on `stream`. */
int bitgnn_spmm_f32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const void *x,
                    int x_is_bits, int32_t C, int64_t ldx, const float *r, const float *f,
                    int epilogue, const float *tau, void *out, int64_t ldo);

/* ADD, the auxiliary merge of two activation tensors (Section 3.1.2: ADD.BBF and ADD.FFF
 * merge the self-connectivity of GraphSAGE), with BIN optionally folded in:
 *   y[i][c] = a[i][c] + b[i][c],  c < C,  one rounded float addition.
 * a, b: x_is_bits == 0: float [n][ld];  != 0: packed +-1 rows, uint64 [n][ld] (read as
 *       +1.0 / -1.0; ADD.BBF is both operands in bits).
 * epilogue SCALE_F32:   out = float [n][ldo] <- y
 *          THRESH_BITS: out = uint64 [n][ldo], ceil(C/64) words per row, bit c = (y >= tau[c]),
 *                       pad bits zero; needs tau (float [C]).
 * out must not overlap a or b.  n == 0 is a no-op.
 * All pointers are device pointers owned by the caller; asynchronous on `stream`. */
int bitgnn_add(bitgnn_ctx *ctx, void *stream, const void *a, int a_is_bits, int64_t lda,
               const void *b, int b_is_bits, int64_t ldb, int64_t n, int32_t C, int epilogue,
               const float *tau, void *out, int64_t ldo);

/* The same aggregation on the output of a BMM kept as integers with its scale (BMM + SCL
 * feeding a full-precision BSpMM): x[j][c] = alpha[c] * (float)z[j][c], one rounded
 * multiply -- the value the BMM's SCALE_F32 epilogue stores -- then as bitgnn_spmm_f32 with
 * float rows; the result is identical to scaling first and aggregating the floats, from
 * half the gathered bytes.  z: int16 [N][ldz] (ldz in int16 elements), 4-byte aligned;
 * alpha: float [C].  Other arguments, epilogues and errors as bitgnn_spmm_f32. */
int bitgnn_spmm_i16(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const int16_t *z,
                    int32_t C, int64_t ldz, const float *alpha, const float *r, const float *f,
                    int epilogue, const float *tau, void *out, int64_t ldo);

/* ---- layers (Section 3.1.2 high-level functions; Table 3 caption recipe) - */

/* GCN hidden layer, BMM.xBB + BSpMM.BBB:
 *   h = (xbits W >= T_mm) ; out = (A_hat h >= T_agg).
 * tmp_bits: caller scratch uint64 [N][ceil(M/64)] for h. */
int bitgnn_gcn_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const uint64_t *xbits,
                     int64_t x_stride, int32_t K, int32_t kwords, const uint64_t *wbits,
                     int32_t M, int64_t w_stride, const int32_t *T_mm, const int32_t *T_agg,
                     uint64_t *tmp_bits, uint64_t *out_bits, int64_t out_stride);
/* First GCN layer on float features, the paper's BMM.FBB + BSpMM.BBB:
 *   h = (bin(x) W >= T_mm) ; out = (A_hat h >= T_agg).  x: float [N][ldx]. */
int bitgnn_gcn_layer_f32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const float *x,
                         int32_t K, int64_t ldx, const float *tau, const uint64_t *wbits,
                         int32_t M, int64_t w_stride, const int32_t *T_mm, const int32_t *T_agg,
                         uint64_t *tmp_bits, uint64_t *out_bits, int64_t out_stride);
/* GCN output layer, BMM.BBF + BSpMM.FBF with one scale at the end:
 *   logits = alpha * (A_hat (xbits W)).  tmp_i32: caller scratch int32 [N][M].
 * No non-linearity sits between the two products, so when the handle has the
 * column-blocked form and K <= 128 the call evaluates (A_hat xbits) W instead: the
 * same integers, aggregated on 1-bit rows. */
int bitgnn_gcn_out_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                         const uint64_t *xbits, int64_t x_stride, int32_t K, int32_t kwords,
                         const uint64_t *wbits, int32_t M, int64_t w_stride, const float *alpha,
                         int32_t *tmp_i32, float *logits, int64_t ldo);
/* GraphSAGE / GraphConv hidden layer in concatenated form (sum aggregation,
 * Section 2.1):  nb = (A self >= T_agg) ; out = ([self | nb] W >= T_mm).
 * cat_bits: uint64 [N][2*kw] with kw = ceil(K_in/64); words [0, kw) of a row
 * hold the node's own bits on entry, words [kw, 2kw) receive nb.  wbits is
 * [M][2*kw] laid out the same way (K = 2*K_in logical bits). */
int bitgnn_sage_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, uint64_t *cat_bits,
                      int32_t K_in, const uint64_t *wbits, int32_t M, int64_t w_stride,
                      const int32_t *T_agg, const int32_t *T_mm, uint64_t *out_bits,
                      int64_t out_stride);
/* GraphSAGE output layer: logits = alpha * ([self | nb] W). */
int bitgnn_sage_out_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                          uint64_t *cat_bits, int32_t K_in, const uint64_t *wbits, int32_t M,
                          int64_t w_stride, const int32_t *T_agg, const float *alpha,
                          float *logits, int64_t ldo);

/* The two hidden layers with a weighted adjacency diag(r) A diag(f) (Section 3.1.1:
 * factorisation vectors; r = f = deg^-1/2: symmetric normalisation, r = 1/deg: mean
 * aggregator).  r, f: float [N] or NULL (= 1); tau_agg: float thresholds of the
 * aggregation, one per aggregated channel.  The weighted sum is bitgnn_spmm_f32's.
 *   GCN:  h = (xbits W >= T_mm) ; out = (r .* (A_hat (f .* h)) >= tau_agg)
 *   SAGE: nb = (r .* (A (f .* self)) >= tau_agg) ; out = ([self | nb] W >= T_mm)
 * Other arguments as in bitgnn_gcn_layer / bitgnn_sage_layer. */
int bitgnn_gcn_layer_weighted(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                              const uint64_t *xbits, int64_t x_stride, int32_t K, int32_t kwords,
                              const uint64_t *wbits, int32_t M, int64_t w_stride,
                              const int32_t *T_mm, const float *r, const float *f,
                              const float *tau_agg, uint64_t *tmp_bits, uint64_t *out_bits,
                              int64_t out_stride);
int bitgnn_sage_layer_weighted(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                               uint64_t *cat_bits, int32_t K_in, const uint64_t *wbits, int32_t M,
                               int64_t w_stride, const float *r, const float *f,
                               const float *tau_agg, const int32_t *T_mm, uint64_t *out_bits,
                               int64_t out_stride);
/* GCN output layer with the weighted adjacency:
 *   logits = r .* (A_hat (f .* (alpha .* (xbits W)))),
 * BMM.BBF with its scale, then the full-precision weighted aggregation.
 * tmp_f32: caller scratch of N*M floats (contents unspecified afterwards).  Other
 * arguments as in bitgnn_gcn_out_layer. */
int bitgnn_gcn_out_layer_weighted(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                  const uint64_t *xbits, int64_t x_stride, int32_t K,
                                  int32_t kwords, const uint64_t *wbits, int32_t M,
                                  int64_t w_stride, const float *alpha, const float *r,
                                  const float *f, float *tmp_f32, float *logits, int64_t ldo);

/* GCN hidden layer with full-precision aggregation (Table 3's "Ours (full)" recipe, the
 * aggregation of Bi-GCN: products binarized, aggregation not), BMM.xBF + BSpMM.FBB:
 *   z = alpha .* (xbits W)  (float);  out = (r .* (A_hat (f .* z)) >= tau_agg).
 * alpha: float [M] scale of the product;  r, f: float [N] or NULL (= 1);  tau_agg: float
 * [M] (the BatchNorm + BIN after the aggregation, folded);  tmp_f32: caller scratch of
 * N*M floats (holds the product as int16 rows when K <= 32767, as float rows otherwise).
 * The float sum is bitgnn_spmm_f32's (step-rounded, reproducible). */
int bitgnn_gcn_layer_full(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                          const uint64_t *xbits, int64_t x_stride, int32_t K, int32_t kwords,
                          const uint64_t *wbits, int32_t M, int64_t w_stride, const float *alpha,
                          const float *r, const float *f, const float *tau_agg, float *tmp_f32,
                          uint64_t *out_bits, int64_t out_stride);
/* The same on float features (BMM.FBF + BSpMM.FBB): x float [N][ldx], binarized by
 * x >= tau_in[k] (tau_in NULL: x >= 0) inside the product. */
int bitgnn_gcn_layer_full_f32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                              const float *x, int32_t K, int64_t ldx, const float *tau_in,
                              const uint64_t *wbits, int32_t M, int64_t w_stride,
                              const float *alpha, const float *r, const float *f,
                              const float *tau_agg, float *tmp_f32, uint64_t *out_bits,
                              int64_t out_stride);

/* ---- tuning utilities (Section 3.4) --------------------------------------- */

/* Type check of a chain of functions in the paper's notation (Section 3.1.2), e.g.
 * "MM.FBB BSpMM.BBB MM.BBF BSpMM.FBF": names BMM / MM, BSpMM / SpMM, ADD, each with a
 * three-letter suffix <input><second operand><output> of F (full precision) and B (binary);
 * separators are spaces, ',', '+' or '>'.  The chain is well typed when every function's
 * output precision is its successor's input precision, and the weight / adjacency operand
 * of a BMM / BSpMM is B: then one variant may replace another.  Host-only; works on any
 * context.  Returns BITGNN_OK, or BITGNN_ERR_INVALID_ARG with *bad_index (may be NULL) =
 * position of the first offending function (0-based) and the reason in bitgnn_last_error. */
int bitgnn_chain_check(bitgnn_ctx *ctx, const char *chain, int32_t *bad_index);

/* Measures the two recipes of a GCN hidden layer of width K -> M on this graph, `reps`
 * timed runs each after one untimed run, on scratch inputs of the right shape:
 *   *bin_ms  <- BMM.BBB + BSpMM.BBB   (bitgnn_gcn_layer, binary aggregation)
 *   *full_ms <- BMM.BBF + BSpMM.FBB   (bitgnn_gcn_layer_full, full-precision aggregation)
 * in milliseconds per layer (host pointers, may be NULL).  The recipes differ in accuracy,
 * so the choice stays with the caller.  Allocates and frees its scratch (about
 * N * (K/8 + M/4 + 4 M) bytes) and synchronizes the stream: a set-up call. */
int bitgnn_gcn_layer_tune(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, int32_t K,
                          int32_t M, int32_t reps, float *bin_ms, float *full_ms);

/* ---- whole model in one launch (Section 3.3: the end-to-end fused kernel) - */

/* Range of bitgnn_gcn2_fused (larger inputs are not launch-bound: use the layer calls). */
#define BITGNN_FUSED_MAX_NODES 65536
#define BITGNN_FUSED_MAX_DEGREE 1024
#define BITGNN_FUSED_MAX_HIDDEN 256
#define BITGNN_FUSED_MAX_CLASSES 64

/* Two-layer GCN on float features in ONE kernel launch, for small graphs: the same
 * result as bitgnn_gcn_layer_f32 (tau = NULL) followed by bitgnn_gcn_out_layer,
 *   h  = (bin(x) W1 >= T_mm);  h1 = (A_hat h >= T_agg);  logits = alpha .* (A_hat (h1 W2)),
 * with grid-wide barriers inside the kernel where those calls have kernel boundaries
 * (the cooperative whole-model kernel of Section 3.3).  Integers and bits are exact, so
 * the outputs are identical to the layer calls'.
 * x: float [N][ldx], K0 features.  w1bits: uint64 [C1][w1_stride] (K0 bits per row),
 * w2bits: uint64 [M][w2_stride] (C1 bits per row), pad bits zero (bitgnn_pack_weights_i8).
 * T_mm, T_agg: int32 [C1].  alpha: float [M].
 * tmp_bits: caller scratch uint64 [N][ceil(C1/64)] (dense) <- h.
 * h_bits:   uint64 [N][h_stride] <- h1 (an output: ceil(C1/64) words per row, pad bits 0).
 * logits:   float [N][ldo].
 * status:   device int32 or NULL.  The kernel's waits are bounded (seconds); if one is
 *           ever abandoned (the grid could not become resident: compute units taken away
 *           from the process), the kernel adds 1 to *status, skips the remaining work and
 *           exits; logits and h_bits are then undefined.  Never cleared by the library.
 * Errors: BITGNN_ERR_RANGE beyond the limits above (N, largest degree, C1, M), with the
 * limits in the message; BITGNN_ERR_INVALID_ARG / BITGNN_ERR_ALIGNMENT as elsewhere.
 * One fused call at a time per context (the barrier counter lives in the context), and no
 * fused call of another context running at the same time on another stream: each grid
 * waits inside the kernel for all of its workgroups, so two such grids can hold the compute
 * units the other needs (the bounded waits then expire and *status says so).  Ordinary
 * kernels on other streams only delay it.  The call is
 * asynchronous on `stream` like every other call, allocates
 * nothing, keeps no host state and is one kernel launch, so it may be recorded into a HIP
 * graph and replayed.  All pointers are device pointers owned
 * by the caller. */
/* Bound on the polls (~1 us each) of one wait at a barrier of bitgnn_gcn2_fused before
 * the wait is abandoned; default 2^22.  polls >= 1.  A tiny bound makes workgroups that
 * arrive early give up: the way to exercise the abandoned-wait path (status raised, every
 * workgroup still exits, the next call works) without taking compute units away. */
int bitgnn_ctx_set_fused_spin_limit(bitgnn_ctx *ctx, uint32_t polls);

int bitgnn_gcn2_fused(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj, const float *x,
                      int32_t K0, int64_t ldx, const uint64_t *w1bits, int32_t C1,
                      int64_t w1_stride, const int32_t *T_mm, const int32_t *T_agg,
                      const uint64_t *w2bits, int32_t M, int64_t w2_stride, const float *alpha,
                      uint64_t *tmp_bits, uint64_t *h_bits, int64_t h_stride, float *logits,
                      int64_t ldo, int32_t *status);

#ifdef __cplusplus
}
#endif
#endif /* BITGNN_H */
