// Layer drivers: the high-level functions of Section 3.1.2 (a BMM followed by a
// BSpMM for GCN; an aggregation, a concatenation and a BMM for GraphSAGE /
// GraphConv), in the "binary aggregation" recipe of Table 3's caption.  They
// only validate and enqueue the kernels of the other files on one stream.
#include "common.h"

extern "C" int bitgnn_gcn_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                const uint64_t *xbits, int64_t x_stride, int32_t K, int32_t kwords,
                                const uint64_t *wbits, int32_t M, int64_t w_stride,
                                const int32_t *T_mm, const int32_t *T_agg, uint64_t *tmp_bits,
                                uint64_t *out_bits, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_layer: adj is null");
    const int64_t n = adj->n;
    const int64_t mw = ((int64_t)M + 63) / 64;
    int rc = bg_check_bgemm(ctx, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                            BITGNN_EPI_THRESH_BITS, T_mm, nullptr, tmp_bits, mw);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_bspmm(ctx, adj, tmp_bits, M, mw, BITGNN_EPI_THRESH_BITS, T_agg, out_bits,
                        out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    rc = bg_launch_bgemm(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                         BITGNN_EPI_THRESH_BITS, T_mm, nullptr, tmp_bits, mw);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_bspmm(ctx, s, adj, tmp_bits, M, mw, BITGNN_EPI_THRESH_BITS, T_agg, out_bits,
                           out_stride);
}

extern "C" int bitgnn_gcn_layer_f32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                    const float *x, int32_t K, int64_t ldx, const float *tau,
                                    const uint64_t *wbits, int32_t M, int64_t w_stride,
                                    const int32_t *T_mm, const int32_t *T_agg, uint64_t *tmp_bits,
                                    uint64_t *out_bits, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_layer_f32: adj is null");
    const int64_t n = adj->n;
    const int64_t mw = ((int64_t)M + 63) / 64;
    int rc = bg_check_bgemm_f32(ctx, x, n, K, ldx, tau, wbits, M, w_stride, BITGNN_EPI_THRESH_BITS,
                                T_mm, nullptr, tmp_bits, mw);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_bspmm(ctx, adj, tmp_bits, M, mw, BITGNN_EPI_THRESH_BITS, T_agg, out_bits,
                        out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    rc = bg_launch_bgemm_f32(ctx, s, x, n, K, ldx, tau, wbits, M, w_stride, BITGNN_EPI_THRESH_BITS,
                             T_mm, nullptr, tmp_bits, mw);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_bspmm(ctx, s, adj, tmp_bits, M, mw, BITGNN_EPI_THRESH_BITS, T_agg, out_bits,
                           out_stride);
}

extern "C" int bitgnn_gcn_out_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                    const uint64_t *xbits, int64_t x_stride, int32_t K,
                                    int32_t kwords, const uint64_t *wbits, int32_t M,
                                    int64_t w_stride, const float *alpha, int32_t *tmp_i32,
                                    float *logits, int64_t ldo)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_out_layer: adj is null");
    BG_REQUIRE(ctx, alpha, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_out_layer: alpha is null");
    const int64_t n = adj->n;
    int rc = bg_check_bgemm(ctx, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                            BITGNN_EPI_RAW_I32, nullptr, nullptr, tmp_i32, M);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_spmm_i32(ctx, adj, tmp_i32, M, M, K, logits, ldo);
    if (rc != BITGNN_OK)
        return rc;
    BG_REQUIRE(ctx, bg_aligned(alpha, 4), BITGNN_ERR_ALIGNMENT,
               "bitgnn_gcn_out_layer: misaligned alpha");
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    // No non-linearity sits between the two products, so A_hat (x W) = (A_hat x) W in
    // exact integers.  With the blocked form the aggregation runs first, on 1-bit rows
    // staged in LDS (128 channels per pass), and the class projection is fused into its
    // merge step (tmp_i32 chains the integer sums of the passes when K > 128); otherwise
    // the int32 rows of x W are aggregated directly.
    if ((int64_t)K * adj->max_degree < (1ll << 29) &&
        bg_prefer_blocked(adj, (K + 127) / 128, 4 * (int64_t)M, 0.25,
                          adj->max_degree < (int64_t)adj->seg_len ? adj->max_degree
                                                                  : (int64_t)adj->seg_len))
        return bg_launch_agg_project_blocked(ctx, s, adj, xbits, K, x_stride, wbits, M, w_stride,
                                             alpha, tmp_i32, logits, ldo);
    rc = bg_launch_bgemm(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                         BITGNN_EPI_RAW_I32, nullptr, nullptr, tmp_i32, M);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_spmm_i32(ctx, s, adj, tmp_i32, M, M, alpha, logits, ldo);
}

extern "C" int bitgnn_sage_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                 uint64_t *cat_bits, int32_t K_in, const uint64_t *wbits,
                                 int32_t M, int64_t w_stride, const int32_t *T_agg,
                                 const int32_t *T_mm, uint64_t *out_bits, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_sage_layer: adj is null");
    BG_REQUIRE(ctx, K_in >= 1 && K_in <= (1 << 29), BITGNN_ERR_INVALID_ARG,
               "bitgnn_sage_layer: K_in=%d", K_in);
    BG_REQUIRE(ctx, cat_bits, BITGNN_ERR_INVALID_ARG, "bitgnn_sage_layer: cat_bits is null");
    const int64_t n = adj->n;
    const int32_t kw = (K_in + 63) / 64;
    int rc = bg_check_bspmm(ctx, adj, cat_bits, K_in, 2 * kw, BITGNN_EPI_THRESH_BITS, T_agg,
                            cat_bits + kw, 2 * kw);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_bgemm(ctx, cat_bits, n, 2 * kw, 2 * K_in, 2 * kw, wbits, M, w_stride,
                        BITGNN_EPI_THRESH_BITS, T_mm, nullptr, out_bits, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    rc = bg_launch_bspmm(ctx, s, adj, cat_bits, K_in, 2 * kw, BITGNN_EPI_THRESH_BITS, T_agg,
                         cat_bits + kw, 2 * kw);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_bgemm(ctx, s, cat_bits, n, 2 * kw, 2 * K_in, 2 * kw, wbits, M, w_stride,
                           BITGNN_EPI_THRESH_BITS, T_mm, nullptr, out_bits, out_stride);
}

extern "C" int bitgnn_sage_out_layer(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                     uint64_t *cat_bits, int32_t K_in, const uint64_t *wbits,
                                     int32_t M, int64_t w_stride, const int32_t *T_agg,
                                     const float *alpha, float *logits, int64_t ldo)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_sage_out_layer: adj is null");
    BG_REQUIRE(ctx, K_in >= 1 && K_in <= (1 << 29), BITGNN_ERR_INVALID_ARG,
               "bitgnn_sage_out_layer: K_in=%d", K_in);
    BG_REQUIRE(ctx, cat_bits, BITGNN_ERR_INVALID_ARG, "bitgnn_sage_out_layer: cat_bits is null");
    const int64_t n = adj->n;
    const int32_t kw = (K_in + 63) / 64;
    int rc = bg_check_bspmm(ctx, adj, cat_bits, K_in, 2 * kw, BITGNN_EPI_THRESH_BITS, T_agg,
                            cat_bits + kw, 2 * kw);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_bgemm(ctx, cat_bits, n, 2 * kw, 2 * K_in, 2 * kw, wbits, M, w_stride,
                        BITGNN_EPI_SCALE_F32, nullptr, alpha, logits, ldo);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    rc = bg_launch_bspmm(ctx, s, adj, cat_bits, K_in, 2 * kw, BITGNN_EPI_THRESH_BITS, T_agg,
                         cat_bits + kw, 2 * kw);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_bgemm(ctx, s, cat_bits, n, 2 * kw, 2 * K_in, 2 * kw, wbits, M, w_stride,
                           BITGNN_EPI_SCALE_F32, nullptr, alpha, logits, ldo);
}

// Full-precision aggregation of a BMM's output alpha .* Z.  The float rows are not
// materialised: the BMM leaves its raw integers (|z| <= K) in the caller's float scratch,
// they are narrowed in place to int16 and the aggregation forms alpha_c * (float)z itself,
// with the same single rounding as the BMM's scale epilogue -- the same bits from half the
// gathered bytes, and the gathers are what bounds the aggregation.
static const int32_t kNarrowMaxK = 32767;
static int aggregate_scaled_integers(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj,
                                     float *scratch, int32_t M, const float *alpha, const float *r,
                                     const float *f, int epilogue, const float *tau, void *out,
                                     int64_t ldo)
{
    int rc = bg_launch_narrow_rows(ctx, s, (int32_t *)scratch, adj->n, M, M);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_spmm_f32(ctx, s, adj, scratch, 0, M, 2 * (int64_t)M, r, f, epilogue, tau, out,
                              ldo, alpha);
}

// The same two layers with a weighted adjacency, diag(r) A diag(f) (Section 3.1.1: a
// weighted adjacency is the 0/1 matrix times its factorisation vectors): r = f = deg^-1/2
// is the symmetric normalisation of GCN, r = 1/deg the mean aggregator of GraphSAGE.  The
// aggregation is the step-rounded float sum of bitgnn_spmm_f32 on the packed +-1 rows,
// binarized again with float thresholds.
extern "C" int bitgnn_gcn_layer_weighted(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                         const uint64_t *xbits, int64_t x_stride, int32_t K,
                                         int32_t kwords, const uint64_t *wbits, int32_t M,
                                         int64_t w_stride, const int32_t *T_mm, const float *r,
                                         const float *f, const float *tau_agg, uint64_t *tmp_bits,
                                         uint64_t *out_bits, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_layer_weighted: adj is null");
    const int64_t n = adj->n;
    const int64_t mw = ((int64_t)M + 63) / 64;
    int rc = bg_check_bgemm(ctx, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                            BITGNN_EPI_THRESH_BITS, T_mm, nullptr, tmp_bits, mw);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_spmm_f32(ctx, adj, tmp_bits, 1, M, mw, r, f, BITGNN_EPI_THRESH_BITS, tau_agg,
                           out_bits, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    rc = bg_launch_bgemm(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                         BITGNN_EPI_THRESH_BITS, T_mm, nullptr, tmp_bits, mw);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_spmm_f32(ctx, s, adj, tmp_bits, 1, M, mw, r, f, BITGNN_EPI_THRESH_BITS,
                              tau_agg, out_bits, out_stride, nullptr);
}

extern "C" int bitgnn_sage_layer_weighted(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                          uint64_t *cat_bits, int32_t K_in, const uint64_t *wbits,
                                          int32_t M, int64_t w_stride, const float *r,
                                          const float *f, const float *tau_agg,
                                          const int32_t *T_mm, uint64_t *out_bits,
                                          int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_sage_layer_weighted: adj is null");
    BG_REQUIRE(ctx, K_in >= 1 && K_in <= (1 << 29), BITGNN_ERR_INVALID_ARG,
               "bitgnn_sage_layer_weighted: K_in=%d", K_in);
    BG_REQUIRE(ctx, cat_bits, BITGNN_ERR_INVALID_ARG, "bitgnn_sage_layer_weighted: cat_bits is null");
    const int64_t n = adj->n;
    const int32_t kw = (K_in + 63) / 64;
    int rc = bg_check_spmm_f32(ctx, adj, cat_bits, 1, K_in, 2 * kw, r, f, BITGNN_EPI_THRESH_BITS,
                               tau_agg, cat_bits + kw, 2 * kw);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_bgemm(ctx, cat_bits, n, 2 * kw, 2 * K_in, 2 * kw, wbits, M, w_stride,
                        BITGNN_EPI_THRESH_BITS, T_mm, nullptr, out_bits, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    rc = bg_launch_spmm_f32(ctx, s, adj, cat_bits, 1, K_in, 2 * kw, r, f, BITGNN_EPI_THRESH_BITS,
                            tau_agg, cat_bits + kw, 2 * kw, nullptr);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_bgemm(ctx, s, cat_bits, n, 2 * kw, 2 * K_in, 2 * kw, wbits, M, w_stride,
                           BITGNN_EPI_THRESH_BITS, T_mm, nullptr, out_bits, out_stride);
}

// Output layer with a weighted adjacency: logits = diag(r) A_hat diag(f) (alpha .* (xbits W)).
// BMM.BBF with its scale writes float rows into the caller's scratch, the full-precision
// weighted aggregation follows (BSpMM with a float activation operand and float output).
extern "C" int bitgnn_gcn_out_layer_weighted(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                             const uint64_t *xbits, int64_t x_stride, int32_t K,
                                             int32_t kwords, const uint64_t *wbits, int32_t M,
                                             int64_t w_stride, const float *alpha, const float *r,
                                             const float *f, float *tmp_f32, float *logits,
                                             int64_t ldo)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_out_layer_weighted: adj is null");
    const int64_t n = adj->n;
    int rc = bg_check_bgemm(ctx, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                            BITGNN_EPI_SCALE_F32, nullptr, alpha, tmp_f32, M);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_spmm_f32(ctx, adj, tmp_f32, 0, M, M, r, f, BITGNN_EPI_SCALE_F32, nullptr, logits,
                           ldo);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    if (K <= kNarrowMaxK) {
        rc = bg_launch_bgemm(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                             BITGNN_EPI_RAW_I32, nullptr, nullptr, tmp_f32, M);
        if (rc != BITGNN_OK)
            return rc;
        return aggregate_scaled_integers(ctx, s, adj, tmp_f32, M, alpha, r, f,
                                         BITGNN_EPI_SCALE_F32, nullptr, logits, ldo);
    }
    rc = bg_launch_bgemm(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                         BITGNN_EPI_SCALE_F32, nullptr, alpha, tmp_f32, M);
    if (rc != BITGNN_OK)
        return rc;
    return bg_launch_spmm_f32(ctx, s, adj, tmp_f32, 0, M, M, r, f, BITGNN_EPI_SCALE_F32, nullptr,
                              logits, ldo, nullptr);
}

// GCN hidden layer of the full-precision-aggregation recipe (Table 3's "Ours (full)": the
// products are binarized, the aggregation is not): BMM.xBF with its scale writes float rows
// into the caller's scratch, BSpMM.FBB aggregates them over the weighted adjacency
// diag(r) A_hat diag(f) in floats and binarizes the result with float thresholds (the
// BatchNorm + BIN that follow, folded).
static int gcn_layer_full_tail(bitgnn_ctx *ctx, hipStream_t s, const bitgnn_adj *adj,
                               const float *tmp_f32, int32_t M, const float *r, const float *f,
                               const float *tau_agg, uint64_t *out_bits, int64_t out_stride)
{
    return bg_launch_spmm_f32(ctx, s, adj, tmp_f32, 0, M, M, r, f, BITGNN_EPI_THRESH_BITS,
                              tau_agg, out_bits, out_stride, nullptr);
}

extern "C" int bitgnn_gcn_layer_full(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                     const uint64_t *xbits, int64_t x_stride, int32_t K,
                                     int32_t kwords, const uint64_t *wbits, int32_t M,
                                     int64_t w_stride, const float *alpha, const float *r,
                                     const float *f, const float *tau_agg, float *tmp_f32,
                                     uint64_t *out_bits, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_layer_full: adj is null");
    const int64_t n = adj->n;
    int rc = bg_check_bgemm(ctx, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                            BITGNN_EPI_SCALE_F32, nullptr, alpha, tmp_f32, M);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_spmm_f32(ctx, adj, tmp_f32, 0, M, M, r, f, BITGNN_EPI_THRESH_BITS, tau_agg,
                           out_bits, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    if (K <= kNarrowMaxK) {
        rc = bg_launch_bgemm(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                             BITGNN_EPI_RAW_I32, nullptr, nullptr, tmp_f32, M);
        if (rc != BITGNN_OK)
            return rc;
        return aggregate_scaled_integers(ctx, s, adj, tmp_f32, M, alpha, r, f,
                                         BITGNN_EPI_THRESH_BITS, tau_agg, out_bits, out_stride);
    }
    rc = bg_launch_bgemm(ctx, s, xbits, n, x_stride, K, kwords, wbits, M, w_stride,
                         BITGNN_EPI_SCALE_F32, nullptr, alpha, tmp_f32, M);
    if (rc != BITGNN_OK)
        return rc;
    return gcn_layer_full_tail(ctx, s, adj, tmp_f32, M, r, f, tau_agg, out_bits, out_stride);
}

extern "C" int bitgnn_gcn_layer_full_f32(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                         const float *x, int32_t K, int64_t ldx,
                                         const float *tau_in, const uint64_t *wbits, int32_t M,
                                         int64_t w_stride, const float *alpha, const float *r,
                                         const float *f, const float *tau_agg, float *tmp_f32,
                                         uint64_t *out_bits, int64_t out_stride)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_layer_full_f32: adj is null");
    const int64_t n = adj->n;
    int rc = bg_check_bgemm_f32(ctx, x, n, K, ldx, tau_in, wbits, M, w_stride,
                                BITGNN_EPI_SCALE_F32, nullptr, alpha, tmp_f32, M);
    if (rc != BITGNN_OK)
        return rc;
    rc = bg_check_spmm_f32(ctx, adj, tmp_f32, 0, M, M, r, f, BITGNN_EPI_THRESH_BITS, tau_agg,
                           out_bits, out_stride);
    if (rc != BITGNN_OK)
        return rc;
    BG_NEED_DEVICE(ctx);
    hipStream_t s = (hipStream_t)stream;
    if (K <= kNarrowMaxK) {
        rc = bg_launch_bgemm_f32(ctx, s, x, n, K, ldx, tau_in, wbits, M, w_stride,
                                 BITGNN_EPI_RAW_I32, nullptr, nullptr, tmp_f32, M);
        if (rc != BITGNN_OK)
            return rc;
        return aggregate_scaled_integers(ctx, s, adj, tmp_f32, M, alpha, r, f,
                                         BITGNN_EPI_THRESH_BITS, tau_agg, out_bits, out_stride);
    }
    rc = bg_launch_bgemm_f32(ctx, s, x, n, K, ldx, tau_in, wbits, M, w_stride,
                             BITGNN_EPI_SCALE_F32, nullptr, alpha, tmp_f32, M);
    if (rc != BITGNN_OK)
        return rc;
    return gcn_layer_full_tail(ctx, s, adj, tmp_f32, M, r, f, tau_agg, out_bits, out_stride);
}
