// Tuning utilities (Section 3.4): the type check that lets one variant of a function be
// swapped for another (a chain of functions is well typed when every function's output
// precision is its successor's input precision, Section 3.1.2), and a run that measures the
// two recipes of a GCN hidden layer on the caller's graph.
#include "common.h"

#include <ctype.h>

namespace {

struct TuneMem { // device scratch of a tuning run, released on every return path
    void *p = nullptr;
    ~TuneMem()
    {
        if (p)
            (void)hipFree(p);
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 8); }
};

enum OpKind { OP_BMM, OP_BSPMM, OP_ADD, OP_NONE };

OpKind op_kind(const char *name, size_t len)
{
    auto is = [&](const char *s) { return strlen(s) == len && !strncmp(name, s, len); };
    if (is("BMM") || is("MM"))
        return OP_BMM;
    if (is("BSpMM") || is("SpMM"))
        return OP_BSPMM;
    if (is("ADD"))
        return OP_ADD;
    return OP_NONE;
}

} // namespace

extern "C" int bitgnn_chain_check(bitgnn_ctx *ctx, const char *chain, int32_t *bad_index)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    if (bad_index)
        *bad_index = -1;
    BG_REQUIRE(ctx, chain, BITGNN_ERR_INVALID_ARG, "bitgnn_chain_check: chain is null");
    const char *p = chain;
    char prev_out = 0;
    int32_t index = 0;
    for (;; ++index) {
        while (*p && (isspace((unsigned char)*p) || *p == ',' || *p == '+' || *p == '>'))
            ++p;
        if (!*p)
            break;
        const char *name = p;
        while (*p && *p != '.' && !isspace((unsigned char)*p) && *p != ',' && *p != '+' &&
               *p != '>')
            ++p;
        const OpKind kind = op_kind(name, (size_t)(p - name));
        if (bad_index)
            *bad_index = index;
        BG_REQUIRE(ctx, kind != OP_NONE, BITGNN_ERR_INVALID_ARG,
                   "bitgnn_chain_check: function %d: unknown name '%.*s' (BMM, MM, BSpMM, SpMM, ADD)",
                   index, (int)(p - name), name);
        BG_REQUIRE(ctx, p[0] == '.' && p[1] && p[2] && p[3], BITGNN_ERR_INVALID_ARG,
                   "bitgnn_chain_check: function %d: expected a three-letter precision suffix",
                   index);
        const char in1 = p[1], in2 = p[2], out = p[3];
        p += 4;
        BG_REQUIRE(ctx,
                   (in1 == 'F' || in1 == 'B') && (in2 == 'F' || in2 == 'B') &&
                       (out == 'F' || out == 'B') &&
                       (!*p || isspace((unsigned char)*p) || *p == ',' || *p == '+' || *p == '>'),
                   BITGNN_ERR_INVALID_ARG,
                   "bitgnn_chain_check: function %d: suffix must be three letters of F and B",
                   index);
        BG_REQUIRE(ctx, kind == OP_ADD || in2 == 'B', BITGNN_ERR_INVALID_ARG,
                   "bitgnn_chain_check: function %d: the %s operand of a binary %s is B", index,
                   kind == OP_BMM ? "weight" : "adjacency", kind == OP_BMM ? "BMM" : "BSpMM");
        BG_REQUIRE(ctx, !prev_out || prev_out == in1, BITGNN_ERR_INVALID_ARG,
                   "bitgnn_chain_check: function %d takes %c but its predecessor produces %c",
                   index, in1, prev_out);
        prev_out = out;
    }
    BG_REQUIRE(ctx, index > 0, BITGNN_ERR_INVALID_ARG, "bitgnn_chain_check: empty chain");
    if (bad_index)
        *bad_index = -1;
    return BITGNN_OK;
}

extern "C" int bitgnn_gcn_layer_tune(bitgnn_ctx *ctx, void *stream, const bitgnn_adj *adj,
                                     int32_t K, int32_t M, int32_t reps, float *bin_ms,
                                     float *full_ms)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, adj, BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_layer_tune: adj is null");
    BG_REQUIRE(ctx, K >= 1 && K <= (1 << 20) && M >= 1 && M <= (1 << 16) && reps >= 1 &&
                        reps <= 1000,
               BITGNN_ERR_INVALID_ARG, "bitgnn_gcn_layer_tune: K=%d M=%d reps=%d (1..1000)", K, M,
               reps);
    BG_NEED_DEVICE(ctx);
    if (bin_ms)
        *bin_ms = -1.0f;
    if (full_ms)
        *full_ms = -1.0f;
    const int64_t n = adj->n;
    if (n == 0)
        return BITGNN_OK;
    hipStream_t s = (hipStream_t)stream;
    const int32_t kw = (K + 63) / 64;
    const int64_t mw = ((int64_t)M + 63) / 64;
    { // a set-up call: it may grow the aggregation workspace
        const int rc_ws =
            bitgnn_ctx_reserve(ctx, bg_adj_workspace_bytes(adj, M > 2048 ? 2048 : M, M));
        if (rc_ws != BITGNN_OK)
            return rc_ws;
    }
    TuneMem x, w, tmp_bits, out, tmp_f32, vecs;
    BG_HIP(ctx, x.alloc((size_t)n * kw * 8));
    BG_HIP(ctx, w.alloc((size_t)M * kw * 8));
    BG_HIP(ctx, tmp_bits.alloc((size_t)n * mw * 8));
    BG_HIP(ctx, out.alloc((size_t)n * mw * 8));
    BG_HIP(ctx, tmp_f32.alloc((size_t)n * M * 4));
    // zeros serve as thresholds (int32 and float alike); 0x3F3F3F3F is a float near 0.75 for
    // the scales and factors; the bit patterns of x and w only have to be there
    const size_t vec_floats = (size_t)(M > n ? M : n);
    BG_HIP(ctx, vecs.alloc(2 * vec_floats * 4));
    float *zeros = (float *)vecs.p, *pos = (float *)vecs.p + vec_floats;
    BG_HIP(ctx, hipMemsetAsync(x.p, 0x5A, (size_t)n * kw * 8, s));
    BG_HIP(ctx, hipMemsetAsync(w.p, 0x33, (size_t)M * kw * 8, s));
    BG_HIP(ctx, hipMemsetAsync(zeros, 0, vec_floats * 4, s));
    BG_HIP(ctx, hipMemsetAsync(pos, 0x3F, vec_floats * 4, s));
    // the timing run multiplies whole words: the fill patterns would otherwise leave pad
    // bits set, which the BMM's contract forbids (the time does not depend on it)
    const int32_t K_whole = kw * 64;
    hipEvent_t e0, e1;
    BG_HIP(ctx, hipEventCreate(&e0));
    BG_HIP(ctx, hipEventCreate(&e1));
    float ms[2] = {-1.0f, -1.0f};
    int rc = BITGNN_OK;
    for (int variant = 0; variant < 2 && rc == BITGNN_OK; ++variant) {
        for (int i = 0; i <= reps && rc == BITGNN_OK; ++i) { // one untimed call first
            if (i == 1)
                (void)hipEventRecord(e0, s);
            if (variant == 0)
                rc = bitgnn_gcn_layer(ctx, s, adj, (const uint64_t *)x.p, kw, K_whole, kw,
                                      (const uint64_t *)w.p, M, kw, (const int32_t *)zeros,
                                      (const int32_t *)zeros, (uint64_t *)tmp_bits.p,
                                      (uint64_t *)out.p, mw);
            else
                rc = bitgnn_gcn_layer_full(ctx, s, adj, (const uint64_t *)x.p, kw, K_whole, kw,
                                           (const uint64_t *)w.p, M, kw, pos, pos, pos, zeros,
                                           (float *)tmp_f32.p, (uint64_t *)out.p, mw);
        }
        if (rc != BITGNN_OK)
            break;
        (void)hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess) {
            rc = bitgnn_fail(ctx, BITGNN_ERR_HIP, "bitgnn_gcn_layer_tune: event synchronize failed");
            break;
        }
        (void)hipEventElapsedTime(&ms[variant], e0, e1);
        ms[variant] /= (float)reps;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipStreamSynchronize(s);
    if (rc != BITGNN_OK)
        return rc;
    if (bin_ms)
        *bin_ms = ms[0];
    if (full_ms)
        *full_ms = ms[1];
    return BITGNN_OK;
}
