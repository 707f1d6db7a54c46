// Context life cycle and error reporting.
#include "common.h"

#include <stdlib.h>

// Largest seed table the bit-SpMM may ask for: 2 parities x 26 planes x 64 words.
static const size_t kSeedTableWords = 2 * 26 * 64;

extern "C" int bitgnn_ctx_create(bitgnn_ctx **out, int device)
{
    if (!out || device < -1)
        return BITGNN_ERR_INVALID_ARG;
    bitgnn_ctx *ctx = (bitgnn_ctx *)calloc(1, sizeof(bitgnn_ctx));
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    ctx->device = device;
    ctx->cb_nodes = 8192;
    ctx->part_len = 255;
    ctx->min_avg_degree = 8;
    ctx->fused_spin_limit = 1u << 22;
    if (const char *e = getenv("BITGNN_BGEMM"))
        ctx->bgemm_path = !strcmp(e, "valu") ? 1 : !strcmp(e, "mfma") ? 2 : 0;
    if (device >= 0) {
        int count = 0;
        hipError_t e = hipGetDeviceCount(&count);
        if (e != hipSuccess || device >= count) {
            free(ctx);
            return BITGNN_ERR_HIP;
        }
        e = hipSetDevice(device);
        if (e == hipSuccess)
            e = hipDeviceGetAttribute(&ctx->n_cus, hipDeviceAttributeMultiprocessorCount, device);
        if (e == hipSuccess)
            e = hipMalloc((void **)&ctx->queue, 256);
        if (e == hipSuccess)
            e = hipMemset(ctx->queue, 0, 256);
        if (e == hipSuccess)
            e = hipMalloc((void **)&ctx->seed_table, kSeedTableWords * sizeof(uint32_t));
        if (e != hipSuccess) {
            free(ctx);
            return BITGNN_ERR_HIP;
        }
        ctx->seed_table_words = kSeedTableWords;
    }
    *out = ctx;
    return BITGNN_OK;
}

extern "C" void bitgnn_ctx_destroy(bitgnn_ctx *ctx)
{
    if (!ctx)
        return;
    if (ctx->seed_table)
        (void)hipFree(ctx->seed_table);
    if (ctx->queue)
        (void)hipFree(ctx->queue);
    if (ctx->ws)
        (void)hipFree(ctx->ws);
    for (int i = 0; i < 2 * kMaxTimed; ++i)
        if (ctx->tev[i])
            (void)hipEventDestroy(ctx->tev[i]);
    free(ctx);
}

extern "C" const char *bitgnn_last_error(const bitgnn_ctx *ctx) { return ctx ? ctx->err : ""; }

extern "C" int bitgnn_ctx_set_tuning(bitgnn_ctx *ctx, int32_t cb_nodes, int32_t part_len,
                                     int32_t min_avg_degree)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, cb_nodes >= 64 && cb_nodes <= 8192 && part_len >= 4 && part_len <= 1023 &&
                        min_avg_degree >= 0,
               BITGNN_ERR_INVALID_ARG,
               "bitgnn_ctx_set_tuning: cb_nodes=%d (64..8192) part_len=%d (4..1023) "
               "min_avg_degree=%d (>= 0)",
               cb_nodes, part_len, min_avg_degree);
    ctx->cb_nodes = cb_nodes;
    ctx->part_len = part_len;
    ctx->min_avg_degree = min_avg_degree;
    return BITGNN_OK;
}

// Grow-only workspace; not safe to call while the stream is being captured.
int bg_ws_reserve(bitgnn_ctx *ctx, size_t bytes)
{
    if (bytes <= ctx->ws_bytes)
        return BITGNN_OK;
    if (ctx->ws) {
        BG_HIP(ctx, hipDeviceSynchronize());
        BG_HIP(ctx, hipFree(ctx->ws));
        ctx->ws = nullptr;
        ctx->ws_bytes = 0;
    }
    bytes = (bytes + (1u << 20)) & ~(size_t)((1u << 20) - 1);
    BG_HIP(ctx, hipMalloc(&ctx->ws, bytes));
    ctx->ws_bytes = bytes;
    return BITGNN_OK;
}

extern "C" int bitgnn_ctx_kernel_timing(bitgnn_ctx *ctx, int enable)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_NEED_DEVICE(ctx);
    if (enable && !ctx->tev[0])
        for (int i = 0; i < 2 * kMaxTimed; ++i)
            BG_HIP(ctx, hipEventCreate(&ctx->tev[i]));
    ctx->timing = enable ? 1 : 0;
    ctx->n_timed = 0;
    return BITGNN_OK;
}

extern "C" int bitgnn_ctx_kernel_times(bitgnn_ctx *ctx, float *ms, int32_t capacity,
                                       int32_t *count)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, ms && count && capacity >= 0, BITGNN_ERR_INVALID_ARG,
               "bitgnn_ctx_kernel_times: null pointer or negative capacity");
    BG_NEED_DEVICE(ctx);
    int k = 0;
    for (; k < ctx->n_timed && k < capacity; ++k) {
        BG_HIP(ctx, hipEventSynchronize(ctx->tev[2 * k + 1]));
        BG_HIP(ctx, hipEventElapsedTime(&ms[k], ctx->tev[2 * k], ctx->tev[2 * k + 1]));
    }
    *count = k;
    ctx->n_timed = 0;
    return BITGNN_OK;
}
