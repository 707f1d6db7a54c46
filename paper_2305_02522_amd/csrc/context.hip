// Context life cycle and error reporting.
#include "common.h"

#include <stdlib.h>

extern "C" int bitgnn_ctx_create(bitgnn_ctx **out, int device)
{
    if (!out || device < -1)
        return BITGNN_ERR_INVALID_ARG;
    bitgnn_ctx *ctx = (bitgnn_ctx *)calloc(1, sizeof(bitgnn_ctx));
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    ctx->device = device;
    ctx->cb_nodes = kMaxCbNodes;
    ctx->part_len = 255;
    ctx->min_avg_degree = 8;
    ctx->fused_spin_limit = 1u << 22;
    ctx->sc = &ctx->own;
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
            e = hipMalloc((void **)&ctx->own.queue, 256);
        if (e == hipSuccess)
            e = hipMemset(ctx->own.queue, 0, 256);
        if (e == hipSuccess)
            e = hipMalloc((void **)&ctx->own.seed_table, kSeedTableWords * sizeof(uint32_t));
        if (e == hipSuccess)
            e = hipMalloc(&ctx->bgemm_ws, kBgemmScratchBytes);
        if (e != hipSuccess) {
            if (ctx->own.queue)
                (void)hipFree(ctx->own.queue);
            if (ctx->own.seed_table)
                (void)hipFree(ctx->own.seed_table);
            free(ctx);
            return BITGNN_ERR_HIP;
        }
        ctx->own.seed_table_words = kSeedTableWords;
        if (bg_static_scratch_init(ctx) != BITGNN_OK) {
            bitgnn_ctx_destroy(ctx);
            return BITGNN_ERR_HIP;
        }
    }
    *out = ctx;
    return BITGNN_OK;
}

extern "C" void bitgnn_ctx_destroy(bitgnn_ctx *ctx)
{
    if (!ctx)
        return;
    if (ctx->own.seed_table)
        (void)hipFree(ctx->own.seed_table);
    if (ctx->own.queue)
        (void)hipFree(ctx->own.queue);
    if (ctx->bgemm_ws)
        (void)hipFree(ctx->bgemm_ws);
    if (ctx->own.ws)
        (void)hipFree(ctx->own.ws);
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
    BG_REQUIRE(ctx, cb_nodes >= 64 && cb_nodes <= kMaxCbNodes && part_len >= 4 && part_len <= 1023 &&
                        min_avg_degree >= 0,
               BITGNN_ERR_INVALID_ARG,
               "bitgnn_ctx_set_tuning: cb_nodes=%d (64..10208) part_len=%d (4..1023) "
               "min_avg_degree=%d (>= 0)",
               cb_nodes, part_len, min_avg_degree);
    ctx->cb_nodes = cb_nodes;
    ctx->part_len = part_len;
    ctx->min_avg_degree = min_avg_degree;
    return BITGNN_OK;
}

extern "C" int bitgnn_ctx_set_bgemm_path(bitgnn_ctx *ctx, int path)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_REQUIRE(ctx, path >= BITGNN_BGEMM_AUTO && path <= BITGNN_BGEMM_MFMA, BITGNN_ERR_INVALID_ARG,
               "bitgnn_ctx_set_bgemm_path: path=%d (0 auto, 1 VALU, 2 matrix cores)", path);
    ctx->bgemm_path = path;
    return BITGNN_OK;
}

extern "C" int bitgnn_ctx_bgemm_kernel(const bitgnn_ctx *ctx, int64_t n, int32_t kwords, int32_t M,
                                       int *kernel)
{
    if (!ctx || !kernel || n < 0 || kwords < 1 || M < 1)
        return BITGNN_ERR_INVALID_ARG;
    *kernel = bg_bgemm_mfma_applies(ctx, n, kwords, M) ? BITGNN_BGEMM_MFMA : BITGNN_BGEMM_VALU;
    return BITGNN_OK;
}

// The aggregation workspace.  Only this set-up call (and bitgnn_adj_build, through it)
// allocates: it may synchronize the device to replace a smaller workspace.
extern "C" int bitgnn_ctx_reserve(bitgnn_ctx *ctx, size_t bytes)
{
    if (!ctx)
        return BITGNN_ERR_INVALID_ARG;
    BG_NEED_DEVICE(ctx);
    if (bytes <= ctx->own.ws_bytes)
        return BITGNN_OK;
    if (ctx->own.ws) {
        BG_HIP(ctx, hipDeviceSynchronize());
        BG_HIP(ctx, hipFree(ctx->own.ws));
        ctx->own.ws = nullptr;
        ctx->own.ws_bytes = 0;
    }
    bytes = (bytes + (1u << 20)) & ~(size_t)((1u << 20) - 1);
    BG_HIP(ctx, hipMalloc(&ctx->own.ws, bytes));
    ctx->own.ws_bytes = bytes;
    return BITGNN_OK;
}

extern "C" int bitgnn_ctx_workspace(const bitgnn_ctx *ctx, size_t *bytes)
{
    if (!ctx || !bytes)
        return BITGNN_ERR_INVALID_ARG;
    *bytes = ctx->own.ws_bytes;
    return BITGNN_OK;
}

// Compute calls never allocate: a workspace that is too small is an error.
int bg_ws_need(bitgnn_ctx *ctx, size_t bytes, const char *who)
{
    if (bytes <= ctx->sc->ws_bytes)
        return BITGNN_OK;
    return bitgnn_fail(ctx, BITGNN_ERR_WORKSPACE,
                       "%s: needs %zu bytes of workspace, %zu available "
                       "(bitgnn_adj_workspace_bytes + bitgnn_ctx_reserve)",
                       who, bytes, ctx->sc->ws_bytes);
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
