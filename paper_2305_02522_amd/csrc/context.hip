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
    if (device >= 0) {
        int count = 0;
        hipError_t e = hipGetDeviceCount(&count);
        if (e != hipSuccess || device >= count) {
            free(ctx);
            return BITGNN_ERR_HIP;
        }
        e = hipSetDevice(device);
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
    free(ctx);
}

extern "C" const char *bitgnn_last_error(const bitgnn_ctx *ctx) { return ctx ? ctx->err : ""; }
