// Context life cycle and the device error latch.
#include "common.h"

extern "C" {

const char *obc_version(void) { return "libobc 0.1 (gfx950)"; }

int obc_create(obc_ctx **out, void *hip_stream)
{
    if (!out) return OBC_ERR_BAD_ARG;
    *out = nullptr;
    obc_ctx *ctx = new (std::nothrow) obc_ctx;
    if (!ctx) return OBC_ERR_BAD_ARG;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->d_status = nullptr;
    ctx->select_scratch = nullptr;
    ctx->err[0] = 0;
    ctx->device = 0;
    ctx->profiling = false;
    ctx->chain_event = nullptr;
    ctx->chain_fresh = false;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->d_status, 256);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->d_status, 0, 256, ctx->stream);
    if (e == hipSuccess && obc_select_scratch_address(ctx->device, &ctx->select_scratch) != OBC_OK) e = hipErrorUnknown;
    if (e != hipSuccess) {
        if (ctx->d_status) (void)hipFree(ctx->d_status);
        delete ctx;
        return OBC_ERR_HIP;
    }
    *out = ctx;
    return OBC_OK;
}

int obc_destroy(obc_ctx *ctx)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->d_status) (void)hipFree(ctx->d_status);
    for (auto &t : ctx->timed) {
        if (t.own_start) (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    for (auto e : ctx->event_pool) (void)hipEventDestroy(e);
    delete ctx;
    return OBC_OK;
}

int obc_profile_begin(obc_ctx *ctx)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    for (auto &t : ctx->timed) {
        if (t.own_start) ctx->event_pool.push_back(t.start);
        ctx->event_pool.push_back(t.stop);
    }
    ctx->timed.clear();
    ctx->chain_fresh = false;
    ctx->profiling = true;
    return OBC_OK;
}

int obc_profile_end(obc_ctx *ctx, obc_kernel_stat stats[OBC_KERNEL_CLASSES])
{
    if (!ctx || !stats) return OBC_ERR_BAD_ARG;
    ctx->profiling = false;
    ctx->chain_fresh = false;
    OBC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (int k = 0; k < OBC_KERNEL_CLASSES; ++k) { stats[k].launches = 0; stats[k].ms = stats[k].bytes = stats[k].flops = 0.0; }
    for (auto &t : ctx->timed) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess && t.kind >= 0 && t.kind < OBC_KERNEL_CLASSES) {
            stats[t.kind].launches += 1;
            stats[t.kind].ms += ms;
            stats[t.kind].bytes += t.bytes;
            stats[t.kind].flops += t.flops;
        }
        if (t.own_start) ctx->event_pool.push_back(t.start);
        ctx->event_pool.push_back(t.stop);
    }
    ctx->timed.clear();
    return OBC_OK;
}

const char *obc_last_error(const obc_ctx *ctx) { return ctx ? ctx->err : "null context"; }

int obc_check(obc_ctx *ctx)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    int h = 0;
    OBC_HIP(ctx, hipMemcpyAsync(&h, ctx->d_status, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    OBC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (h != 0) {
        OBC_HIP(ctx, hipMemsetAsync(ctx->d_status, 0, sizeof(int), ctx->stream));
        OBC_HIP(ctx, hipStreamSynchronize(ctx->stream));
        return obc_fail(ctx, h, "a kernel reported error %d (%s)", h,
                        h == OBC_ERR_NUMERIC   ? "non-positive or non-finite pivot in a row solver"
                        : h == OBC_ERR_NOT_SPD ? "matrix is not positive definite"
                                               : "unknown");
    }
    return OBC_OK;
}

}  // extern "C"
