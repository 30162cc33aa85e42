// Shared host-side pieces of libobc: the context object, error plumbing, small helpers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/obc.h"

// One timed kernel launch (only while profiling is on): events on the context's stream.  Launches
// that follow each other with nothing in between share an event: the stop of one is the start of
// the next (an event record costs a few microseconds of stream time; own_start says which scope
// created `start`).
struct obc_timed {
    hipEvent_t start, stop;
    bool own_start;
    int kind;           // OBC_KERNEL_*
    double bytes, flops;   // algorithmic work of the launch
};

struct obc_ctx {
    hipStream_t stream;
    int device;
    int *d_status;      // device error latch: 0, or the first OBC_ERR_* a kernel saw
    void *select_scratch;   // this device's copy of the built-in scratch of obc_global_select_static
    char err[512];
    bool profiling;
    std::vector<obc_timed> timed;
    std::vector<hipEvent_t> event_pool;
    hipEvent_t chain_event;   // stop event of the last timed launch ...
    bool chain_fresh;         // ... valid as the next one's start: nothing was enqueued after it
};

// Bracket a launch with events when profiling is on.
struct obc_scope {
    obc_ctx *ctx;
    obc_timed t;
    bool on;
    obc_scope(obc_ctx *c, int kind, double bytes, double flops) : ctx(c), on(c->profiling)
    {
        if (!on) return;
        t.kind = kind; t.bytes = bytes; t.flops = flops;
        auto get = [&]() {
            hipEvent_t e;
            if (!ctx->event_pool.empty()) { e = ctx->event_pool.back(); ctx->event_pool.pop_back(); return e; }
            if (hipEventCreate(&e) != hipSuccess) e = nullptr;
            return e;
        };
        t.own_start = !ctx->chain_fresh;
        t.start = t.own_start ? get() : ctx->chain_event;
        t.stop = get();
        if (!t.start || !t.stop) { on = false; ctx->chain_fresh = false; return; }
        if (t.own_start) (void)hipEventRecord(t.start, ctx->stream);
    }
    ~obc_scope()
    {
        if (!on) return;
        (void)hipEventRecord(t.stop, ctx->stream);
        ctx->chain_event = t.stop;
        ctx->chain_fresh = true;
        ctx->timed.push_back(t);
    }
};

// global_select.hip: device address of the built-in scratch array on `device` (the current device)
int obc_select_scratch_address(int device, void **ptr);

static inline int obc_fail(obc_ctx *ctx, int code, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

#define OBC_HIP(ctx, call)                                                              \
    do {                                                                                \
        hipError_t e__ = (call);                                                        \
        if (e__ != hipSuccess)                                                          \
            return obc_fail((ctx), OBC_ERR_HIP, "%s failed: %s (%s:%d)", #call,        \
                            hipGetErrorString(e__), __FILE__, __LINE__);                \
    } while (0)

#define OBC_LAUNCH_CHECK(ctx, name)                                                     \
    do {                                                                                \
        hipError_t e__ = hipGetLastError();                                             \
        if (e__ != hipSuccess)                                                          \
            return obc_fail((ctx), OBC_ERR_HIP, "launch of %s failed: %s", (name),      \
                            hipGetErrorString(e__));                                    \
    } while (0)

__host__ __device__ static inline size_t obc_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Latch the first error seen by any kernel (device side).
__device__ static inline void obc_latch(int *status, int code)
{
    atomicCAS(status, 0, code);
}
