// Measurement support: what this GPU's memory system gives the simplest possible kernels -- a pure
// read, a pure write and a copy with 16-byte accesses -- so that the row solver's kernels, which are
// bound by HBM traffic, can be compared with a ceiling measured on the same box rather than with the
// data-sheet figure alone; and what its matrix cores sustain on a loop of nothing but independent
// MFMA instructions (the ceiling of the Hessian and of the fp64 factorisation kernels).  Not part of
// the method.
#include "common.h"

namespace {

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// Grid-stride over n16 16-byte words, four independent accesses in flight per thread.
//   KIND 0: read src (the words are folded into one value that is stored only if it has a bit
//           pattern it cannot have, which keeps the loads alive without a store stream)
//   KIND 1: write dst      KIND 2: dst = src
//   STREAM: the stores use the streaming (non-temporal) policy, as the flush's stores do
template <int KIND, bool STREAM>
__global__ __launch_bounds__(256) void membench_kernel(const uintx4 *__restrict__ src, uintx4 *__restrict__ dst,
                                                       size_t n16, unsigned *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    uintx4 acc = {0u, 0u, 0u, 0u};
    const uintx4 fill = {1u, 2u, 3u, (unsigned)i};
    auto put = [&](size_t e, uintx4 v) {
        if (STREAM) __builtin_nontemporal_store(v, dst + e);
        else dst[e] = v;
    };
    for (; i + 3 * stride < n16; i += 4 * stride) {
        if (KIND == 1) {
            put(i, fill); put(i + stride, fill); put(i + 2 * stride, fill); put(i + 3 * stride, fill);
        } else {
            const uintx4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], e = src[i + 3 * stride];
            if (KIND == 0) acc |= (a | b) | (c | e);
            else { put(i, a); put(i + stride, b); put(i + 2 * stride, c); put(i + 3 * stride, e); }
        }
    }
    for (; i < n16; i += stride) {
        if (KIND == 1) put(i, fill);
        else {
            const uintx4 a = src[i];
            if (KIND == 0) acc |= a;
            else put(i, a);
        }
    }
    // the benchmark buffers are filled with words whose low bit is clear
    if (KIND == 0 && ((acc.x | acc.y | acc.z | acc.w) & 1u)) sink[0] = acc.x;
}

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef double doublex4 __attribute__((ext_vector_type(4)));

// `iters` rounds of four independent matrix-core instructions per wavefront (v_mfma_f32_32x32x2_f32 or
// v_mfma_f64_16x16x4_f64); the sums are stored only if they take a value they cannot take
template <bool F64>
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, unsigned *sink)
{
    const float a = 1e-3f * (float)(threadIdx.x & 63), b = 1.f + 1e-3f * (float)(threadIdx.x >> 6);
    if (F64) {
        doublex4 acc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = doublex4{0.0, 0.0, 0.0, 0.0};
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a, (double)b, acc[q], 0, 0, 0);
        }
        double t = 0.0;
#pragma unroll
        for (int q = 0; q < 4; ++q) t += acc[q][0] + acc[q][1] + acc[q][2] + acc[q][3];
        if (t == -1.0) sink[0] = 1u;
    } else {
        floatx16 acc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[q], 0, 0, 0);
        }
        float t = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) t += acc[q][v];
        if (t == -1.f) sink[0] = 1u;
    }
}

}  // namespace

extern "C" int obc_membench(obc_ctx *ctx, int kind, int streaming, const void *src, void *dst, size_t bytes,
                            int reps, double *ms_per_pass)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (kind < 0 || kind > 2 || reps < 1 || !ms_per_pass || bytes < 16 || (bytes & 15))
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_membench: bad argument");
    if ((kind != 1 && !src) || (kind != 0 && !dst) || (((uintptr_t)src | (uintptr_t)dst) & 15))
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_membench: buffers must be non-null and 16-byte aligned");
    const size_t n16 = bytes / 16;
    // 8 workgroups of 256 threads per compute unit keep every CU's memory pipeline full
    int cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, ctx->device) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    size_t want = (n16 + 256 * 4 - 1) / (256 * 4);
    const unsigned blocks = (unsigned)(want < (size_t)cus * 8 ? (want ? want : 1) : (size_t)cus * 8);
    hipStream_t st = ctx->stream;
    const uintx4 *s = (const uintx4 *)src;
    uintx4 *d = (uintx4 *)dst;
    unsigned *sink = (unsigned *)ctx->d_status + 32;   // spare words of the context's device block
    hipEvent_t e0, e1;
    OBC_HIP(ctx, hipEventCreate(&e0));
    OBC_HIP(ctx, hipEventCreate(&e1));
    auto launch = [&]() {
        if (kind == 0) membench_kernel<0, false><<<blocks, 256, 0, st>>>(s, d, n16, sink);
        else if (kind == 1 && streaming) membench_kernel<1, true><<<blocks, 256, 0, st>>>(s, d, n16, sink);
        else if (kind == 1) membench_kernel<1, false><<<blocks, 256, 0, st>>>(s, d, n16, sink);
        else if (streaming) membench_kernel<2, true><<<blocks, 256, 0, st>>>(s, d, n16, sink);
        else membench_kernel<2, false><<<blocks, 256, 0, st>>>(s, d, n16, sink);
    };
    launch();                                     // warm-up (page tables, clocks)
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r) launch();
    (void)hipEventRecord(e1, st);
    hipError_t err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess) return obc_fail(ctx, OBC_ERR_HIP, "obc_membench: %s", hipGetErrorString(err));
    OBC_LAUNCH_CHECK(ctx, "membench_kernel");
    *ms_per_pass = (double)ms / reps;
    return OBC_OK;
}

extern "C" int obc_mfmabench(obc_ctx *ctx, int kind, int iters, int reps, double *ms_per_pass, double *flops_per_pass)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (kind < 0 || kind > 1 || iters < 1 || reps < 1 || !ms_per_pass || !flops_per_pass)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_mfmabench: bad argument");
    int cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, ctx->device) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    // four workgroups of four wavefronts per compute unit: four wavefronts on every SIMD
    const unsigned blocks = (unsigned)cus * 4;
    hipStream_t st = ctx->stream;
    unsigned *sink = (unsigned *)ctx->d_status + 32;
    hipEvent_t e0, e1;
    OBC_HIP(ctx, hipEventCreate(&e0));
    OBC_HIP(ctx, hipEventCreate(&e1));
    auto launch = [&]() {
        if (kind == 1) mfma_loop_kernel<true><<<blocks, 256, 0, st>>>(iters, sink);
        else mfma_loop_kernel<false><<<blocks, 256, 0, st>>>(iters, sink);
    };
    launch();                                     // warm-up (clocks)
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r) launch();
    (void)hipEventRecord(e1, st);
    hipError_t err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess) return obc_fail(ctx, OBC_ERR_HIP, "obc_mfmabench: %s", hipGetErrorString(err));
    OBC_LAUNCH_CHECK(ctx, "mfma_loop_kernel");
    *ms_per_pass = (double)ms / reps;
    // 2 * M * N * K flops per instruction: 32 x 32 x 2 (fp32), 16 x 16 x 4 (fp64)
    *flops_per_pass = (double)blocks * 4.0 * (double)iters * 4.0 * (kind == 1 ? 2048.0 : 4096.0);
    return OBC_OK;
}
