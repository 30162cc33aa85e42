// obc_global_select: the global step of ExactOBS (Appendix Algorithm 2 of arxiv 2208.11580).
//
// Algorithm 2 pops, k times, the row whose *next* loss change is smallest.  A heap would make
// that k log(d_row) sequential steps; on the GPU the same result is reached in parallel:
//
//   An element (i, j) is popped as soon as every earlier element of its row is out and its own
//   value is the frontier minimum.  Once the largest value seen so far in row i (its prefix
//   maximum m_ij = max_{j' <= j} L[i][j']) has been popped, every following element of row i that
//   is not larger is popped right away, before any other row moves.  So Algorithm 2 pops the
//   elements in ascending order of the key (m_ij, i, j), and after k pops row i has lost
//   exactly the elements whose key is among the k smallest.
//
// Steps: per-row prefix maximum -> order-preserving uint32 keys; radix select (four 8-bit
// passes, integer histograms) of the k-th smallest key value v; per row the counts of keys
// < v and == v (keys are non-decreasing along a row, so those are prefixes); ties at v are
// handed out in row order; finally the mask is scattered from the per-row pruning order.
#include <mutex>

#include "common.h"

namespace {

struct SelState {
    unsigned long long remaining;   // rank still to find inside the current prefix bucket
    unsigned int prefix;            // key bits fixed so far
    unsigned int pad;
    unsigned int hist[256];
};

__device__ inline unsigned int float_key(float f)
{
    unsigned int u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// keys[i][j] = key(max(L[i][0..j])); one workgroup per row, chunked inclusive max-scan
__global__ __launch_bounds__(256) void prefix_max_kernel(const float *__restrict__ loss, int d,
                                                         unsigned int *__restrict__ keys)
{
    __shared__ float wave_max[4];
    __shared__ float carry_s;
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = -__builtin_inff();
    __syncthreads();
    for (int base = 0; base < d; base += 256) {
        int j = base + tid;
        float v = (j < d) ? loss[(size_t)row * d + j] : -__builtin_inff();
        if (v != v) v = __builtin_inff();   // a NaN loss sorts last
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            float o = __shfl_up(v, off, 64);
            if (lane >= off) v = fmaxf(v, o);
        }
        if (lane == 63) wave_max[wave] = v;
        __syncthreads();
        float carry = carry_s;
        for (int wv = 0; wv < wave; ++wv) carry = fmaxf(carry, wave_max[wv]);
        v = fmaxf(v, carry);
        if (j < d) keys[(size_t)row * d + j] = float_key(v);
        __syncthreads();
        if (tid == 255) carry_s = v;
        __syncthreads();
    }
}

__global__ void sel_init_kernel(SelState *st, unsigned long long k)
{
    if (threadIdx.x == 0) { st->remaining = k; st->prefix = 0; st->pad = 0; }
    st->hist[threadIdx.x] = 0;
}

// histogram of byte `pass` (3 = most significant) over the keys that match the fixed prefix
__global__ __launch_bounds__(256) void sel_hist_kernel(const unsigned int *__restrict__ keys,
                                                       int64_t n, int pass, SelState *st)
{
    __shared__ unsigned int h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int shift = pass * 8;
    const unsigned int prefix = st->prefix;
    const unsigned int himask = (pass == 3) ? 0u : (0xffffffffu << (shift + 8));
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (int64_t)gridDim.x * blockDim.x) {
        unsigned int u = keys[e];
        if ((u & himask) == (prefix & himask)) atomicAdd(&h[(u >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&st->hist[threadIdx.x], h[threadIdx.x]);
}

// choose the byte bucket that holds the wanted rank; clear the histogram for the next pass
__global__ void sel_pick_kernel(SelState *st, int pass)
{
    __shared__ unsigned int h[256];
    h[threadIdx.x] = st->hist[threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long rem = st->remaining;   // 1-based rank inside the current bucket
        unsigned int b = 0;
        for (; b < 255; ++b) {
            if (rem <= h[b]) break;
            rem -= h[b];
        }
        st->remaining = rem;
        st->prefix |= b << (pass * 8);
    }
    __syncthreads();
    st->hist[threadIdx.x] = 0;
}

// per row: number of keys below / equal to the selected key value (prefixes of the row)
__global__ __launch_bounds__(256) void row_counts_kernel(const unsigned int *__restrict__ keys, int d,
                                                         const SelState *st, int *__restrict__ c_lt,
                                                         int *__restrict__ c_eq)
{
    __shared__ int s_lt, s_eq;
    const int row = blockIdx.x;
    if (threadIdx.x == 0) { s_lt = 0; s_eq = 0; }
    __syncthreads();
    const unsigned int v = st->prefix;
    int lt = 0, eq = 0;
    for (int j = threadIdx.x; j < d; j += blockDim.x) {
        unsigned int u = keys[(size_t)row * d + j];
        lt += (u < v);
        eq += (u == v);
    }
    atomicAdd(&s_lt, lt);
    atomicAdd(&s_eq, eq);
    __syncthreads();
    if (threadIdx.x == 0) { c_lt[row] = s_lt; c_eq[row] = s_eq; }
}

// one workgroup: ties at the selected value go to the rows in index order
__global__ __launch_bounds__(1024) void assign_counts_kernel(const int *__restrict__ c_lt,
                                                             const int *__restrict__ c_eq, int R,
                                                             long long k, int *__restrict__ counts)
{
    __shared__ long long scan[1024];
    __shared__ long long base_s;
    const int tid = threadIdx.x;
    // total of strictly-smaller keys
    long long s = 0;
    for (int i = tid; i < R; i += 1024) s += c_lt[i];
    scan[tid] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (tid < w) scan[tid] += scan[tid + w];
        __syncthreads();
    }
    long long need = k - scan[0];   // ties still to hand out (>= 0 by construction of the select)
    __syncthreads();
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int b0 = 0; b0 < R; b0 += 1024) {
        int i = b0 + tid;
        long long e = (i < R) ? c_eq[i] : 0;
        scan[tid] = e;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {   // inclusive Hillis-Steele scan
            long long o = (tid >= off) ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += o;
            __syncthreads();
        }
        long long excl = base_s + scan[tid] - e;
        if (i < R) {
            long long take = need - excl;
            take = take < 0 ? 0 : (take > e ? e : take);
            counts[i] = c_lt[i] + (int)take;
        }
        __syncthreads();
        if (tid == 1023) base_s += scan[1023];
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void zero_u8_kernel(uint8_t *p, int64_t n)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) p[e] = 0;
}

__global__ __launch_bounds__(256) void scatter_mask_kernel(const int32_t *__restrict__ order,
                                                           const int *__restrict__ counts, int d,
                                                           uint8_t *__restrict__ mask)
{
    const int row = blockIdx.x;
    const int c = counts[row];
    for (int t = threadIdx.x; t < c; t += blockDim.x) {
        int p = order[(size_t)row * d + t];
        if (p >= 0 && p < d) mask[(size_t)row * d + p] = 1;
    }
}

__global__ void fill_i32_kernel(int *p, int n, int v)
{
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) p[e] = v;
}

}  // namespace

// ---- the variant that allocates nothing: its scratch region is a device array of this library.
// Every GPU holds its own copy of the array at its own address; in host code the array's name is
// only a handle for hipGetSymbolAddress, never a pointer to pass on.
static __device__ __align__(256) unsigned char select_scratch[OBC_SELECT_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex select_scratch_mutex;
static void *select_scratch_ptr[kMaxDevices];   // device address of select_scratch on each device, once known

// Device address of select_scratch on `device`, which must be the current device (obc_create
// calls this, so a context always finds its device's entry filled).
int obc_select_scratch_address(int device, void **ptr)
{
    if (device < 0 || device >= kMaxDevices || !ptr) return OBC_ERR_BAD_ARG;
    std::lock_guard<std::mutex> lock(select_scratch_mutex);
    if (!select_scratch_ptr[device]) {
        int cur = -1;
        if (hipGetDevice(&cur) != hipSuccess || cur != device) return OBC_ERR_HIP;
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(select_scratch)) != hipSuccess || !p) return OBC_ERR_HIP;
        select_scratch_ptr[device] = p;
    }
    *ptr = select_scratch_ptr[device];
    return OBC_OK;
}

extern "C" {

int obc_global_select_workspace_bytes(int R, int d, size_t *bytes)
{
    if (!bytes || R < 0 || d <= 0) return OBC_ERR_BAD_ARG;
    size_t keys = obc_align_up((size_t)R * d * sizeof(unsigned int), 256);
    size_t cnt = obc_align_up((size_t)R * sizeof(int), 256);
    *bytes = keys + 2 * cnt + obc_align_up(sizeof(SelState), 256);
    return OBC_OK;
}

// The kernels of the global step on a scratch region laid out as obc_global_select_workspace_bytes
// describes (the caller has checked the arguments and the region's size).
static int global_select_enqueue(obc_ctx *ctx, const float *loss, const int32_t *order, int R, int d, int64_t k,
                                 int32_t *counts, uint8_t *mask, void *ws)
{
    hipStream_t st = ctx->stream;
    const int64_t n = (int64_t)R * d;
    char *base = (char *)ws;
    unsigned int *keys = (unsigned int *)base;
    size_t off = obc_align_up((size_t)n * sizeof(unsigned int), 256);
    int *c_lt = (int *)(base + off);
    off += obc_align_up((size_t)R * sizeof(int), 256);
    int *c_eq = (int *)(base + off);
    off += obc_align_up((size_t)R * sizeof(int), 256);
    SelState *sel = (SelState *)(base + off);

    zero_u8_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(mask, n);
    if (k == 0) {
        fill_i32_kernel<<<(R + 255) / 256, 256, 0, st>>>(counts, R, 0);
        OBC_LAUNCH_CHECK(ctx, "fill_i32_kernel");
        return OBC_OK;
    }
    prefix_max_kernel<<<R, 256, 0, st>>>(loss, d, keys);
    sel_init_kernel<<<1, 256, 0, st>>>(sel, (unsigned long long)k);
    int blocks = (int)((n + 256 * 8 - 1) / (256 * 8));
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    for (int pass = 3; pass >= 0; --pass) {
        sel_hist_kernel<<<blocks, 256, 0, st>>>(keys, n, pass, sel);
        sel_pick_kernel<<<1, 256, 0, st>>>(sel, pass);
    }
    row_counts_kernel<<<R, 256, 0, st>>>(keys, d, sel, c_lt, c_eq);
    assign_counts_kernel<<<1, 1024, 0, st>>>(c_lt, c_eq, R, (long long)k, counts);
    scatter_mask_kernel<<<R, 256, 0, st>>>(order, counts, d, mask);
    OBC_LAUNCH_CHECK(ctx, "global select kernels");
    return OBC_OK;
}

static int global_select_check_args(obc_ctx *ctx, const char *who, const float *loss, const int32_t *order, int R,
                                    int d, int64_t k, const int32_t *counts, const uint8_t *mask)
{
    if (!loss || !order || !counts || !mask) return obc_fail(ctx, OBC_ERR_BAD_ARG, "%s: null argument", who);
    if (R < 0 || d <= 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "%s: bad size", who);
    if (k < 0 || k > (int64_t)R * d)
        return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "%s: k (%lld) outside [0, R*d]", who, (long long)k);
    return OBC_OK;
}

int obc_global_select(obc_ctx *ctx, const float *loss, const int32_t *order, int R, int d, int64_t k,
                      int32_t *counts, uint8_t *mask, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    int rc = global_select_check_args(ctx, "obc_global_select", loss, order, R, d, k, counts, mask);
    if (rc != OBC_OK) return rc;
    size_t need;
    obc_global_select_workspace_bytes(R, d, &need);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "obc_global_select: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    if (R == 0) return OBC_OK;
    return global_select_enqueue(ctx, loss, order, R, d, k, counts, mask, ws);
}

int obc_global_select_static(obc_ctx *ctx, const float *loss, const int32_t *order, int R, int d, int64_t k,
                             int32_t *counts, uint8_t *mask)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    int rc = global_select_check_args(ctx, "obc_global_select_static", loss, order, R, d, k, counts, mask);
    if (rc != OBC_OK) return rc;
    size_t need;
    obc_global_select_workspace_bytes(R, d, &need);
    if ((int64_t)R * d > (int64_t)OBC_SELECT_STATIC_MAX_WEIGHTS || R > OBC_SELECT_STATIC_MAX_ROWS ||
        need > (size_t)OBC_SELECT_STATIC_SCRATCH_BYTES)
        return obc_fail(ctx, OBC_ERR_WORKSPACE,
                        "obc_global_select_static: %d x %d exceeds the built-in scratch (at most %d weights in at "
                        "most %d rows); use obc_global_select with a workspace", R, d,
                        OBC_SELECT_STATIC_MAX_WEIGHTS, OBC_SELECT_STATIC_MAX_ROWS);
    if (!ctx->select_scratch)
        return obc_fail(ctx, OBC_ERR_HIP, "obc_global_select_static: the scratch address is unknown on device %d", ctx->device);
    if (R == 0) return OBC_OK;
    return global_select_enqueue(ctx, loss, order, R, d, k, counts, mask, ctx->select_scratch);
}

}  // extern "C"
