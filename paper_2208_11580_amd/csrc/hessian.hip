// obc_hessian: H = 2 X X^T (+ dampening), Sec. 4 of arxiv 2208.11580, and obc_cross: 2 Y X^T, the
// second moment that the sequential variant (appendix "Sequential Quantization with OBQ")
// accumulates beside it.
//
// A dense symmetric rank-N contraction, so it runs on the fp32 matrix cores:
// v_mfma_f32_32x32x2_f32, 128x128 output tiles per 256-thread workgroup (four waves, each
// 64x64 = 2x2 MFMA tiles), X staged through LDS k-major so that the MFMA operand reads are
// bank-conflict free.  Only tiles on or above the block diagonal are computed; the
// contraction length N is cut into S slices so that small d still fills 256 CUs.  Slices go
// to a workspace and are summed in a fixed order by a second kernel, which also mirrors the
// upper tiles into the lower triangle (H comes out exactly symmetric) -- no float atomics,
// results are deterministic.
#include "common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;       // tile edge
constexpr int BK = 16;        // k-slab per LDS stage
constexpr int LDT = BM + 4;   // padded LDS row

__host__ __device__ inline int tiles_of(int d) { return (d + BM - 1) / BM; }

// How many slices of the sample axis, and how long each is (multiple of BK), for a launch of
// `ntri` output tiles of `tile_elems` results each.  Workgroups are dealt evenly to the 256 CUs,
// which work on several at a time, so the launch lasts as long as the CU with the most
// workgroups: ceil(ntri S / 256) of them, each 1 / S of a tile's contraction.  More slices even
// that out but cost S partial results written and read back; the plan minimises the sum of both
// (matrix-core time at ~120 TFLOP/s, partial traffic at ~4 TB/s).
inline void split_plan_tiles(int64_t ntri, int64_t N, int *S, int64_t *kchunk, double tile_elems = (double)BM * BM)
{
    const int64_t smax = (N + 2047) / 2048 > 0 ? (N + 2047) / 2048 : 1;
    const double flops_tile = 2.0 * tile_elems * (double)N;
    const double cu_rate = 120e12 / 256.0;
    double best = 0.0;
    int64_t s = 1;
    for (int64_t c = 1; c <= smax && c <= 64; ++c) {
        double per_cu = (double)((ntri * c + 255) / 256);   // workgroups on the busiest CU
        if (per_cu < 4.0) per_cu = 4.0;                     // fewer than ~4 resident do not go faster
        const double cost = per_cu * (flops_tile / (double)c) / cu_rate
                            + (double)c * (double)ntri * tile_elems * 8.0 / 4e12;
        if (c == 1 || cost < best) { best = cost; s = c; }
    }
    int64_t kc = (N + s - 1) / s;
    kc = (kc + BK - 1) / BK * BK;
    if (kc < BK) kc = BK;
    s = (N + kc - 1) / kc;
    if (s < 1) s = 1;
    *S = (int)s;
    *kchunk = kc;
}

inline void split_plan(int d, int64_t N, int *S, int64_t *kchunk)
{
    int nt = tiles_of(d);
    split_plan_tiles((int64_t)nt * (nt + 1) / 2, N, S, kchunk);
}

// One slice of P = Ya Xb^T over the samples [kbeg, kend): Ya is da x N (leading dimension lda),
// Xb is db x N (ldb).  SYM: Ya and Xb are the same matrix and only the tiles on or above the block
// diagonal are formed.
template <bool SYM>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void nt_partial_kernel(const float *__restrict__ Ya, int da,
                                                         int64_t lda, const float *__restrict__ Xb,
                                                         int db, int64_t ldb, int64_t N,
                                                         int64_t kchunk, float *__restrict__ partial,
                                                         int vec_ok)
{
    __shared__ float As[BK][LDT];
    __shared__ float Bs[BK][LDT];

    const int tile_id = blockIdx.x, slice = blockIdx.y;
    int ti, tj;
    if (SYM) {
        // upper-triangular tile enumeration: tile_id -> (ti <= tj)
        const int nt = tiles_of(da);
        int t = tile_id, rowlen = nt;
        ti = 0;
        while (t >= rowlen) { t -= rowlen; ++ti; --rowlen; }
        tj = ti + t;
    } else {
        const int ntb = tiles_of(db);
        ti = tile_id / ntb;
        tj = tile_id % ntb;
    }
    const bool on_diag = SYM && (ti == tj);

    const int64_t kbeg = (int64_t)slice * kchunk;
    const int64_t kend = (kbeg + kchunk < N) ? kbeg + kchunk : N;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // loader: a 128 x 16 slab is 512 float4; thread takes quads tid and tid + 256
    float4 ra[2], rb[2];
    auto fetch = [&](const float *M, int rows, int64_t ld, int tile, int64_t k0, float4(&r)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int f = tid + h * 256;
            int row = tile * BM + (f >> 2);
            int64_t k = k0 + (f & 3) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < rows) {
                const float *src = M + (int64_t)row * ld + k;
                if (vec_ok && k + 3 < kend) {
                    v = *reinterpret_cast<const float4 *>(src);
                } else {
                    if (k + 0 < kend) v.x = src[0];
                    if (k + 1 < kend) v.y = src[1];
                    if (k + 2 < kend) v.z = src[2];
                    if (k + 3 < kend) v.w = src[3];
                }
            }
            r[h] = v;
        }
    };
    auto stash = [&](float(&T)[BK][LDT], const float4(&r)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int f = tid + h * 256;
            int row = f >> 2, kq = (f & 3) * 4;
            T[kq + 0][row] = r[h].x;
            T[kq + 1][row] = r[h].y;
            T[kq + 2][row] = r[h].z;
            T[kq + 3][row] = r[h].w;
        }
    };

    // A slab that lies wholly inside the slice is fetched without a per-lane condition (rows beyond
    // the matrix re-read its last row: their products only reach outputs that are never stored), so
    // that the loop body is straight-line code and the loads overlap with the MFMAs; the slab at the
    // end of the slice and unaligned inputs take the general loader.
    auto fetch_full = [&](const float *M, int rows, int64_t ld, int tile, int64_t k0, float4(&r)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int f = tid + h * 256;
            int row = tile * BM + (f >> 2);
            row = row < rows ? row : rows - 1;
            r[h] = *reinterpret_cast<const float4 *>(M + (int64_t)row * ld + k0 + (f & 3) * 4);
        }
    };
    const float(*Bt)[LDT] = on_diag ? As : Bs;
    const int kl = lane >> 5, il = lane & 31;
    auto mma_slab = [&]() {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a0 = As[kk + kl][wm * 64 + il];
            float a1 = As[kk + kl][wm * 64 + 32 + il];
            float b0 = Bt[kk + kl][wn * 64 + il];
            float b1 = Bt[kk + kl][wn * 64 + 32 + il];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    };

    if (kbeg < kend) {
        fetch(Ya, da, lda, ti, kbeg, ra);
        if (!on_diag) fetch(Xb, db, ldb, tj, kbeg, rb);
    }
    int64_t k0 = kbeg;
    if (vec_ok) {
        // slabs whose successor is a full slab
        for (; k0 + 2 * BK <= kend; k0 += BK) {
            stash(As, ra);
            if (!on_diag) stash(Bs, rb);
            __syncthreads();
            fetch_full(Ya, da, lda, ti, k0 + BK, ra);
            if (!on_diag) fetch_full(Xb, db, ldb, tj, k0 + BK, rb);
            mma_slab();
            __syncthreads();
        }
    }
    for (; k0 < kend; k0 += BK) {
        stash(As, ra);
        if (!on_diag) stash(Bs, rb);
        __syncthreads();
        if (k0 + BK < kend) {
            fetch(Ya, da, lda, ti, k0 + BK, ra);
            if (!on_diag) fetch(Xb, db, ldb, tj, k0 + BK, rb);
        }
        mma_slab();
        __syncthreads();
    }

    // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32) and, for register v,
    // row 8 * (v / 4) + 4 * (lane / 32) + v % 4
    float *out = partial + (int64_t)slice * da * db;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int i = ti * BM + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                int j = tj * BM + wn * 64 + b * 32 + (lane & 31);
                if (i < da && j < db) out[(int64_t)i * db + j] = acc[a][b][v];
            }
}

// H (+)= 2 * sum_s partial[s] on the tiles on or above the block diagonal, slices added in index
// order, and the mirror image below it.  One workgroup per 32 x 32 piece of such a tile: the sums
// are read and written along rows, the mirrored piece goes through LDS so that it is written
// along rows too.
__global__ __launch_bounds__(256) void syrk_reduce_kernel(const float *__restrict__ partial, int S,
                                                          int d, int accumulate,
                                                          float *__restrict__ H)
{
    __shared__ float Tt[32][33];
    const int pi = blockIdx.y, pj = blockIdx.x;           // 32 x 32 piece (pi, pj)
    if (pi / (BM / 32) > pj / (BM / 32)) return;          // its 128-tile lies below the block diagonal
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const bool mirror = (pi / (BM / 32) != pj / (BM / 32));
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = pi * 32 + ty + 8 * r, j = pj * 32 + tx;
        float s = 0.f;
        if (i < d && j < d) {
            const int64_t e = (int64_t)i * d + j;
            for (int k = 0; k < S; ++k) s += partial[(int64_t)k * d * d + e];
            s *= 2.f;
            H[e] = accumulate ? H[e] + s : s;
        }
        Tt[ty + 8 * r][tx] = s;
    }
    if (!mirror) return;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = pj * 32 + ty + 8 * r, j = pi * 32 + tx;   // (i, j) of the mirrored piece
        if (i < d && j < d) {
            const int64_t e = (int64_t)i * d + j;
            const float s = Tt[tx][ty + 8 * r];
            H[e] = accumulate ? H[e] + s : s;
        }
    }
}

// C[e] (+)= 2 * sum_s partial[s][e] over a dense da x db result, slices added in index order.
__global__ __launch_bounds__(256) void nt_reduce_kernel(const float *__restrict__ partial, int S,
                                                        int64_t n, int accumulate, float *__restrict__ C)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    float s = 0.f;
    for (int k = 0; k < S; ++k) s += partial[(int64_t)k * n + e];
    s *= 2.f;
    C[e] = accumulate ? C[e] + s : s;
}

// diag(H) += damp_rel * mean(diag(H)); one workgroup, fixed-order tree sum in fp64.
__global__ __launch_bounds__(1024) void dampen_kernel(float *__restrict__ H, int d, float damp_rel)
{
    __shared__ double red[1024];
    double s = 0.0;
    for (int j = threadIdx.x; j < d; j += blockDim.x) s += (double)H[(int64_t)j * d + j];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = blockDim.x / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    float lam = (float)((double)damp_rel * red[0] / (double)d);
    for (int j = threadIdx.x; j < d; j += blockDim.x) H[(int64_t)j * d + j] += lam;
}

}  // namespace

extern "C" {

int obc_hessian_workspace_bytes(int d, int64_t N, size_t *bytes)
{
    if (!bytes || d <= 0 || N < 0) return OBC_ERR_BAD_ARG;
    int S;
    int64_t kc;
    split_plan(d, N > 0 ? N : 1, &S, &kc);
    *bytes = obc_align_up((size_t)S * d * d * sizeof(float), 256);
    return OBC_OK;
}

int obc_hessian(obc_ctx *ctx, const float *X, int d, int64_t N, int64_t ldx, float damp_rel,
                int accumulate, float *H, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!X || !H) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_hessian: null X or H");
    if (d <= 0 || N <= 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_hessian: d and N must be positive");
    if (ldx < N) return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "obc_hessian: ldx (%lld) < N (%lld)", (long long)ldx, (long long)N);
    size_t need;
    obc_hessian_workspace_bytes(d, N, &need);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "obc_hessian: workspace of %zu bytes needed, %zu given", need, ws_bytes);

    int S;
    int64_t kchunk;
    split_plan(d, N, &S, &kchunk);
    const int nt = tiles_of(d);
    const int ntri = nt * (nt + 1) / 2;
    const int vec_ok = (ldx % 4 == 0) && (((uintptr_t)X & 15) == 0);
    float *partial = (float *)ws;

    nt_partial_kernel<true><<<dim3(ntri, S), 256, 0, ctx->stream>>>(X, d, ldx, X, d, ldx, N, kchunk, partial, vec_ok);
    OBC_LAUNCH_CHECK(ctx, "nt_partial_kernel");
    const unsigned np32 = (unsigned)((d + 31) / 32);
    syrk_reduce_kernel<<<dim3(np32, np32), 256, 0, ctx->stream>>>(partial, S, d, accumulate, H);
    OBC_LAUNCH_CHECK(ctx, "syrk_reduce_kernel");
    if (damp_rel >= 0.f) {
        dampen_kernel<<<1, 1024, 0, ctx->stream>>>(H, d, damp_rel);
        OBC_LAUNCH_CHECK(ctx, "dampen_kernel");
    }
    return OBC_OK;
}

static void cross_plan(int d_row, int d_col, int64_t N, int *S, int64_t *kchunk)
{
    split_plan_tiles((int64_t)tiles_of(d_row) * tiles_of(d_col), N, S, kchunk);
}

int obc_cross_workspace_bytes(int d_row, int d_col, int64_t N, size_t *bytes)
{
    if (!bytes || d_row <= 0 || d_col <= 0 || N < 0) return OBC_ERR_BAD_ARG;
    int S;
    int64_t kc;
    cross_plan(d_row, d_col, N > 0 ? N : 1, &S, &kc);
    *bytes = obc_align_up((size_t)S * d_row * d_col * sizeof(float), 256);
    return OBC_OK;
}

int obc_cross(obc_ctx *ctx, const float *X, const float *Y, int d_col, int d_row, int64_t N, int64_t ldx,
              int64_t ldy, int accumulate, float *C, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!X || !Y || !C) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_cross: null X, Y or C");
    if (d_col <= 0 || d_row <= 0 || N <= 0)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_cross: d_col, d_row and N must be positive");
    if (ldx < N || ldy < N)
        return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "obc_cross: ldx (%lld) or ldy (%lld) < N (%lld)", (long long)ldx,
                        (long long)ldy, (long long)N);
    size_t need;
    obc_cross_workspace_bytes(d_row, d_col, N, &need);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "obc_cross: workspace of %zu bytes needed, %zu given", need, ws_bytes);

    int S;
    int64_t kchunk;
    cross_plan(d_row, d_col, N, &S, &kchunk);
    const int ntiles = tiles_of(d_row) * tiles_of(d_col);
    const int vec_ok = (ldx % 4 == 0) && (ldy % 4 == 0) && (((uintptr_t)X & 15) == 0) && (((uintptr_t)Y & 15) == 0);
    float *partial = (float *)ws;
    nt_partial_kernel<false><<<dim3(ntiles, S), 256, 0, ctx->stream>>>(Y, d_row, ldy, X, d_col, ldx, N, kchunk, partial, vec_ok);
    OBC_LAUNCH_CHECK(ctx, "nt_partial_kernel");
    const int64_t n = (int64_t)d_row * d_col;
    nt_reduce_kernel<<<(unsigned)((n + 255) / 256), 256, 0, ctx->stream>>>(partial, S, n, accumulate, C);
    OBC_LAUNCH_CHECK(ctx, "nt_reduce_kernel");
    return OBC_OK;
}

}  // extern "C"
