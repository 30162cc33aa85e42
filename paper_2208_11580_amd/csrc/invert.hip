// obc_invert: H^-1 of the dampened Hessian through its Cholesky factor (Sec. 4 Step 1 of
// arxiv 2208.11580 needs the full inverse once per layer).
//
// This step is Theta(d^3) once per layer, next to Theta(d_row d^3) for the row solver, so it is
// written for accuracy first: everything is done in fp64 and only the final result is rounded
// to fp32 (the fp32 Hessians of correlated post-ReLU activations have condition numbers of
// 1e4..1e5; an fp32 factorisation would already cost three to four digits of H^-1).
//
//   1. A = double(H);  blocked right-looking Cholesky A = L L^T with 64-wide block columns:
//      the diagonal block is factored and inverted by a single wavefront (16 x 16 sub-blocks in
//      registers, the rest of the block on the fp64 matrix core out of LDS), the panel below
//      is a product with the inverted diagonal block, the trailing update is a tiled GEMM.
//   2. Y = L^-1 by right-looking blocked forward substitution on the identity (two GEMMs per
//      block row, each over the whole remaining matrix, so all CUs are busy).
//   3. H^-1 = Y^T Y, lower tiles only, mirrored on store so the result is exactly symmetric.
// All GEMMs run on the fp64 matrix cores (v_mfma_f64_16x16x4_f64), 64x64 tiles staged through LDS.
#include "dense64.h"

namespace {

using namespace obc_dense64;

__global__ void f32_to_f64_kernel(const float *__restrict__ src, double *__restrict__ dst, int64_t n)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) dst[e] = (double)src[e];
}

__global__ void f64_to_f32_kernel(const double *__restrict__ src, float *__restrict__ dst, int64_t n)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) dst[e] = (float)src[e];
}

// Batched use (one block per matrix): block b works on A + b strideA and Linv + b strideL; err is
// the code latched on a bad pivot.
__global__ __launch_bounds__(64) void potrf_wave_kernel(double *__restrict__ A, int lda, int bs,
                                                        double *__restrict__ Linv, int *status,
                                                        int64_t strideA, int64_t strideL, int err)
{
    __shared__ double lds[POTRF_LDS];
    potrf_wave(A + (int64_t)blockIdx.x * strideA, lda, bs, Linv + (int64_t)blockIdx.x * strideL, status, err, lds);
}

__global__ __launch_bounds__(256) void gemm64_kernel(GemmArgs g)
{
    __shared__ double lds[GEMM_LDS];
    gemm64_tile(g, blockIdx.y, blockIdx.x, lds);
}

// Two independent products in one launch (blockIdx.z picks the problem): the small products of a
// factorisation step are latency-bound, so pairing them halves the number of launches.
__global__ __launch_bounds__(256) void gemm64_dual_kernel(GemmArgs g0, GemmArgs g1)
{
    __shared__ double lds[GEMM_LDS];
    if (blockIdx.z == 0) gemm64_tile(g0, blockIdx.y, blockIdx.x, lds);
    else gemm64_tile(g1, blockIdx.y, blockIdx.x, lds);
}

// The trailing update of a factorisation step (g0: A22 -= L21 L21^T, lower tiles) and the update of
// Y below the step's block row (g1), with the NEXT step's diagonal block looked ahead: the workgroup
// that updates tile (0, 0) of A22 -- the next diagonal block -- goes on to factor it and invert its
// factor (one wavefront), while the other workgroups do the rest of the two updates.  The
// factorisation of a diagonal block (about 35 us on one wavefront) is the longest item of a step; this
// takes it off the stream's serial chain.  That workgroup is the first one dispatched.
struct LookAhead {
    double *Akk;     // tile (0, 0) of A22
    int lda, bs;
    double *Linv;    // NB x NB out
    int *status;
};

__global__ __launch_bounds__(256) void trailing_lookahead_kernel(GemmArgs g0, GemmArgs g1, LookAhead la)
{
    // (the factorisation reuses the tile product's LDS: the two never overlap in time)
    __shared__ double lds[POTRF_LDS > GEMM_LDS ? POTRF_LDS : GEMM_LDS];
    if (blockIdx.z != 0) {
        gemm64_tile(g1, blockIdx.y, blockIdx.x, lds);
        return;
    }
    gemm64_tile(g0, blockIdx.y, blockIdx.x, lds);
    if (blockIdx.x != 0 || blockIdx.y != 0) return;
    __threadfence();                           // the tile's entries, written by four waves, ...
    __syncthreads();                           // ... are read back by the first
    if (threadIdx.x < 64) potrf_wave(la.Akk, la.lda, la.bs, la.Linv, la.status, OBC_ERR_NOT_SPD, lds);
}

// Y = identity (d x d)
__global__ void eye_f64_kernel(double *__restrict__ dst, int d)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < (int64_t)d * d) dst[e] = (e / d == e % d) ? 1.0 : 0.0;
}

inline dim3 grid64(int M, int N) { return dim3((N + NB - 1) / NB, (M + NB - 1) / NB); }

}  // namespace

extern "C" {

int obc_invert_workspace_bytes(int d, size_t *bytes)
{
    if (!bytes || d <= 0) return OBC_ERR_BAD_ARG;
    size_t nblk = (size_t)(d + NB - 1) / NB;
    size_t mat = obc_align_up((size_t)d * d * sizeof(double), 256);
    size_t blocks = obc_align_up(nblk * NB * NB * sizeof(double), 256);
    *bytes = 2 * mat + blocks;
    return OBC_OK;
}

}  // extern "C"

namespace {

// Steps 1 and 2 on the workspace `ws` (laid out as obc_invert_workspace_bytes says): on return
// *Yout is L^-1 in fp64, lower triangular with exact zeros above the diagonal.
int factor_inverse(obc_ctx *ctx, const float *H, int d, void *ws, double **Yout)
{
    hipStream_t st = ctx->stream;
    const int nblk = (d + NB - 1) / NB;
    const size_t mat = obc_align_up((size_t)d * d * sizeof(double), 256);
    char *base = (char *)ws;
    double *A = (double *)base;
    double *Y = (double *)(base + mat);
    double *Lb = (double *)(base + 2 * mat);
    const int64_t n = (int64_t)d * d;

    f32_to_f64_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(H, A, n);
    eye_f64_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(Y, d);
    OBC_LAUNCH_CHECK(ctx, "f32_to_f64_kernel");

    auto dual_grid = [](const GemmArgs &a, const GemmArgs &b) {
        unsigned gx = (unsigned)((((a.N > b.N) ? a.N : b.N) + NB - 1) / NB);
        unsigned gy = (unsigned)((((a.M > b.M) ? a.M : b.M) + NB - 1) / NB);
        return dim3(gx, gy, 2);
    };

    // 1 + 2. Cholesky A = L L^T and Y = L^-1 together, block column by block column.  Step kb:
    //   (L_kk and its inverse: by the previous step's launch B; the first block by a launch of its own)
    //   launch A: L21 = A21 Linv_kk^T   |  Y[kb] = Linv_kk Y[kb]
    //   launch B: A22 -= L21 L21^T (lower tiles)  |  Y[rows below] -= L21 Y[kb]
    //             | the next diagonal block, once updated, is factored and its factor inverted
    // (Y starts as the identity: forward substitution on the identity, right-looking; before step
    // kb its block row kb holds I_kb - sum_{j<kb} L[kb,j] Y[j], non-zero only in columns < k0 + bs.)
    for (int kb = 0; kb < nblk; ++kb) {
        const int k0 = kb * NB;
        const int bs = (d - k0 < NB) ? d - k0 : NB;
        const int nc = k0 + bs;
        const int m = d - k0 - bs;
        double *Akk = A + (int64_t)k0 * d + k0;
        double *Lk = Lb + (int64_t)kb * NB * NB;
        double *Yk = Y + (int64_t)k0 * d;
        if (kb == 0) potrf_wave_kernel<<<1, 64, 0, st>>>(Akk, d, bs, Lk, ctx->d_status, 0, 0, OBC_ERR_NOT_SPD);
        // each workgroup overwrites exactly the rows / columns it has read
        GemmArgs trsm_row = mk(bs, nc, bs, 1.0, Lk, NB, 1, Yk, d, 1, 0.0, Yk, d, 0, 0, nullptr);
        if (m > 0) {
            double *A21 = A + (int64_t)(k0 + bs) * d + k0;
            double *A22 = A + (int64_t)(k0 + bs) * d + (k0 + bs);
            GemmArgs panel = mk(m, bs, bs, 1.0, A21, d, 1, Lk, 1, NB, 0.0, A21, d, 0, 0, nullptr);
            gemm64_dual_kernel<<<dual_grid(panel, trsm_row), 256, 0, st>>>(panel, trsm_row);
            GemmArgs trail = mk(m, m, bs, -1.0, A21, d, 1, A21, 1, d, 1.0, A22, d, 1, 0, nullptr);
            GemmArgs trsm_upd = mk(m, nc, bs, -1.0, A21, d, 1, Yk, d, 1, 1.0, Y + (int64_t)(k0 + bs) * d, d, 0, 0, nullptr);
            LookAhead la;
            la.Akk = A22; la.lda = d; la.bs = (m < NB) ? m : NB; la.Linv = Lk + (int64_t)NB * NB;
            la.status = ctx->d_status;
            trailing_lookahead_kernel<<<dual_grid(trail, trsm_upd), 256, 0, st>>>(trail, trsm_upd, la);
        } else {
            gemm64_kernel<<<grid64(bs, nc), 256, 0, st>>>(trsm_row);
        }
    }
    OBC_LAUNCH_CHECK(ctx, "factorisation kernels");
    *Yout = Y;
    return OBC_OK;
}

// 3. H^-1 = Y^T Y, rounded to fp32, mirrored
int inverse_from_factor(obc_ctx *ctx, const double *Y, int d, float *H)
{
    gemm64_kernel<<<grid64(d, d), 256, 0, ctx->stream>>>(mk(d, d, d, 1.0, Y, 1, d, Y, d, 1, 0.0, nullptr, d, 1, 2, H));
    OBC_LAUNCH_CHECK(ctx, "gemm64_kernel");
    return OBC_OK;
}

}  // namespace

namespace obc_rows {

// R independent 64 x 64 symmetric positive definite matrices M (row-major, lower triangle used,
// R x 4096 doubles) -> their Cholesky factors in place and the inverses of the factors in T
// (R x 4096 doubles, zeros above the diagonal).  A bad pivot latches OBC_ERR_NUMERIC.
int potrf64_batched_launch(obc_ctx *ctx, double *M, double *T, int R)
{
    if (R <= 0) return OBC_OK;
    potrf_wave_kernel<<<R, 64, 0, ctx->stream>>>(M, NB, NB, T, ctx->d_status, (int64_t)NB * NB, (int64_t)NB * NB,
                                                 OBC_ERR_NUMERIC);
    OBC_LAUNCH_CHECK(ctx, "potrf_wave_kernel");
    return OBC_OK;
}

}  // namespace obc_rows

extern "C" {

int obc_invert(obc_ctx *ctx, float *H, int d, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!H) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_invert: null matrix");
    if (d <= 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_invert: d must be positive");
    size_t need;
    obc_invert_workspace_bytes(d, &need);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "obc_invert: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    double *Y;
    int rc = factor_inverse(ctx, H, d, ws, &Y);
    if (rc != OBC_OK) return rc;
    rc = inverse_from_factor(ctx, Y, d, H);
    if (rc != OBC_OK) return rc;
    return obc_check(ctx);
}

int obc_refit_workspace_bytes(int d_col, int d_row, size_t *bytes)
{
    if (!bytes || d_col <= 0 || d_row <= 0) return OBC_ERR_BAD_ARG;
    size_t inv;
    obc_invert_workspace_bytes(d_col, &inv);
    *bytes = inv + 2 * obc_align_up((size_t)d_row * d_col * sizeof(double), 256);
    return OBC_OK;
}

int obc_refit(obc_ctx *ctx, float *H, int d_col, const float *C, int d_row, float *W_out,
              int invert_in_place, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!H || !C || !W_out) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_refit: null H, C or W_out");
    if (d_col <= 0 || d_row <= 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_refit: d_col and d_row must be positive");
    size_t need, inv;
    obc_refit_workspace_bytes(d_col, d_row, &need);
    obc_invert_workspace_bytes(d_col, &inv);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "obc_refit: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    hipStream_t st = ctx->stream;
    const int d = d_col, R = d_row;
    double *Y;
    int rc = factor_inverse(ctx, H, d, ws, &Y);
    if (rc != OBC_OK) return rc;
    const size_t rd = obc_align_up((size_t)R * d * sizeof(double), 256);
    double *C64 = (double *)((char *)ws + inv);
    double *T1 = (double *)((char *)ws + inv + rd);
    const int64_t n = (int64_t)R * d;
    f32_to_f64_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(C, C64, n);
    // W = C H^-1 = (C Y^T) Y with Y = L^-1: both products in fp64
    gemm64_kernel<<<grid64(R, d), 256, 0, st>>>(mk(R, d, d, 1.0, C64, d, 1, Y, 1, d, 0.0, T1, d, 0, 0, nullptr));
    gemm64_kernel<<<grid64(R, d), 256, 0, st>>>(mk(R, d, d, 1.0, T1, d, 1, Y, d, 1, 0.0, C64, d, 0, 1, nullptr));
    f64_to_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(C64, W_out, n);
    OBC_LAUNCH_CHECK(ctx, "refit kernels");
    if (invert_in_place) {
        rc = inverse_from_factor(ctx, Y, d, H);
        if (rc != OBC_OK) return rc;
    }
    return obc_check(ctx);
}

}  // extern "C"
