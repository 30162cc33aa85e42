// obc_invert: H^-1 of the dampened Hessian through its Cholesky factor (Sec. 4 Step 1 of
// arxiv 2208.11580 needs the full inverse once per layer).
//
// This step is Theta(d^3) once per layer, next to Theta(d_row d^3) for the row solver, so it is
// written for accuracy first: everything is done in fp64 and only the final result is rounded
// to fp32 (the fp32 Hessians of correlated post-ReLU activations have condition numbers of
// 1e4..1e5; an fp32 factorisation would already cost three to four digits of H^-1).
//
//   1. A = double(H);  blocked right-looking Cholesky A = L L^T with 64-wide block columns:
//      diagonal block factored (and inverted) inside one workgroup's LDS, the panel below is a
//      product with the inverted diagonal block, the trailing update is a tiled GEMM.
//   2. Y = L^-1 by blocked forward substitution (two GEMMs per block row).
//   3. H^-1 = Y^T Y, lower tiles only, mirrored on store so the result is exactly symmetric.
#include "common.h"

namespace {

constexpr int NB = 64;   // block-column width and GEMM tile edge
constexpr int GK = 16;   // GEMM k-slab

__global__ void f32_to_f64_kernel(const float *__restrict__ src, double *__restrict__ dst, int64_t n)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) dst[e] = (double)src[e];
}

__global__ void zero_f64_kernel(double *__restrict__ dst, int64_t n)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) dst[e] = 0.0;
}

// Factor the bs x bs diagonal block at A (leading dimension lda) in place (lower triangle), and
// write the inverse of that triangular factor to Linv (NB x NB, row-major, zeros above the diagonal).
__global__ __launch_bounds__(256) void potrf_block_kernel(double *__restrict__ A, int lda, int bs,
                                                          double *__restrict__ Linv, int *status)
{
    __shared__ double S[NB][NB + 1];
    __shared__ double T[NB][NB + 1];
    __shared__ int bad;
    const int tid = threadIdx.x;
    if (tid == 0) bad = 0;
    for (int e = tid; e < NB * NB; e += 256) {
        int i = e / NB, j = e % NB;
        S[i][j] = (i < bs && j <= i) ? A[(int64_t)i * lda + j] : 0.0;
        T[i][j] = 0.0;
    }
    __syncthreads();
    for (int j = 0; j < bs; ++j) {
        if (tid == 0) {
            double p = S[j][j];
            if (!(p > 0.0) || !isfinite(p)) { bad = 1; p = 1.0; }
            S[j][j] = sqrt(p);
        }
        __syncthreads();
        double ljj = S[j][j];
        for (int i = j + 1 + tid; i < bs; i += 256) S[i][j] /= ljj;
        __syncthreads();
        // trailing update of the lower triangle: S[i][c] -= S[i][j] * S[c][j], j < c <= i
        int n = bs - j - 1;
        for (int e = tid; e < n * n; e += 256) {
            int i = j + 1 + e / n, c = j + 1 + e % n;
            if (c <= i) S[i][c] -= S[i][j] * S[c][j];
        }
        __syncthreads();
    }
    // inverse of the triangular block, one column per thread
    if (tid < bs) {
        int c = tid;
        T[c][c] = 1.0 / S[c][c];
        for (int i = c + 1; i < bs; ++i) {
            double s = 0.0;
            for (int k = c; k < i; ++k) s -= S[i][k] * T[k][c];
            T[i][c] = s / S[i][i];
        }
    }
    __syncthreads();
    for (int e = tid; e < NB * NB; e += 256) {
        int i = e / NB, j = e % NB;
        if (i < bs && j <= i) A[(int64_t)i * lda + j] = S[i][j];
        Linv[e] = T[i][j];
    }
    if (tid == 0 && bad) obc_latch(status, OBC_ERR_NOT_SPD);
}

// C (M x N, leading dimension ldc) = alpha * sum_k a(i,k) b(k,j) + beta * C, with
// a(i,k) = A[i*as_i + k*as_k] and b(k,j) = B[k*bs_k + j*bs_j] (strides express transposes).
//   lower_only : skip tiles strictly above the block diagonal
//   klo_mode   : 0 = k starts at 0; 1 = at the tile's first column (b is lower triangular);
//                2 = at max(first row, first column) (a^T and b lower triangular)
//   out32      : nullable; when given the result is rounded to fp32 there (leading dimension
//                ldc) and mirrored across the diagonal instead of being written to C
__global__ __launch_bounds__(256) void gemm64_kernel(int M, int N, int K, double alpha,
                                                     const double *A, int64_t as_i, int64_t as_k,
                                                     const double *B, int64_t bs_k, int64_t bs_j,
                                                     double beta, double *C, int64_t ldc,
                                                     int lower_only, int klo_mode, float *out32)
{
    const int ti = blockIdx.y, tj = blockIdx.x;
    if (lower_only && tj > ti) return;
    __shared__ double As[GK][NB + 1];
    __shared__ double Bs[GK][NB + 1];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;   // 16 x 16 threads, 4 x 4 outputs each
    const int i0 = ti * NB, j0 = tj * NB;
    int kbeg = 0;
    if (klo_mode == 1) kbeg = j0;
    if (klo_mode == 2) kbeg = i0 > j0 ? i0 : j0;
    kbeg = kbeg / GK * GK;

    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;

    const bool a_kfast = (as_k == 1);
    const bool b_jfast = (bs_j == 1);
    for (int k0 = kbeg; k0 < K; k0 += GK) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            int e = tid + h * 256;
            int i, k;
            if (a_kfast) { i = e / GK; k = e % GK; } else { k = e / NB; i = e % NB; }
            double v = 0.0;
            if (i0 + i < M && k0 + k < K) v = A[(int64_t)(i0 + i) * as_i + (int64_t)(k0 + k) * as_k];
            As[k][i] = v;
            int j, kb;
            if (b_jfast) { kb = e / NB; j = e % NB; } else { j = e / GK; kb = e % GK; }
            double u = 0.0;
            if (j0 + j < N && k0 + kb < K) u = B[(int64_t)(k0 + kb) * bs_k + (int64_t)(j0 + j) * bs_j];
            Bs[kb][j] = u;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            double a[4], b[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) a[r] = As[k][ty * 4 + r];
#pragma unroll
            for (int c = 0; c < 4; ++c) b[c] = Bs[k][tx * 4 + c];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = fma(a[r], b[c], acc[r][c]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            int i = i0 + ty * 4 + r, j = j0 + tx * 4 + c;
            if (i >= M || j >= N) continue;
            if (out32) {
                float v = (float)(alpha * acc[r][c]);
                if (ti != tj) {
                    out32[(int64_t)i * ldc + j] = v;
                    out32[(int64_t)j * ldc + i] = v;
                } else {
                    out32[(int64_t)i * ldc + j] = v;
                }
            } else {
                double v = alpha * acc[r][c];
                if (beta != 0.0) v += beta * C[(int64_t)i * ldc + j];
                C[(int64_t)i * ldc + j] = v;
            }
        }
}

// Copy the NB x NB inverse diagonal block into Y's diagonal block.
__global__ void place_block_kernel(const double *__restrict__ Linv, double *__restrict__ Y, int ldy, int bs)
{
    for (int e = threadIdx.x; e < NB * NB; e += blockDim.x) {
        int i = e / NB, j = e % NB;
        if (i < bs && j < bs) Y[(int64_t)i * ldy + j] = Linv[e];
    }
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
    size_t tmp = obc_align_up((size_t)NB * d * sizeof(double), 256);
    *bytes = 2 * mat + blocks + tmp;
    return OBC_OK;
}

int obc_invert(obc_ctx *ctx, float *H, int d, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!H) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_invert: null matrix");
    if (d <= 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_invert: d must be positive");
    size_t need;
    obc_invert_workspace_bytes(d, &need);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "obc_invert: workspace of %zu bytes needed, %zu given", need, ws_bytes);

    hipStream_t st = ctx->stream;
    const int nblk = (d + NB - 1) / NB;
    const size_t mat = obc_align_up((size_t)d * d * sizeof(double), 256);
    char *base = (char *)ws;
    double *A = (double *)base;
    double *Y = (double *)(base + mat);
    double *Lb = (double *)(base + 2 * mat);
    double *T = (double *)(base + 2 * mat + obc_align_up((size_t)nblk * NB * NB * sizeof(double), 256));
    const int64_t n = (int64_t)d * d;

    f32_to_f64_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(H, A, n);
    zero_f64_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(Y, n);
    OBC_LAUNCH_CHECK(ctx, "f32_to_f64_kernel");

    // 1. Cholesky, block column by block column
    for (int kb = 0; kb < nblk; ++kb) {
        const int k0 = kb * NB;
        const int bs = (d - k0 < NB) ? d - k0 : NB;
        double *Akk = A + (int64_t)k0 * d + k0;
        double *Lk = Lb + (int64_t)kb * NB * NB;
        potrf_block_kernel<<<1, 256, 0, st>>>(Akk, d, bs, Lk, ctx->d_status);
        const int m = d - k0 - bs;
        if (m > 0) {
            double *A21 = A + (int64_t)(k0 + bs) * d + k0;
            // L21 = A21 * Linv_kk^T  (each workgroup overwrites exactly the rows it has read)
            gemm64_kernel<<<grid64(m, bs), 256, 0, st>>>(m, bs, bs, 1.0, A21, d, 1, Lk, 1, NB, 0.0,
                                                          A21, d, 0, 0, nullptr);
            // A22 -= L21 L21^T on the lower tiles
            double *A22 = A + (int64_t)(k0 + bs) * d + (k0 + bs);
            gemm64_kernel<<<grid64(m, m), 256, 0, st>>>(m, m, bs, -1.0, A21, d, 1, A21, 1, d, 1.0,
                                                         A22, d, 1, 0, nullptr);
        }
    }
    OBC_LAUNCH_CHECK(ctx, "cholesky kernels");

    // 2. Y = L^-1, block row by block row
    for (int ib = 0; ib < nblk; ++ib) {
        const int i0 = ib * NB;
        const int bs = (d - i0 < NB) ? d - i0 : NB;
        const double *Li = Lb + (int64_t)ib * NB * NB;
        place_block_kernel<<<1, 256, 0, st>>>(Li, Y + (int64_t)i0 * d + i0, d, bs);
        if (i0 > 0) {
            // T = L[i0.., 0..i0) * Y[0..i0, 0..i0)   (Y lower triangular: k starts at the tile column)
            gemm64_kernel<<<grid64(bs, i0), 256, 0, st>>>(bs, i0, i0, 1.0, A + (int64_t)i0 * d, d, 1, Y, d, 1,
                                                           0.0, T, d, 0, 1, nullptr);
            // Y[i0.., 0..i0) = -Linv_ii * T
            gemm64_kernel<<<grid64(bs, i0), 256, 0, st>>>(bs, i0, bs, -1.0, Li, NB, 1, T, d, 1, 0.0,
                                                           Y + (int64_t)i0 * d, d, 0, 0, nullptr);
        }
    }
    OBC_LAUNCH_CHECK(ctx, "triangular inverse kernels");

    // 3. H^-1 = Y^T Y, rounded to fp32, mirrored
    gemm64_kernel<<<grid64(d, d), 256, 0, st>>>(d, d, d, 1.0, Y, 1, d, Y, d, 1, 0.0, nullptr, d, 1, 2, H);
    OBC_LAUNCH_CHECK(ctx, "gemm64_kernel");

    return obc_check(ctx);
}

}  // extern "C"
