// obc_invert: H^-1 of the dampened Hessian through its Cholesky factor (Sec. 4 Step 1 of
// arxiv 2208.11580 needs the full inverse once per layer).
//
// This step is Theta(d^3) once per layer, next to Theta(d_row d^3) for the row solver, so it is
// written for accuracy first: everything is done in fp64 and only the final result is rounded
// to fp32 (the fp32 Hessians of correlated post-ReLU activations have condition numbers of
// 1e4..1e5; an fp32 factorisation would already cost three to four digits of H^-1).
//
//   1. A = double(H);  blocked right-looking Cholesky A = L L^T with 64-wide block columns, one
//      launch per block column (chol_step_kernel): every 64 x 64 tile of the trailing update forms
//      the piece of the panel it needs itself, the workgroup of the next diagonal block goes on to
//      factor that block and invert its factor on a single wavefront (16 x 16 sub-blocks in
//      registers, the rest of the block on the fp64 matrix core out of LDS).
//   2. Y = L^-1 by right-looking blocked forward substitution on the identity, in the same launches.
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

// ---- one factorisation step in one launch ----------------------------------------------------
// 64 x 64 x (K <= 64) products with the whole contraction staged in LDS at once: every operand is
// requested from memory before any is waited for, so a product costs one trip to memory instead of
// one per 16-wide slab.  Operand tiles sit k-major in LDS, S[k * PL + i], padded like the
// factorisation's block (PL = 65) so that both can use the same memory.

// 16 elements per thread of a rows x cols piece of a row-major matrix (element e = tid + 256 h is
// (e / 64, e % 64): consecutive threads read along a row); zero outside the piece
__device__ __forceinline__ void tile_fetch(double (&r)[16], const double *__restrict__ p, int64_t ld, int rows, int cols)
{
#pragma unroll
    for (int h = 0; h < 16; ++h) {
        const int e = threadIdx.x + h * 256;
        const int row = e >> 6, col = e & 63;
        r[h] = (row < rows && col < cols) ? p[(int64_t)row * ld + col] : 0.0;
    }
}
// park a fetched piece in LDS: element (row, col) at S[row][col], or transposed at S[col][row]
template <bool TRANSPOSE>
__device__ __forceinline__ void tile_park(double *S, const double (&r)[16])
{
#pragma unroll
    for (int h = 0; h < 16; ++h) {
        const int e = threadIdx.x + h * 256;
        const int row = e >> 6, col = e & 63;
        S[TRANSPOSE ? col * PL + row : row * PL + col] = r[h];
    }
}
// acc(i, j) (+)= sum_k As[k][i] Bs[k][j] over all 64 k; wave (wm, wn) of the 2 x 2 owns 32 x 32 outputs.
// v_mfma_f64_16x16x4: lane l supplies a(i = l % 16, k = l / 16) and b(k = l / 16, j = l % 16) and
// holds c(4 r + l / 16, l % 16) in accumulator register r.
template <bool ACCUMULATE = false>
__device__ __forceinline__ void tile_mma(doublex4 (&acc)[2][2], const double *As, const double *Bs)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1, kl = lane >> 4, il = lane & 15;
    if (!ACCUMULATE) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) acc[a][b] = doublex4{0.0, 0.0, 0.0, 0.0};
    }
#pragma unroll
    for (int kk = 0; kk < NB; kk += 4) {
        const double a0 = As[(kk + kl) * PL + wm * 32 + il], a1 = As[(kk + kl) * PL + wm * 32 + 16 + il];
        const double b0 = Bs[(kk + kl) * PL + wn * 32 + il], b1 = Bs[(kk + kl) * PL + wn * 32 + 16 + il];
        acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
    }
}
// visit the calling thread's 16 accumulator entries: f(row, col, value)
template <typename F>
__device__ __forceinline__ void tile_each(doublex4 (&acc)[2][2], F f)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                f(wm * 32 + a * 16 + 4 * r + (lane >> 4), wn * 32 + b * 16 + (lane & 15), (double)acc[a][b][r]);
}
// set them: acc(row, col) = f(row, col)
template <typename F>
__device__ __forceinline__ void tile_fill(doublex4 (&acc)[2][2], F f)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[a][b][r] = f(wm * 32 + a * 16 + 4 * r + (lane >> 4), wn * 32 + b * 16 + (lane & 15));
}

template <typename F>
__device__ __forceinline__ void tile_each2(doublex4 (&x)[2][2], doublex4 (&y)[2][2], F f)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                f(wm * 32 + a * 16 + 4 * r + (lane >> 4), wn * 32 + b * 16 + (lane & 15), (double)x[a][b][r], (double)y[a][b][r]);
}

// Step 3: tile (ti, tj), tj <= ti, of H^-1 = Y^T Y with Y = L^-1 lower triangular: the sum runs over
// k >= the tile's first row only.  Y's rows are the contraction index, so both operand tiles are
// pieces of Y as they lie in memory; 64-deep slabs, requested two ahead.  The result is rounded to fp32 and written on both sides of the diagonal.
__global__ __launch_bounds__(256) void yty_kernel(const double *__restrict__ Y, int d, float *__restrict__ H)
{
    __shared__ double lds[2 * NB * PL];
    double *As = lds, *Bs = lds + NB * PL;
    const int ti = blockIdx.y, tj = blockIdx.x;
    if (tj > ti) return;
    const int i0 = ti * NB, j0 = tj * NB;
    const int Mi = (d - i0 < NB) ? d - i0 : NB, Nj = (d - j0 < NB) ? d - j0 : NB;
    const bool diag = (ti == tj);
    doublex4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = doublex4{0.0, 0.0, 0.0, 0.0};
    // two slabs are in flight at any time (the long tiles near the top of the triangle are a chain of
    // d / 64 slabs each: what they wait for is memory latency)
    double ra[2][16], rb[2][16];
    auto fetch = [&](int k0, double (&fa)[16], double (&fb)[16]) {
        const int kr = (d - k0 < NB) ? d - k0 : NB;
        tile_fetch(fa, Y + (int64_t)k0 * d + i0, d, kr, Mi);              // a(i, k) = Y[k][i0 + i]
        if (!diag) tile_fetch(fb, Y + (int64_t)k0 * d + j0, d, kr, Nj);   // b(k, j) = Y[k][j0 + j]
    };
    auto slab = [&](int knext, double (&fa)[16], double (&fb)[16]) {
        tile_park<false>(As, fa);
        if (!diag) tile_park<false>(Bs, fb);
        __syncthreads();
        if (knext < d) fetch(knext, fa, fb);
        tile_mma<true>(acc, As, diag ? As : Bs);
        __syncthreads();
    };
    fetch(i0, ra[0], rb[0]);
    if (i0 + NB < d) fetch(i0 + NB, ra[1], rb[1]);
    for (int k0 = i0; k0 < d; k0 += 2 * NB) {
        slab(k0 + 2 * NB, ra[0], rb[0]);
        if (k0 + NB >= d) break;
        slab(k0 + 3 * NB, ra[1], rb[1]);
    }
    tile_each(acc, [&](int i, int j, double v) {
        if (i < Mi && j < Nj) {
            const float f = (float)v;
            H[(int64_t)(i0 + i) * d + j0 + j] = f;
            if (!diag) H[(int64_t)(j0 + j) * d + i0 + i] = f;
        }
    });
}

// C (M x N, row-major) = A B over k in a range that skips known zeros, in 64 x 64 tiles with 64-deep
// slabs requested two ahead (as yty_kernel).  A is row-major (M x K, leading dimension lda); B is
// either B_T: given as its transpose (b(k, j) = Bt[j][k]; with `tri` the rows of Bt are those of a
// lower triangular matrix, so k stops at the end of the tile's last column) or plain (b(k, j) =
// B[k][j]; with `tri` B is lower triangular and k starts at the tile's first column).
template <bool B_T>
__global__ __launch_bounds__(256) void slab_gemm_kernel(const double *__restrict__ A, int64_t lda,
                                                        const double *__restrict__ B, int64_t ldb,
                                                        double *__restrict__ C, int64_t ldc, int M, int N, int K, int tri)
{
    __shared__ double lds[2 * NB * PL];
    double *As = lds, *Bs = lds + NB * PL;
    const int i0 = blockIdx.y * NB, j0 = blockIdx.x * NB;
    if (i0 >= M || j0 >= N) return;
    const int Mi = (M - i0 < NB) ? M - i0 : NB, Nj = (N - j0 < NB) ? N - j0 : NB;
    const int kbeg = (!B_T && tri) ? j0 : 0;
    const int kend = (B_T && tri && j0 + NB < K) ? j0 + NB : K;
    doublex4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = doublex4{0.0, 0.0, 0.0, 0.0};
    double ra[2][16], rb[2][16];
    auto fetch = [&](int k0, double (&fa)[16], double (&fb)[16]) {
        const int kr = (kend - k0 < NB) ? kend - k0 : NB;
        tile_fetch(fa, A + (int64_t)i0 * lda + k0, lda, Mi, kr);                  // (i, k)
        if (B_T) tile_fetch(fb, B + (int64_t)j0 * ldb + k0, ldb, Nj, kr);         // (j, k)
        else tile_fetch(fb, B + (int64_t)k0 * ldb + j0, ldb, kr, Nj);             // (k, j)
    };
    auto slab = [&](int knext, double (&fa)[16], double (&fb)[16]) {
        tile_park<true>(As, fa);
        if (B_T) tile_park<true>(Bs, fb);
        else tile_park<false>(Bs, fb);
        __syncthreads();
        if (knext < kend) fetch(knext, fa, fb);
        tile_mma<true>(acc, As, Bs);
        __syncthreads();
    };
    fetch(kbeg, ra[0], rb[0]);
    if (kbeg + NB < kend) fetch(kbeg + NB, ra[1], rb[1]);
    for (int k0 = kbeg; k0 < kend; k0 += 2 * NB) {
        slab(k0 + 2 * NB, ra[0], rb[0]);
        if (k0 + NB >= kend) break;
        slab(k0 + 3 * NB, ra[1], rb[1]);
    }
    tile_each(acc, [&](int i, int j, double v) {
        if (i < Mi && j < Nj) C[(int64_t)(i0 + i) * ldc + j0 + j] = v;
    });
}

// The diagonal-block factorisation of potrf_wave for a whole workgroup of four wavefronts, block
// already in LDS (layout and contract of potrf_wave_core; the factor is not written out).  The 64
// dependent column steps stay on wavefront 0, everything else moves off its chain:
//  * wavefront 0 factors a whole 16-column panel at a time -- lane l holds row (16 s + l) of the
//    panel, so the sub-blocks below the diagonal one come out of the same instructions as the
//    diagonal sub-block (no product with its inverse);
//  * the inverse of diagonal sub-block s - 1 is computed by wavefront 1 while wavefront 0 factors
//    panel s;
//  * the trailing sub-block updates of a panel are dealt to all four wavefronts, the three block
//    columns of the off-diagonal part of L^-1 to three of them, the final stores to all.
// LDS: POTRF_LDS doubles as for potrf_wave, then two more 16 x 17 scratch sub-blocks, then 2 x 16
// reciprocal pivots.
// rsqrt_f64 (hardware estimate and two Newton steps) one operation at a time, so that the caller can
// place the nine dependent operations among independent work: stage 0 .. 8, result in r after stage 8
__device__ __forceinline__ void rsqrt_stage(int st, double x, double &r, double &a)
{
    switch (st) {
    case 0: r = __builtin_amdgcn_rsq(x); break;
    case 1: case 5: a = r * r; break;
    case 2: case 6: a = x * a; break;
    case 3: case 7: a = fma(-0.5, a, 1.5); break;
    case 4: case 8: r = r * a; break;
    default: break;
    }
}

constexpr int POTRF_WG_LDS = POTRF_LDS + 2 * SB * (SB + 1) + 2 * SB;

__device__ __forceinline__ void potrf_wg_core(double *__restrict__ Linv, int *status, int err, double *lds)
{
    double *Ls = lds;
    double *Ts = lds + NB * PL;
    double *Xs0 = lds + 2 * NB * PL;
    double *Rj = lds + POTRF_LDS + 2 * SB * (SB + 1);
    const int lane = threadIdx.x & 63, l16 = lane & 15, lg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    bool bad = false;

    // inverse of the 16 x 16 factor at sub-block o (rows in LDS, reciprocal pivots in rjs), lane c
    // computes column c:  t[i] = (delta_ic - sum_{k<i} L[i][k] t[k]) / L[i][i]
    auto invert_diag = [&](int o, const double *rjs) {
        double row[SB], t[SB];
#pragma unroll
        for (int c = 0; c < SB; ++c) row[c] = Ls[(o + l16) * PL + o + c];
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            double acc = (l16 == i) ? 1.0 : 0.0;
            // the lane to read from, made to depend on the previous row's result: otherwise
            // the lane reads of all rows are issued up front and overflow the scalar registers
            int sel = i;
            if (i > 0) asm volatile("" : "+s"(sel) : "v"(t[i > 0 ? i - 1 : 0]));
#pragma unroll
            for (int k = 0; k < i; ++k) acc = fma(-readlane_f64(row[k], sel), t[k], acc);
            t[i] = acc * rjs[i];
        }
        if (lane < SB) {
#pragma unroll
            for (int c = 0; c < SB; ++c) Ts[(o + c) * PL + o + lane] = t[c];
        }
    };

#pragma unroll
    for (int s = 0; s < NB / SB; ++s) {
        const int o = SB * s;
        if (wave == 0) {
            // ---- panel s: row (o + lane) in registers
            int ls = lane;
            asm volatile("" : "+v"(ls));   // (an opaque copy per panel: keeps the lane masks out of scalar registers)
            const bool has = o + lane < NB;
            double row[SB], rj[SB];
#pragma unroll
            for (int c = 0; c < SB; ++c) row[c] = has ? Ls[(o + lane) * PL + o + c] : 0.0;
            // The pivot of column j + 1 is known as soon as column j has updated row entry j + 1: its
            // reciprocal square root (a chain of dependent fp64 operations) is started right there,
            // among the remaining updates of column j, instead of after them.
            double pj = readlane_f64(row[0], 0);
            if (!(pj > 0.0) || !(pj < __builtin_inf())) { bad = true; pj = 1.0; }
            double r = rsqrt_f64(pj);
#pragma unroll
            for (int j = 0; j < SB; ++j) {
                rj[j] = r;                                          // 1 / L[j][j]
                const double cj = row[j] * r;
                row[j] = (ls == j) ? pj * r : (ls > j ? cj : 0.0);
                const double mine = (ls > j) ? cj : 0.0;            // L[o + lane][j] below the diagonal
                double pn = 1.0, rn = 1.0, an = 0.0;
#pragma unroll
                for (int c = j + 1; c < SB; ++c) {
                    const double lcj = readlane_f64(cj, c);         // L[o + c][j]
                    row[c] = fma(-mine, lcj, row[c]);
                    // pin the update here: left to itself the compiler defers it to the column's
                    // turn and keeps every L[c][j] alive in scalar registers until then
                    asm volatile("" : "+v"(row[c]));
                    if (c == j + 1) {
                        pn = readlane_f64(row[c], c);
                        if (!(pn > 0.0) || !(pn < __builtin_inf())) { bad = true; pn = 1.0; }
                    }
                    rsqrt_stage(c - (j + 1), pn, rn, an);           // one operation of it per update
                }
#pragma unroll
                for (int st = (SB - 1 - j > 0 ? SB - 1 - j : 0); st < 9; ++st) rsqrt_stage(st, pn, rn, an);
                pj = pn;
                r = rn;
            }
            if (has) {
#pragma unroll
                for (int c = 0; c < SB; ++c) Ls[(o + lane) * PL + o + c] = row[c];
            }
            if (lane == 0) {
#pragma unroll
                for (int j = 0; j < SB; ++j) Rj[(s & 1) * SB + j] = rj[j];
            }
        } else if (wave == 1 && s > 0) {
            double rjs[SB];
#pragma unroll
            for (int i = 0; i < SB; ++i) rjs[i] = Rj[((s - 1) & 1) * SB + i];
            invert_diag(o - SB, rjs);
        }
        __syncthreads();                       // panel s (and the inverse of sub-block s - 1) in LDS
        // ---- trailing sub-blocks: A_ij -= L_is L_js^T  (s < j <= i), dealt to the four wavefronts
        int pair = 0;
#pragma unroll
        for (int ib = s + 1; ib < NB / SB; ++ib)
#pragma unroll
            for (int jb = s + 1; jb <= ib; ++jb, ++pair) {
                if ((pair & 3) != wave) continue;
                doublex4 acc;
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = Ls[(SB * ib + 4 * r + lg) * PL + SB * jb + l16];
#pragma unroll
                for (int kc = 0; kc < SB / 4; ++kc) {
                    const double av = -Ls[(SB * ib + l16) * PL + o + 4 * kc + lg];
                    const double bv = Ls[(SB * jb + l16) * PL + o + 4 * kc + lg];
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) Ls[(SB * ib + 4 * r + lg) * PL + SB * jb + l16] = acc[r];
            }
        if (s + 1 < NB / SB) __syncthreads();
    }
    if (wave == 1) {
        double rjs[SB];
#pragma unroll
        for (int i = 0; i < SB; ++i) rjs[i] = Rj[((NB / SB - 1) & 1) * SB + i];
        invert_diag(NB - SB, rjs);
    }
    __syncthreads();
    // ---- off-diagonal sub-blocks of T = L^-1: block column s on wavefront s, top to bottom
    //      T_is = -T_ii sum_{s <= k < i} L_ik T_ks  (a wavefront only reads what it wrote itself,
    //      the factor and the diagonal sub-blocks)
#pragma unroll
    for (int s = 0; s + 1 < NB / SB; ++s) {
        if (wave != s) continue;
        double *Xs = Xs0 + s * SB * (SB + 1);
#pragma unroll
        for (int ib = s + 1; ib < NB / SB; ++ib) {
            doublex4 x = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kb = s; kb < ib; ++kb)
#pragma unroll
                for (int kc = 0; kc < SB / 4; ++kc) {
                    const double av = Ls[(SB * ib + l16) * PL + SB * kb + 4 * kc + lg];
                    const double bv = Ts[(SB * kb + 4 * kc + lg) * PL + SB * s + l16];
                    x = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, x, 0, 0, 0);
                }
#pragma unroll
            for (int r = 0; r < 4; ++r) Xs[(4 * r + lg) * (SB + 1) + l16] = x[r];
            wave_lds_sync();
            doublex4 y = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kc = 0; kc < SB / 4; ++kc) {
                const double av = -Ts[(SB * ib + l16) * PL + SB * ib + 4 * kc + lg];
                const double bv = Xs[(4 * kc + lg) * (SB + 1) + l16];
                y = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, y, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) Ts[(SB * ib + 4 * r + lg) * PL + SB * s + l16] = y[r];
            wave_lds_sync();
        }
    }
    __syncthreads();
    // ---- L^-1 to memory (it also stays in LDS for the caller): 16 rows per wavefront
    {
        double tv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) tv[r] = Ts[(wave * 16 + r) * PL + lane];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = wave * 16 + r;
            Linv[i * NB + lane] = (lane <= i) ? tv[r] : 0.0;
        }
    }
    if (threadIdx.x == 0 && bad) obc_latch(status, err);
}

// One step of the factorisation (block column kb, columns k0 .. k0 + bs) in ONE launch.  With
// T = L_kk^-1 and G = T^T T = A_kk^-1 (both left by the step before), P = the block column below the
// diagonal block as the earlier trailing updates left it (L21 = P T^T is never formed or stored),
// and Yk = block row kb of Y before its own solve:
//   z = 0, tile (i, j), j <= i:   A22[i, j] -= (P_i G) P_j^T            (= L21_i L21_j^T)
//   z = 1, tile (i, c):           Y[below][i, c] -= (P_i G) Yk[c]       (= L21_i (T Yk)[c])
//   z = 2, tile c:                Y[kb - 1][c] = T_prev Y[kb - 1][c]    (the previous block row's solve:
//                                 nobody reads its unsolved values any more)
// Every z = 0 / 1 workgroup forms its own Q = P_i G in LDS first: the panel solve that used to be a
// launch of its own on the stream's serial chain now costs each tile one more small product.  The
// workgroup of tile (0, 0), the first one dispatched, keeps the block it has just updated -- the next
// diagonal block -- in LDS, factors it there on one wavefront, and leaves T and G for the next step.
// Per step the stream waits for: one trip to memory, two tile products, one 64 x 64 factorisation,
// one product out of LDS.
struct StepArgs {
    double *A, *Y;
    int d, k0, bs;
    const double *T, *G;         // of this step's diagonal block (NB x NB, row-major)
    const double *Tprev;         // of the previous step's; its block row starts at kprev0 (bsprev rows,
    int kprev0, bsprev;          // ncprev = kprev0 + bsprev columns); bsprev = 0: nothing to finish
    double *Tnext, *Gnext;       // out: of the next diagonal block
    int *status;
};

__global__ __launch_bounds__(256) void chol_step_kernel(StepArgs s)
{
    // (the factorisation reuses the products' LDS: they never overlap in time)
    __shared__ double lds[POTRF_WG_LDS];
    double *As = lds, *Bs = lds + NB * PL;
    const int d = s.d, k0 = s.k0, bs = s.bs;
    const int nc = k0 + bs, m = d - nc;
    doublex4 acc[2][2];
    if (blockIdx.z == 2) {
        const int ncprev = s.kprev0 + s.bsprev, c0 = blockIdx.x * NB;
        if (blockIdx.y != 0 || s.bsprev <= 0 || c0 >= ncprev) return;
        double *Yp = s.Y + (int64_t)s.kprev0 * d + c0;
        const int Nc = (ncprev - c0 < NB) ? ncprev - c0 : NB;
        double ra[16], rb[16];
        tile_fetch(ra, s.Tprev, NB, s.bsprev, s.bsprev);     // a(i, k) = T[i][k]
        tile_fetch(rb, Yp, d, s.bsprev, Nc);                 // b(k, j) = Y[k][j]
        tile_park<true>(As, ra);
        tile_park<false>(Bs, rb);
        __syncthreads();
        tile_mma(acc, As, Bs);
        // the workgroup overwrites exactly the block it has read
        tile_each(acc, [&](int i, int j, double v) { if (i < s.bsprev && j < Nc) Yp[(int64_t)i * d + j] = v; });
        return;
    }
    const int ti = blockIdx.y, tj = blockIdx.x;
    const int i0 = ti * NB;
    if (i0 >= m) return;
    if (blockIdx.z == 0 && tj > ti) return;
    if (blockIdx.z == 1 && tj * NB >= nc) return;
    const int Mi = (m - i0 < NB) ? m - i0 : NB;
    // the second product's right operand and the tile it updates
    const bool upd_a = (blockIdx.z == 0);
    const int j0 = tj * NB;
    const int Nj = upd_a ? ((m - j0 < NB) ? m - j0 : NB) : ((nc - j0 < NB) ? nc - j0 : NB);
    double *C = upd_a ? s.A + (int64_t)(nc + i0) * d + nc + j0 : s.Y + (int64_t)(nc + i0) * d + j0;
    {
        double rp[16], rg[16];
        tile_fetch(rp, s.A + (int64_t)(nc + i0) * d + k0, d, Mi, bs);    // a(i, k) = P_i[i][k]
        tile_fetch(rg, s.G, NB, bs, bs);                                   // b(k, j) = G[k][j]
        tile_park<true>(As, rp);
        tile_park<false>(Bs, rg);
    }
    double rb[16];
    if (upd_a) tile_fetch(rb, s.A + (int64_t)(nc + j0) * d + k0, d, Nj, bs);   // b(k, j) = P_j[j][k]
    else tile_fetch(rb, s.Y + (int64_t)k0 * d + j0, d, bs, Nj);                 // b(k, j) = Yk[k][j]
    doublex4 cold[2][2];
    tile_fill(cold, [&](int i, int j) { return (i < Mi && j < Nj) ? C[(int64_t)i * d + j] : 0.0; });
    __syncthreads();
    tile_mma(acc, As, Bs);                      // Q = P_i G
    __syncthreads();                            // everybody is done reading As / Bs
    tile_each(acc, [&](int i, int j, double v) { As[j * PL + i] = v; });   // a(i, k) = Q[i][k]
    if (upd_a) tile_park<true>(Bs, rb);
    else tile_park<false>(Bs, rb);
    __syncthreads();
    tile_mma(acc, As, Bs);                      // Q B
    const bool chain = upd_a && ti == 0 && tj == 0;
    if (!chain) {
        tile_each2(acc, cold, [&](int i, int j, double v, double c) {
            if (i < Mi && j < Nj) C[(int64_t)i * d + j] = c - v;
        });
        return;
    }
    // the next diagonal block goes straight into the factorisation's LDS layout (lower triangle,
    // identity where the block is padded), the inverse's area is cleared
    __syncthreads();                            // everybody is done reading As / Bs
    tile_each2(acc, cold, [&](int i, int j, double v, double c) {
        As[i * PL + j] = (i < Mi && j <= i) ? c - v : (i == j ? 1.0 : 0.0);
        Bs[i * PL + j] = 0.0;
    });
    __syncthreads();
    // (the factor itself is not needed again: T and G carry the step)
    potrf_wg_core(s.Tnext, s.status, OBC_ERR_NOT_SPD, lds);
    __syncthreads();                            // T of the next block, in LDS where the factorisation left it
    tile_mma(acc, Bs, Bs);                      // G = T^T T
    tile_each(acc, [&](int i, int j, double v) { s.Gnext[i * NB + j] = v; });
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
    size_t blocks = obc_align_up(2 * nblk * NB * NB * sizeof(double), 256);   // T and G of every diagonal block
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

    // 1 + 2. Cholesky A = L L^T and Y = L^-1 together, block column by block column, one launch per
    // step (chol_step_kernel); the first diagonal block and the last block row have launches of
    // their own.  (Y starts as the identity: forward substitution on the identity, right-looking;
    // before step kb its block row kb holds I_kb - sum_{j<kb} L[kb,j] Y[j], non-zero only in columns
    // < k0 + bs.)
    double *Gb = Lb + (int64_t)nblk * NB * NB;
    {
        const int bs0 = d < NB ? d : NB;
        potrf_wave_kernel<<<1, 64, 0, st>>>(A, d, bs0, Lb, ctx->d_status, 0, 0, OBC_ERR_NOT_SPD);
        gemm64_kernel<<<1, 256, 0, st>>>(mk(NB, NB, NB, 1.0, Lb, 1, NB, Lb, NB, 1, 0.0, Gb, NB, 0, 0, nullptr));
    }
    int kprev0 = 0, bsprev = 0;
    for (int kb = 0; kb < nblk; ++kb) {
        const int k0 = kb * NB;
        const int bs = (d - k0 < NB) ? d - k0 : NB;
        const int nc = k0 + bs;
        const int m = d - nc;
        double *Tk = Lb + (int64_t)kb * NB * NB;
        if (m > 0) {
            StepArgs sa;
            sa.A = A; sa.Y = Y; sa.d = d; sa.k0 = k0; sa.bs = bs;
            sa.T = Tk; sa.G = Gb + (int64_t)kb * NB * NB;
            sa.Tprev = (kb > 0) ? Tk - (int64_t)NB * NB : nullptr;
            sa.kprev0 = kprev0; sa.bsprev = bsprev;
            sa.Tnext = Tk + (int64_t)NB * NB; sa.Gnext = Gb + (int64_t)(kb + 1) * NB * NB;
            sa.status = ctx->d_status;
            const int tm = (m + NB - 1) / NB, tc = (nc + NB - 1) / NB;
            chol_step_kernel<<<dim3((unsigned)(tm > tc ? tm : tc), (unsigned)tm, 3), 256, 0, st>>>(sa);
        } else {
            // the last block column: finish the previous block row and this one
            if (bsprev > 0) {
                double *Yp = Y + (int64_t)kprev0 * d;
                const int ncp = kprev0 + bsprev;
                gemm64_kernel<<<grid64(bsprev, ncp), 256, 0, st>>>(
                    mk(bsprev, ncp, bsprev, 1.0, Tk - (int64_t)NB * NB, NB, 1, Yp, d, 1, 0.0, Yp, d, 0, 0, nullptr));
            }
            double *Yk = Y + (int64_t)k0 * d;
            gemm64_kernel<<<grid64(bs, nc), 256, 0, st>>>(mk(bs, nc, bs, 1.0, Tk, NB, 1, Yk, d, 1, 0.0, Yk, d, 0, 0, nullptr));
        }
        kprev0 = k0;
        bsprev = bs;
    }
    OBC_LAUNCH_CHECK(ctx, "factorisation kernels");
    *Yout = Y;
    return OBC_OK;
}

// 3. H^-1 = Y^T Y, rounded to fp32, mirrored
int inverse_from_factor(obc_ctx *ctx, const double *Y, int d, float *H)
{
    yty_kernel<<<grid64(d, d), 256, 0, ctx->stream>>>(Y, d, H);
    OBC_LAUNCH_CHECK(ctx, "yty_kernel");
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
    slab_gemm_kernel<true><<<grid64(R, d), 256, 0, st>>>(C64, d, Y, d, T1, d, R, d, d, 1);     // T1 = C Y^T
    slab_gemm_kernel<false><<<grid64(R, d), 256, 0, st>>>(T1, d, Y, d, C64, d, R, d, d, 1);    // W = T1 Y
    f64_to_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(C64, W_out, n);
    OBC_LAUNCH_CHECK(ctx, "refit kernels");
    if (invert_in_place) {
        rc = inverse_from_factor(ctx, Y, d, H);
        if (rc != OBC_OK) return rc;
    }
    return obc_check(ctx);
}

}  // extern "C"
