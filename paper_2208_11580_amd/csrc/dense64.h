// fp64 building blocks on 64 x 64 blocks, shared by the inverse (invert.hip) and the closed-form
// recovery of pruned rows (reconstruct.hip): the one-wavefront Cholesky factorisation + inverse of a
// diagonal block, and a 64 x 64 tile of a strided product on the fp64 matrix core
// (v_mfma_f64_16x16x4_f64).
#pragma once

#include "common.h"

namespace obc_dense64 {

constexpr int NB = 64;   // block-column width and GEMM tile edge
constexpr int GK = 16;   // GEMM k-slab
typedef double doublex4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double readlane_f64(double v, int l)
{
    long long b = __double_as_longlong(v);
    unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, l);
    unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)((unsigned long long)b >> 32), l);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// 1 / sqrt(x) in full fp64: hardware estimate and two Newton steps
__device__ __forceinline__ double rsqrt_f64(double x)
{
    double r = __builtin_amdgcn_rsq(x);
    r = r * (1.5 - 0.5 * x * r * r);
    r = r * (1.5 - 0.5 * x * r * r);
    return r;
}

// Factor the bs x bs (bs <= 64) diagonal block at A (leading dimension lda) in place (lower
// triangle), and write the inverse of that triangular factor to Linv (NB x NB, row-major, zeros
// above the diagonal).  A block smaller than 64 is padded with the identity.
//
// One wavefront, the block in LDS, worked on in 16 x 16 sub-blocks.  For each of the four block
// columns: the diagonal sub-block is factored and its factor inverted in registers (lane i < 16
// holds row i; values cross lanes with v_readlane), the sub-blocks below are multiplied by that
// inverse and the trailing sub-blocks updated, both on the fp64 matrix core
// (v_mfma_f64_16x16x4: lane l supplies a(i = l % 16, k = l / 16) and b(k = l / 16, j = l % 16)
// and holds c(4 r + l / 16, l % 16) in accumulator register r).  The off-diagonal sub-blocks of
// L^-1 then follow from  T_is = -T_ii sum_{s <= k < i} L_ik T_ks.
//
// LDS of one diagonal-block factorisation (doubles): the block, the inverse of its factor, one sub-block
constexpr int PL = NB + 1;
constexpr int SB = 16;                        // sub-block edge
constexpr int POTRF_LDS = 2 * NB * PL + SB * (SB + 1);

// The factorisation runs on ONE wavefront; its LDS accesses are ordered with this (all earlier LDS
// operations of the wavefront are complete and none later is moved before it).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
}

// The part of potrf_wave after the block has been parked in LDS: expects the block at lds[i * PL + j]
// (lower triangle; identity where the block is padded, zeros above the diagonal) and zeros in the
// NB * PL doubles after it, all visible to the calling wavefront.
__device__ __forceinline__ void potrf_wave_core(double *__restrict__ A, int lda, int bs, double *__restrict__ Linv,
                                                int *status, int err, double *lds);

__device__ __forceinline__ void potrf_wave(double *__restrict__ A, int lda, int bs, double *__restrict__ Linv,
                                           int *status, int err, double *lds)
{
    double *Ls = lds;                         // the block; becomes L (lower triangle)
    double *Ts = lds + NB * PL;               // L^-1
    const int lane = threadIdx.x & 63;
    // the block's rows are requested in batches of 16 (all in flight at once: each batch is one trip
    // to memory, and the block is on the factorisation's serial chain), then parked in LDS
#pragma unroll 1
    for (int i0 = 0; i0 < NB; i0 += 16) {
        double v[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = i0 + r;
            v[r] = (i == lane) ? 1.0 : 0.0;
            if (i < bs && lane <= i) v[r] = A[(int64_t)i * lda + lane];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            Ls[(i0 + r) * PL + lane] = v[r];
            Ts[(i0 + r) * PL + lane] = 0.0;
        }
    }
    wave_lds_sync();

    potrf_wave_core(A, lda, bs, Linv, status, err, lds);
}

__device__ __forceinline__ void potrf_wave_core(double *__restrict__ A, int lda, int bs, double *__restrict__ Linv,
                                                int *status, int err, double *lds)
{
    double *Ls = lds;
    double *Ts = lds + NB * PL;
    double *Xs = lds + 2 * NB * PL;
    const int lane = threadIdx.x & 63, l16 = lane & 15, lg = lane >> 4;
    bool bad = false;
#pragma unroll
    for (int s = 0; s < NB / SB; ++s) {
        const int o = SB * s;
        // (an opaque copy of the lane index per block column: otherwise the lane masks below are
        // shared by the four unrolled block columns and stay live in scalar registers throughout)
        int l16s = l16;
        asm volatile("" : "+v"(l16s));
        // ---- diagonal sub-block: row (o + l16) in registers (lanes >= 16 duplicate lanes < 16)
        double row[SB], rj[SB], t[SB];
#pragma unroll
        for (int c = 0; c < SB; ++c) row[c] = Ls[(o + l16) * PL + o + c];
#pragma unroll
        for (int j = 0; j < SB; ++j) {
            double pj = readlane_f64(row[j], j);
            if (!(pj > 0.0) || !(pj < __builtin_inf())) { bad = true; pj = 1.0; }
            const double r = rsqrt_f64(pj);
            rj[j] = r;                                          // 1 / L[j][j]
            const double cj = row[j] * r;
            row[j] = (l16s == j) ? pj * r : (l16s > j ? cj : 0.0);
            const double mine = (l16s > j) ? cj : 0.0;          // L[l16][j] below the diagonal
#pragma unroll
            for (int c = j + 1; c < SB; ++c) {
                const double lcj = readlane_f64(cj, c);         // L[c][j]
                row[c] = fma(-mine, lcj, row[c]);
                // pin the update here: left to itself the compiler defers it to the column's
                // turn and keeps every L[c][j] alive in scalar registers until then
                asm volatile("" : "+v"(row[c]));
            }
        }
        // ---- inverse of the 16 x 16 factor, lane c computes column c:
        //      t[i] = (delta_ic - sum_{k<i} L[i][k] t[k]) / L[i][i]
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            double acc = (l16s == i) ? 1.0 : 0.0;
            // the lane to read from, made to depend on the previous row's result: otherwise
            // the lane reads of all rows are issued up front and overflow the scalar registers
            int sel = i;
            if (i > 0) asm volatile("" : "+s"(sel) : "v"(t[i > 0 ? i - 1 : 0]));
#pragma unroll
            for (int k = 0; k < i; ++k) acc = fma(-readlane_f64(row[k], sel), t[k], acc);
            t[i] = acc * rj[i];
        }
        if (lane < SB) {
#pragma unroll
            for (int c = 0; c < SB; ++c) {
                Ls[(o + lane) * PL + o + c] = row[c];
                Ts[(o + c) * PL + o + lane] = t[c];
            }
        }
        wave_lds_sync();
        // ---- sub-blocks below: L_is = A_is T_ss^T
        doublex4 P[NB / SB];
#pragma unroll
        for (int ib = s + 1; ib < NB / SB; ++ib) {
            doublex4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kc = 0; kc < SB / 4; ++kc) {
                const double av = Ls[(SB * ib + l16) * PL + o + 4 * kc + lg];
                const double bv = Ts[(o + l16) * PL + o + 4 * kc + lg];
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
            }
            P[ib] = acc;
        }
        wave_lds_sync();
#pragma unroll
        for (int ib = s + 1; ib < NB / SB; ++ib)
#pragma unroll
            for (int r = 0; r < 4; ++r) Ls[(SB * ib + 4 * r + lg) * PL + o + l16] = P[ib][r];
        wave_lds_sync();
        // ---- trailing sub-blocks: A_ij -= L_is L_js^T  (s < j <= i)
#pragma unroll
        for (int ib = s + 1; ib < NB / SB; ++ib)
#pragma unroll
            for (int jb = s + 1; jb <= ib; ++jb) {
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
        wave_lds_sync();
    }
    // ---- off-diagonal sub-blocks of T = L^-1, block column by block column, top to bottom
#pragma unroll
    for (int s = 0; s + 1 < NB / SB; ++s)
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
    // results to memory, 16 rows per batch (all LDS reads of a batch in flight at once)
#pragma unroll 1
    for (int i0 = 0; i0 < NB; i0 += 16) {
        double lv[16], tv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            lv[r] = Ls[(i0 + r) * PL + lane];
            tv[r] = Ts[(i0 + r) * PL + lane];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = i0 + r;
            if (i < bs && lane <= i) A[(int64_t)i * lda + lane] = lv[r];
            Linv[i * NB + lane] = (lane <= i) ? tv[r] : 0.0;
        }
    }
    if (lane == 0 && bad) obc_latch(status, err);
}

// C (M x N, leading dimension ldc) = alpha * sum_k a(i,k) b(k,j) + beta * C, with
// a(i,k) = A[i*as_i + k*as_k] and b(k,j) = B[k*bs_k + j*bs_j] (strides express transposes).
//   lower_only : skip tiles strictly above the block diagonal
//   klo_mode   : 0 = k starts at 0; 1 = at the tile's first column (b is lower triangular);
//                2 = at max(first row, first column) (a^T and b lower triangular)
//   out32      : nullable; when given the result is rounded to fp32 there (leading dimension
//                ldc) and mirrored across the diagonal instead of being written to C
struct GemmArgs {
    int M, N, K;
    double alpha;
    const double *A;
    int64_t as_i, as_k;
    const double *B;
    int64_t bs_k, bs_j;
    double beta;
    double *C;
    int64_t ldc;
    int lower_only, klo_mode;
    float *out32;
};

constexpr int GEMM_LDS = 2 * GK * (NB + 1);   // doubles: the two operand slabs of a tile

__device__ __forceinline__ void gemm64_tile(const GemmArgs &g, int ti, int tj, double *lds)
{
    const int M = g.M, N = g.N, K = g.K;
    const double alpha = g.alpha, beta = g.beta;
    const double *A = g.A, *B = g.B;
    double *C = g.C;
    const int64_t as_i = g.as_i, as_k = g.as_k, bs_k = g.bs_k, bs_j = g.bs_j, ldc = g.ldc;
    const int lower_only = g.lower_only, klo_mode = g.klo_mode;
    float *out32 = g.out32;
    if (ti * NB >= M || tj * NB >= N) return;
    if (lower_only && tj > ti) return;
    double(*As)[NB + 1] = reinterpret_cast<double(*)[NB + 1]>(lds);
    double(*Bs)[NB + 1] = reinterpret_cast<double(*)[NB + 1]>(lds + GK * (NB + 1));
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;   // 2 x 2 waves, 32 x 32 outputs each (2 x 2 MFMA tiles)
    const int i0 = ti * NB, j0 = tj * NB;
    int kbeg = 0;
    if (klo_mode == 1) kbeg = j0;
    if (klo_mode == 2) kbeg = i0 > j0 ? i0 : j0;
    kbeg = kbeg / GK * GK;

    doublex4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = doublex4{0.0, 0.0, 0.0, 0.0};

    const bool a_kfast = (as_k == 1);
    const bool b_jfast = (bs_j == 1);
    // the next k-slab is fetched into registers while the current one is multiplied
    double ra[4], rb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            int e = tid + h * 256;
            int i, k;
            if (a_kfast) { i = e / GK; k = e % GK; } else { k = e / NB; i = e % NB; }
            double v = 0.0;
            if (i0 + i < M && k0 + k < K) v = A[(int64_t)(i0 + i) * as_i + (int64_t)(k0 + k) * as_k];
            ra[h] = v;
            int j, kb;
            if (b_jfast) { kb = e / NB; j = e % NB; } else { j = e / GK; kb = e % GK; }
            double u = 0.0;
            if (j0 + j < N && k0 + kb < K) u = B[(int64_t)(k0 + kb) * bs_k + (int64_t)(j0 + j) * bs_j];
            rb[h] = u;
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            int e = tid + h * 256;
            int i, k;
            if (a_kfast) { i = e / GK; k = e % GK; } else { k = e / NB; i = e % NB; }
            As[k][i] = ra[h];
            int j, kb;
            if (b_jfast) { kb = e / NB; j = e % NB; } else { j = e / GK; kb = e % GK; }
            Bs[kb][j] = rb[h];
        }
    };
    if (kbeg < K) fetch(kbeg);
    for (int k0 = kbeg; k0 < K; k0 += GK) {
        stash();
        __syncthreads();
        if (k0 + GK < K) fetch(k0 + GK);
        // v_mfma_f64_16x16x4: lane l supplies a(i = l % 16, k = l / 16) and b(k = l / 16, j = l % 16)
        const int kl = lane >> 4, il = lane & 15;
#pragma unroll
        for (int kk = 0; kk < GK; kk += 4) {
            double a0 = As[kk + kl][wm * 32 + il];
            double a1 = As[kk + kl][wm * 32 + 16 + il];
            double b0 = Bs[kk + kl][wn * 32 + il];
            double b1 = Bs[kk + kl][wn * 32 + 16 + il];
            acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }
    // accumulator layout of the fp64 16x16 MFMA: lane holds column (lane % 16) and rows
    // 4 * r + lane / 16, r = 0..3
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int i = i0 + wm * 32 + mt * 16 + 4 * r + (lane >> 4);
                int j = j0 + wn * 32 + nt * 16 + (lane & 15);
                if (i >= M || j >= N) continue;
                double av = acc[mt][nt][r];
                if (out32) {
                    float v = (float)(alpha * av);
                    out32[(int64_t)i * ldc + j] = v;
                    if (ti != tj) out32[(int64_t)j * ldc + i] = v;
                } else {
                    double v = alpha * av;
                    if (beta != 0.0) v += beta * C[(int64_t)i * ldc + j];
                    C[(int64_t)i * ldc + j] = v;
                }
            }
}

__host__ __device__ inline GemmArgs mk(int M, int N, int K, double alpha, const double *A, int64_t as_i, int64_t as_k, const double *B,
            int64_t bs_k, int64_t bs_j, double beta, double *C, int64_t ldc, int lower_only, int klo_mode,
            float *out32)
{
    GemmArgs g;
    g.M = M; g.N = N; g.K = K; g.alpha = alpha; g.A = A; g.as_i = as_i; g.as_k = as_k; g.B = B;
    g.bs_k = bs_k; g.bs_j = bs_j; g.beta = beta; g.C = C; g.ldc = ldc; g.lower_only = lower_only;
    g.klo_mode = klo_mode; g.out32 = out32;
    return g;
}

}  // namespace obc_dense64
