// obc_reconstruct_rows: the weights of a given mask by the group-OBS closed form (Sec. 4 Step 2 of
// arxiv 2208.11580; the sign as in eq. (5)).  With P the pruned indices of a row,
//
//     w_hat = w - H^-1[:, P] ((H^-1)[P, P])^-1 w_P,        w_hat[P] = 0,
//
// from the ORIGINAL weights and inverse Hessian: no trace and no second run of the greedy loop.  The
// paper names it as the cheaper way to get a row's weights once the global step has fixed how many
// weights the row gives up.
//
// Everything in fp64 (the principal submatrix of H^-1 on half of the indices is as ill-conditioned as
// H^-1 itself, and its fp32 entries are exact inputs), all rows of the layer side by side:
//   1. per row: the list P of its pruned indices, G = (H^-1)[P, P] (lower triangle) and w_P in the
//      workspace (recon_prepare_kernel)
//   2. G = L L^T for all rows at once, block column by block column of 64, three launches per step
//      (host loop up to the caller's bound on the pruned count; a row that is through skips): the
//      diagonal blocks on one wavefront each (factor + inverse of the factor), the panels below them
//      and the trailing updates as 64 x 64 tile products on the fp64 matrix core -- the device code
//      obc_invert uses, here with one grid dimension running over the rows
//   3. per row: L y = w_P and L^T z = y block by block with the inverted diagonal factors, then
//      w_hat = w - H^-1[:, P] z along rows of H^-1 (it is symmetric), pruned entries set to 0
//      (recon_solve_kernel)
#include "dense64.h"

namespace {

using namespace obc_dense64;

struct ReconArgs {
    const float *W, *Hinv;
    const uint8_t *mask;
    int d, cmax, ldg;
    float *W_out;
    double *G;       // R x ldg x ldg
    double *Linv;    // R x (ldg / 64) x 64 x 64
    double *vec;     // R x ldg   (w_P, then y, then z)
    int *idx;        // R x ldg
    int *cnt;        // R     pruned weights of the row (0: nothing to do)
    int *status;
};

// ---- 1. pruned indices (ascending), their count, G and the right-hand side
__global__ __launch_bounds__(256) void recon_prepare_kernel(ReconArgs a)
{
    __shared__ int wcnt[4];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int d = a.d, ldg = a.ldg;
    const float *w = a.W + (size_t)row * d;
    float *wo = a.W_out + (size_t)row * d;
    const uint8_t *mk_row = a.mask + (size_t)row * d;
    int *idx = a.idx + (size_t)row * ldg;
    double *G = a.G + (size_t)row * ldg * ldg;
    double *v = a.vec + (size_t)row * ldg;

    int c = 0;                               // (every thread ends with the same count)
    for (int j0 = 0; j0 < d; j0 += 256) {
        const int j = j0 + tid;
        const bool pr = j < d && mk_row[j] != 0;
        const unsigned long long bal = __ballot(pr);
        if (lane == 0) wcnt[wave] = __popcll(bal);
        __syncthreads();
        int before = c, total = 0;
        for (int wv = 0; wv < 4; ++wv) {
            if (wv < wave) before += wcnt[wv];
            total += wcnt[wv];
        }
        const int rank = before + __popcll(bal & ((1ull << lane) - 1ull));
        if (pr && rank < a.cmax) idx[rank] = j;
        c += total;
        __syncthreads();
    }
    for (int j = tid; j < d; j += 256) wo[j] = w[j];
    if (c > a.cmax) {                        // more pruned weights than the workspace was sized for:
        if (tid == 0) {                      // the row stays a copy of W
            obc_latch(a.status, OBC_ERR_WORKSPACE);
            a.cnt[row] = 0;
        }
        return;
    }
    if (tid == 0) a.cnt[row] = c;
    if (c == 0) return;
    __threadfence_block();
    __syncthreads();
    for (int i = 0; i < c; ++i) {
        const float *hrow = a.Hinv + (size_t)idx[i] * d;
        for (int j = tid; j <= i; j += 256) G[(size_t)i * ldg + j] = (double)hrow[idx[j]];
    }
    for (int i = tid; i < c; i += 256) v[i] = (double)w[idx[i]];
}

// ---- 2. one block column (first index k0) of the factorisation, for every row that still has it
__global__ __launch_bounds__(64) void recon_potrf_kernel(ReconArgs a, int k0)
{
    __shared__ double lds[POTRF_LDS];
    const int row = blockIdx.x;
    const int c = a.cnt[row];
    if (k0 >= c) return;
    const int bs = (c - k0 < NB) ? c - k0 : NB;
    double *G = a.G + (size_t)row * a.ldg * a.ldg;
    double *Lk = a.Linv + ((size_t)row * (a.ldg / NB) + k0 / NB) * NB * NB;
    potrf_wave(G + (size_t)k0 * a.ldg + k0, a.ldg, bs, Lk, a.status, OBC_ERR_NUMERIC, lds);
}

// panel (trailing == 0): L21 = A21 Linv_kk^T, one workgroup per 64 rows of it (each overwrites exactly
// what it has read); trailing (== 1): A22 -= L21 L21^T, one workgroup per lower 64 x 64 tile
// (blockIdx.x enumerates the tiles of the largest row; smaller rows skip what they do not have)
__global__ __launch_bounds__(256) void recon_update_kernel(ReconArgs a, int k0, int trailing)
{
    __shared__ double lds[GEMM_LDS];
    const int row = blockIdx.y;
    const int c = a.cnt[row];
    const int m = c - k0 - NB;               // rows below a full diagonal block
    if (m <= 0) return;
    const int ldg = a.ldg;
    double *G = a.G + (size_t)row * ldg * ldg;
    const double *Lk = a.Linv + ((size_t)row * (ldg / NB) + k0 / NB) * NB * NB;
    double *A21 = G + (size_t)(k0 + NB) * ldg + k0;
    if (!trailing) {
        const int ti = blockIdx.x;
        if (ti * NB >= m) return;
        gemm64_tile(mk(m, NB, NB, 1.0, A21, ldg, 1, Lk, 1, NB, 0.0, A21, ldg, 0, 0, nullptr), ti, 0, lds);
    } else {
        // tile number -> (ti, tj), tj <= ti
        int t = blockIdx.x, ti = 0;
        while (t > ti) { t -= ti + 1; ++ti; }
        const int tj = t;
        if (ti * NB >= m) return;
        double *A22 = G + (size_t)(k0 + NB) * ldg + (k0 + NB);
        gemm64_tile(mk(m, m, NB, -1.0, A21, ldg, 1, A21, 1, ldg, 1.0, A22, ldg, 1, 0, nullptr), ti, tj, lds);
    }
}

// ---- 3. L y = w_P, L^T z = y (v holds w_P, y and z in turn), then w_hat = w - H^-1[:, P] z
__global__ __launch_bounds__(256) void recon_solve_kernel(ReconArgs a)
{
    __shared__ double blk[NB];
    const int row = blockIdx.x, tid = threadIdx.x;
    const int d = a.d, ldg = a.ldg;
    const int c = a.cnt[row];
    if (c == 0) return;
    const float *w = a.W + (size_t)row * d;
    float *wo = a.W_out + (size_t)row * d;
    const int *idx = a.idx + (size_t)row * ldg;
    const double *G = a.G + (size_t)row * ldg * ldg;
    const double *Li = a.Linv + (size_t)row * (ldg / NB) * NB * NB;
    double *v = a.vec + (size_t)row * ldg;
    const int nblk = (c + NB - 1) / NB;
    for (int kb = 0; kb < nblk; ++kb) {
        const int k0 = kb * NB;
        const int bs = (c - k0 < NB) ? c - k0 : NB;
        const double *Lk = Li + (size_t)kb * NB * NB;
        if (tid < bs) {
            double acc = 0.0;
            for (int j = 0; j <= tid; ++j) acc = fma(Lk[tid * NB + j], v[k0 + j], acc);
            blk[tid] = acc;
        }
        __syncthreads();
        if (tid < bs) v[k0 + tid] = blk[tid];
        for (int i = k0 + bs + tid; i < c; i += 256) {
            const double *gi = G + (size_t)i * ldg + k0;
            double acc = 0.0;
            for (int j = 0; j < bs; ++j) acc = fma(gi[j], blk[j], acc);
            v[i] -= acc;
        }
        __threadfence_block();
        __syncthreads();
    }
    for (int kb = nblk - 1; kb >= 0; --kb) {
        const int k0 = kb * NB;
        const int bs = (c - k0 < NB) ? c - k0 : NB;
        const double *Lk = Li + (size_t)kb * NB * NB;
        if (tid < bs) {
            double acc = 0.0;
            for (int j = tid; j < bs; ++j) acc = fma(Lk[j * NB + tid], v[k0 + j], acc);
            blk[tid] = acc;
        }
        __syncthreads();
        if (tid < bs) v[k0 + tid] = blk[tid];
        for (int i = tid; i < k0; i += 256) {
            double acc = 0.0;
            for (int r = 0; r < bs; ++r) acc = fma(G[(size_t)(k0 + r) * ldg + i], blk[r], acc);
            v[i] -= acc;
        }
        __threadfence_block();
        __syncthreads();
    }
    // (row idx[t] of the symmetric H^-1 is its column idx[t])
    for (int j = tid; j < d; j += 256) {
        double acc = 0.0;
        for (int t = 0; t < c; ++t) acc = fma((double)a.Hinv[(size_t)idx[t] * d + j], v[t], acc);
        wo[j] = (float)((double)w[j] - acc);
    }
    __syncthreads();
    for (int t = tid; t < c; t += 256) wo[idx[t]] = 0.f;
}

size_t recon_carve(ReconArgs *a, void *base, int R, int cmax)
{
    const size_t ldg = obc_align_up((size_t)(cmax > 0 ? cmax : 1), NB);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += obc_align_up(bytes, 256);
        return base ? (char *)base + o : (char *)nullptr;
    };
    char *pg = take((size_t)R * ldg * ldg * sizeof(double));
    char *pl = take((size_t)R * ldg * NB * sizeof(double));
    char *pv = take((size_t)R * ldg * sizeof(double));
    char *pi = take((size_t)R * ldg * sizeof(int));
    char *pc = take((size_t)R * sizeof(int));
    if (a) {
        a->G = (double *)pg; a->Linv = (double *)pl; a->vec = (double *)pv; a->idx = (int *)pi; a->cnt = (int *)pc;
        a->ldg = (int)ldg;
    }
    return off;
}

}  // namespace

extern "C" {

int obc_reconstruct_workspace_bytes(int R, int d, int max_pruned, size_t *bytes)
{
    if (!bytes || R < 0 || d <= 0 || max_pruned < 0 || max_pruned > d) return OBC_ERR_BAD_ARG;
    *bytes = recon_carve(nullptr, nullptr, R, max_pruned);
    return OBC_OK;
}

int obc_reconstruct_rows(obc_ctx *ctx, const float *W, const float *Hinv, const uint8_t *mask, int R, int d,
                         int max_pruned, float *W_out, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!W || !Hinv || !mask || !W_out) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_reconstruct_rows: null argument");
    if (R < 0 || d <= 0 || max_pruned < 0 || max_pruned > d)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_reconstruct_rows: bad size");
    ReconArgs a;
    const size_t need = recon_carve(&a, ws, R, max_pruned);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "obc_reconstruct_rows: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    if (R == 0) return OBC_OK;
    a.W = W; a.Hinv = Hinv; a.mask = mask; a.d = d; a.cmax = max_pruned; a.W_out = W_out; a.status = ctx->d_status;
    hipStream_t st = ctx->stream;
    recon_prepare_kernel<<<R, 256, 0, st>>>(a);
    OBC_LAUNCH_CHECK(ctx, "recon_prepare_kernel");
    for (int k0 = 0; k0 < max_pruned; k0 += NB) {
        recon_potrf_kernel<<<R, 64, 0, st>>>(a, k0);
        const int mt = (max_pruned - k0 - NB + NB - 1) / NB;      // 64-row tiles below the block, at most
        if (mt > 0) {
            recon_update_kernel<<<dim3(mt, R), 256, 0, st>>>(a, k0, 0);
            recon_update_kernel<<<dim3(mt * (mt + 1) / 2, R), 256, 0, st>>>(a, k0, 1);
        }
    }
    recon_solve_kernel<<<R, 256, 0, st>>>(a);
    OBC_LAUNCH_CHECK(ctx, "closed-form recovery kernels");
    return OBC_OK;
}

}  // extern "C"
