// Row solver, rank-1 strategy: Algorithm 1 (pruning, with the N:M rule) and Algorithm 3 (OBQ)
// of arxiv 2208.11580 exactly as written -- one Lemma-1 elimination per greedy step.
//
// One workgroup owns one row of W and a private copy A of H^-1.  A lives in LDS when it fits
// (d <= 192: the whole loop then never touches HBM) and otherwise in the caller's workspace,
// where every step streams the live rows of A through the CU with float4 accesses.
//
// As in the blocked solver, the O(d) quantities that decide the argmin -- the weights and the
// maintained diagonal of A -- are kept in fp64; A itself is fp32.
//
// Per step: (1) argmin of the score over the live, eligible indices (per-thread scan, wave
// shuffle reduction, cross-wave LDS reduction; ties to the lowest index); (2) row p of A -- equal
// to column p, A stays symmetric -- is staged in LDS; (3) w and the maintained diagonal are
// updated; (4) A[i,:] -= (A[i,p] / A_pp) A[p,:] for the live rows i.  Eliminated rows are never
// read or written again; eliminated columns of live rows are updated but never read.
//
// Block pruning (Sec. 4 "Block-Sparsity", eq. (5)) runs in the same loop: every c-th step chooses
// a block by its score w_P^T ((H^-1)_P)^-1 w_P -- evaluated per candidate block as the sum of the
// c single-weight scores met when the block's indices are eliminated one after another inside a
// c x c copy -- and the next c steps take the block's indices in ascending order.  c single
// eliminations with the single-weight update give exactly the block update of eq. (5).
#include "rows_common.h"

namespace {

using namespace obc_rows;

struct Rank1Args {
    const float *W;
    const float *Hinv;
    float *Aws;              // R x d x d private copies, or nullptr when A is LDS-resident
    int R, d, k_steps;
    int nm_n, nm_m;
    const int32_t *stop_counts;
    const float *delta, *offset;
    int maxq;
    const uint8_t *live_in;
    int outliers;            // OBQ: restrict the choice to outliers while there are any
    int blk_c;               // block pruning: block size (0 otherwise)
    int32_t *order;
    float *loss;
    int32_t *codes;
    float *W_out;
    float *trace;
    int out_ld;              // leading dimension of order / loss / trace steps
    int *status;
};

// Score of one block for block pruning: v^T M^-1 v for the block's weights v and its c x c
// diagonal block M of the current inverse (diagonal from the fp64 copy, the rest from A), as
// the sum of v_k^2 / M_kk over a Gaussian elimination of the block.  NaN when a pivot fails.
template <int CMAX>
__device__ __forceinline__ double block_score(const double *w, const double *diag, const float *A, int d,
                                              int j0, int c)
{
    double v[CMAX], M[CMAX][CMAX];
#pragma unroll
    for (int i = 0; i < CMAX; ++i) {
        if (i >= c) continue;
        v[i] = w[j0 + i];
#pragma unroll
        for (int j = 0; j < CMAX; ++j) {
            if (j > i) continue;
            M[i][j] = (i == j) ? diag[j0 + i] : (double)A[(size_t)(j0 + i) * d + (j0 + j)];
        }
    }
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < CMAX; ++k) {
        if (k >= c) continue;
        const double piv = M[k][k];
        if (!(piv > 0.0)) return __builtin_nan("");
        const double ip = 1.0 / piv;
        s += v[k] * v[k] * ip;
#pragma unroll
        for (int i = 0; i < CMAX; ++i) {
            if (i <= k || i >= c) continue;
            const double f = M[i][k] * ip;
            v[i] -= f * v[k];
#pragma unroll
            for (int j = 0; j < CMAX; ++j) {
                if (j <= k || j > i) continue;
                M[i][j] -= f * M[j][k];
            }
        }
    }
    return s;
}

template <int MODE, int CMAX>
__global__ __launch_bounds__(1024) void rows_rank1_kernel(Rank1Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int d = a.d;
    const int row = blockIdx.x;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthr >> 6;
    const int dpad = (d + 3) & ~3;

    double *w = reinterpret_cast<double *>(smem);
    double *diag = w + dpad;
    float *colp = reinterpret_cast<float *>(diag + dpad);
    float *fcol = colp + dpad;
    uint16_t *lidx = reinterpret_cast<uint16_t *>(fcol + dpad);   // compact list of live indices
    uint16_t *pos = lidx + dpad;                        // position of index j in lidx (0xffff: not live)
    uint16_t *dead = pos + dpad;                        // indices removed up front (quant on survivors)
    float *red_s = reinterpret_cast<float *>(dead + dpad);
    int *red_j = reinterpret_cast<int *>(red_s + 32);
    int *misc = red_j + 32;                             // [0] live count, [1] dead count
    uint8_t *blk = reinterpret_cast<uint8_t *>(misc + 8);  // pruned weights per N:M block
    float *A = a.Aws ? a.Aws + (size_t)row * d * d
                     : reinterpret_cast<float *>(smem + obc_align_up(
                           (size_t)dpad * 30 + 72 * 4 + (a.nm_m > 0 ? (size_t)dpad : 0), 16));

    // ---- set-up: private copy of H^-1, the row, the diagonal, the live list
    const float *Hinv = a.Hinv;
    for (size_t e = tid; e < (size_t)d * d; e += nthr) A[e] = Hinv[e];
    for (int j = tid; j < d; j += nthr) {
        bool alive = (MODE != MODE_BLOCK && a.live_in) ? (a.live_in[(size_t)row * d + j] != 0) : true;
        w[j] = alive ? (double)a.W[(size_t)row * d + j] : 0.0;
        diag[j] = (double)Hinv[(size_t)j * d + j];
        pos[j] = alive ? 0 : 0xffff;
        if (MODE == MODE_QUANT) a.codes[(size_t)row * d + j] = -1;
    }
    if (a.nm_m > 0)
        for (int b = tid; b < d / a.nm_m; b += nthr) blk[b] = 0;
    __syncthreads();
    if (tid == 0) {
        int m = 0, nd = 0;
        for (int j = 0; j < d; ++j) {
            if (pos[j] == 0) { lidx[m] = (uint16_t)j; pos[j] = (uint16_t)m; ++m; }
            else dead[nd++] = (uint16_t)j;
        }
        misc[0] = m;
        misc[1] = nd;
    }
    __syncthreads();
    const int n_dead = misc[1];
    int m = misc[0];   // live count, tracked in a register by every thread

    int steps = a.k_steps;   // block pruning: block steps
    if (MODE == MODE_QUANT) steps = m;
    if (MODE == MODE_PRUNE && steps > m) steps = m;   // an already sparse row has fewer candidates
    if (a.stop_counts) {
        int sc = a.stop_counts[row];
        sc = sc < 0 ? 0 : sc;
        steps = sc < steps ? sc : steps;
    }
    double qd = 1.0, qo = 0.0;
    const double qmax = (double)a.maxq;
    if (MODE == MODE_QUANT) { qd = (double)a.delta[row]; qo = (double)a.offset[row]; }
    const double iqd = 1.0 / qd;

    const int bc = (MODE == MODE_BLOCK) ? a.blk_c : 1;
    if (MODE == MODE_BLOCK) steps *= bc;   // from here on in single eliminations
    int pblock = 0;                        // block being eliminated
    double block_loss = 0.0;               // its accumulated loss (thread 0)

    const bool vec4 = (d % 4 == 0);
    bool failed = false;

    // dead indices are eliminated first, in ascending order, with no weight change; they are
    // kept on a separate list, so the live list only ever holds survivors
    for (int t = -n_dead; t < steps; ++t) {
        int p;
        double target = 0.0, wp = 0.0, app;
        if (t < 0) {
            p = dead[t + n_dead];
            app = diag[p];
        } else if (MODE == MODE_BLOCK) {
            const int sub = t % bc;
            if (sub == 0) {
                // ---- (1) selection over the live blocks
                Cand c;
                c.s = __builtin_inff();
                c.j = 0x7fffffff;
                for (int b = tid; b < d / bc; b += nthr) {
                    if (pos[b * bc] == 0xffff) continue;
                    float s = (float)block_score<CMAX>(w, diag, A, d, b * bc, bc);
                    if (cand_less(s, b, c.s, c.j)) { c.s = s; c.j = b; }
                }
                c = block_argmin(c, red_s, red_j);
                pblock = c.j;
                if (pblock == 0x7fffffff) { failed = true; break; }
                block_loss = 0.0;
            }
            p = pblock * bc + sub;
            app = diag[p];
            wp = w[p];
            if (tid == 0) {
                block_loss += wp * wp / (2.0 * app);
                if (sub == bc - 1) {
                    a.order[(size_t)row * a.out_ld + t / bc] = pblock;
                    a.loss[(size_t)row * a.out_ld + t / bc] = (float)block_loss;
                }
            }
        } else {
            // ---- (1) selection: error in fp64, the compared ratio in fp32 (hardware reciprocal)
            Cand c;
            c.s = __builtin_inff();
            c.j = 0x7fffffff;
            for (int q = tid; q < m; q += nthr) {
                int j = lidx[q];
                if (a.nm_m > 0 && blk[j / a.nm_m] >= a.nm_m - a.nm_n) continue;
                double wj = w[j];
                double tj = 0.0;
                if (MODE == MODE_QUANT) {
                    double cq = rint((wj - qo) * iqd);
                    cq = fmin(fmax(cq, 0.0), qmax);
                    tj = qo + qd * cq;
                }
                double er = tj - wj;
                float s = (float)(er * er) * __builtin_amdgcn_rcpf((float)diag[j]);
                // an outlier (error beyond half a grid step) sorts before every non-outlier
                if (MODE == MODE_QUANT && a.outliers && fabs(er) > 0.5 * qd) s = outlier_first(s);
                if (cand_less(s, j, c.s, c.j)) { c.s = s; c.j = j; }
            }
            c = block_argmin(c, red_s, red_j);
            p = c.j;
            if (p == 0x7fffffff) { failed = true; break; }
            app = diag[p];
            wp = w[p];
            double code = 0.0;
            if (MODE == MODE_QUANT) {
                code = rint((wp - qo) * iqd);   // same expression as in the selection
                code = fmin(fmax(code, 0.0), qmax);
                target = qo + qd * code;
            }
            if (tid == 0) {
                double e = target - wp;
                a.order[(size_t)row * a.out_ld + t] = p;
                a.loss[(size_t)row * a.out_ld + t] = (float)(e * e / (2.0 * app));
                if (MODE == MODE_QUANT) a.codes[(size_t)row * d + p] = (int)code;
            }
        }
        if (!(app > 0.0) || !(app < __builtin_inf())) { failed = true; break; }
        const float appf = (float)app;

        // ---- (2) row p of A (= column p), and the multipliers A[i,p] / A_pp
        const float *Ap = A + (size_t)p * d;
        for (int j = tid; j < d; j += nthr) {
            float v = Ap[j];
            colp[j] = v;
            fcol[j] = __fdiv_rn(v, appf);
        }
        __syncthreads();

        // During the up-front phase the not-yet-eliminated dead indices still belong to the
        // matrix being reduced: their rows and diagonal entries are updated like live ones.
        const int dnext = t + n_dead + 1;
        const int rem = (t < 0) ? n_dead - dnext : 0;
        const int mtot = m + rem;

        // ---- (3) compensation of the live weights, maintained diagonal
        const double g = (wp - target) / app;
        const double invapp = 1.0 / app;
        for (int q = tid; q < mtot; q += nthr) {
            int j = (q < m) ? lidx[q] : dead[dnext + q - m];
            if (j == p) continue;
            const double cd = (double)colp[j];
            if (q < m) w[j] -= cd * g;
            diag[j] -= cd * cd * invapp;
        }

        // ---- (4) Lemma 1 on the remaining rows; one wave per row, float4 along the row
        for (int q = wave; q < mtot; q += nwaves) {
            int i = (q < m) ? lidx[q] : dead[dnext + q - m];
            if (i == p) continue;
            float f = fcol[i];
            float *Ai = A + (size_t)i * d;
            if (vec4) {
                for (int j = lane * 4; j < d; j += 256) {
                    float4 v = *reinterpret_cast<float4 *>(Ai + j);
                    float4 c4 = *reinterpret_cast<const float4 *>(colp + j);
                    v.x = fmaf(-f, c4.x, v.x);
                    v.y = fmaf(-f, c4.y, v.y);
                    v.z = fmaf(-f, c4.z, v.z);
                    v.w = fmaf(-f, c4.w, v.w);
                    *reinterpret_cast<float4 *>(Ai + j) = v;
                }
            } else {
                for (int j = lane; j < d; j += 64) Ai[j] = fmaf(-f, colp[j], Ai[j]);
            }
        }
        __syncthreads();

        // ---- bookkeeping: p leaves the live set
        if (t >= 0) {
            if (tid == 0) {
                w[p] = target;
                int qp = pos[p];
                int last = lidx[m - 1];
                lidx[qp] = (uint16_t)last;
                pos[last] = (uint16_t)qp;
                pos[p] = 0xffff;
                if (a.nm_m > 0) blk[p / a.nm_m] += 1;
            }
            m -= 1;
        }
        __syncthreads();
        if (t >= 0 && a.trace && (t + 1) % bc == 0) {
            float *tr = a.trace + ((size_t)row * a.out_ld + t / bc) * d;
            for (int j = tid; j < d; j += nthr) tr[j] = (float)w[j];
        }
    }

    if (failed && tid == 0) obc_latch(a.status, OBC_ERR_NUMERIC);
    // trace entries of the steps this row does not take are zero
    if (a.trace) {
        const int t0 = (steps < 0 ? 0 : steps) / bc;
        const int t1 = (MODE == MODE_QUANT) ? t0 : a.k_steps;
        for (int t = t0; t < t1; ++t) {
            float *tr = a.trace + ((size_t)row * a.out_ld + t) * d;
            for (int j = tid; j < d; j += nthr) tr[j] = 0.f;
        }
    }
    __syncthreads();
    for (int j = tid; j < d; j += nthr) a.W_out[(size_t)row * d + j] = (float)w[j];
}

inline size_t rank1_vec_lds(int d, int nm_m)
{
    size_t dpad = (size_t)((d + 3) & ~3);
    return obc_align_up(dpad * 30 + 72 * 4 + (nm_m > 0 ? dpad : 0), 16);
}

constexpr size_t LDS_LIMIT = 160 * 1024;

}  // namespace

namespace obc_rows {

// True when A fits in LDS next to the row vectors.
bool rank1_lds_resident(int d, int nm_m)
{
    return rank1_vec_lds(d, nm_m) + (size_t)d * d * 4 <= LDS_LIMIT;
}

size_t rank1_workspace_bytes(int R, int d)
{
    if (rank1_lds_resident(d, 8)) return 256;
    return obc_align_up((size_t)R * d * d * sizeof(float), 256);
}

int rank1_launch(obc_ctx *ctx, int mode, const float *W, const float *Hinv, int R, int d, int k_steps,
                 int nm_n, int nm_m, int blk_c, const int32_t *stop_counts, const float *delta,
                 const float *offset, int maxq, const uint8_t *live, int flags, int32_t *order, float *loss,
                 int32_t *codes, float *W_out, float *trace, int out_ld, void *ws, size_t ws_bytes)
{
    ctx->chain_fresh = false;   // whatever ran since the last timed launch is not part of this one
    Rank1Args a;
    a.outliers = (flags & OBC_QUANT_OUTLIERS) ? 1 : 0;
    a.blk_c = (mode == MODE_BLOCK) ? blk_c : 0;
    a.W = W; a.Hinv = Hinv; a.R = R; a.d = d; a.k_steps = k_steps; a.nm_n = nm_n; a.nm_m = nm_m;
    a.stop_counts = stop_counts; a.delta = delta; a.offset = offset; a.maxq = maxq; a.live_in = live;
    a.order = order; a.loss = loss; a.codes = codes; a.W_out = W_out; a.trace = trace;
    a.out_ld = out_ld; a.status = ctx->d_status;

    const bool resident = rank1_lds_resident(d, nm_m);
    size_t lds = rank1_vec_lds(d, nm_m);
    if (resident) {
        a.Aws = nullptr;
        lds += (size_t)d * d * 4;
    } else {
        size_t need = obc_align_up((size_t)R * d * d * sizeof(float), 256);
        if (!ws || ws_bytes < need)
            return obc_fail(ctx, OBC_ERR_WORKSPACE, "row solver: workspace of %zu bytes needed, %zu given", need, ws_bytes);
        a.Aws = (float *)ws;
    }
    if (lds > LDS_LIMIT)
        return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "row solver (rank-1): d = %d needs %zu bytes of LDS", d, lds);
    const int threads = d <= 64 ? 256 : (d <= 192 ? 512 : 1024);
    if (R == 0) return OBC_OK;
    // live-set model of Algorithm 1: step t reads and writes the (d - t)^2 live entries
    double mm = 0.0;
    const int singles = (mode == MODE_BLOCK) ? k_steps * a.blk_c : k_steps;
    for (int t = 0; t < singles; ++t) mm += (double)(d - t) * (double)(d - t);
    obc_scope sc(ctx, OBC_KERNEL_RANK1, resident ? 0.0 : (double)R * 8.0 * mm, (double)R * 2.0 * mm);
    if (mode == MODE_PRUNE) {
        OBC_HIP(ctx, hipFuncSetAttribute((const void *)rows_rank1_kernel<MODE_PRUNE, 1>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        rows_rank1_kernel<MODE_PRUNE, 1><<<R, threads, lds, ctx->stream>>>(a);
    } else if (mode == MODE_QUANT) {
        OBC_HIP(ctx, hipFuncSetAttribute((const void *)rows_rank1_kernel<MODE_QUANT, 1>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        rows_rank1_kernel<MODE_QUANT, 1><<<R, threads, lds, ctx->stream>>>(a);
    } else if (a.blk_c <= 4) {
        OBC_HIP(ctx, hipFuncSetAttribute((const void *)rows_rank1_kernel<MODE_BLOCK, 4>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        rows_rank1_kernel<MODE_BLOCK, 4><<<R, threads, lds, ctx->stream>>>(a);
    } else {
        OBC_HIP(ctx, hipFuncSetAttribute((const void *)rows_rank1_kernel<MODE_BLOCK, 8>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        rows_rank1_kernel<MODE_BLOCK, 8><<<R, threads, lds, ctx->stream>>>(a);
    }
    OBC_LAUNCH_CHECK(ctx, "rows_rank1_kernel");
    return OBC_OK;
}

}  // namespace obc_rows
