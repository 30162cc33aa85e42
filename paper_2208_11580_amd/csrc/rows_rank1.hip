// Row solver, rank-1 strategy: Algorithm 1 (pruning, with the N:M rule) and Algorithm 3 (OBQ)
// of arxiv 2208.11580 exactly as written -- one Lemma-1 elimination per greedy step.
//
// One workgroup owns one row of W and a private copy A of H^-1.  A lives in LDS when it fits
// (d <= 192: the whole loop then never touches HBM) and otherwise in the caller's workspace,
// where every step streams the live rows of A through the CU with float4 accesses.
//
// Per step: (1) argmin of the score over the live, eligible indices (per-thread scan, wave
// shuffle reduction, cross-wave LDS reduction; ties to the lowest index); (2) row p of A -- equal
// to column p, A stays symmetric -- is staged in LDS; (3) w and the maintained diagonal are
// updated; (4) A[i,:] -= (A[i,p] / A_pp) A[p,:] for the live rows i.  Eliminated rows are never
// read or written again; eliminated columns of live rows are updated but never read.
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
    int32_t *order;
    float *loss;
    int32_t *codes;
    float *W_out;
    float *trace;
    int out_ld;              // leading dimension of order / loss / trace steps
    int *status;
};

template <int MODE>
__global__ __launch_bounds__(1024) void rows_rank1_kernel(Rank1Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int d = a.d;
    const int row = blockIdx.x;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthr >> 6;
    const int dpad = (d + 3) & ~3;

    float *w = reinterpret_cast<float *>(smem);
    float *diag = w + dpad;
    float *colp = diag + dpad;
    float *fcol = colp + dpad;
    int *lidx = reinterpret_cast<int *>(fcol + dpad);   // compact list of live indices
    int *pos = lidx + dpad;                             // position of index j in lidx
    int *dead = pos + dpad;                             // indices removed up front (quant on survivors)
    float *red_s = reinterpret_cast<float *>(dead + dpad);
    int *red_j = reinterpret_cast<int *>(red_s + 32);
    int *misc = red_j + 32;                             // [0] live count, [1] dead count
    uint8_t *blk = reinterpret_cast<uint8_t *>(misc + 8);  // pruned weights per N:M block
    float *A = a.Aws ? a.Aws + (size_t)row * d * d
                     : reinterpret_cast<float *>(smem + obc_align_up(
                           (size_t)dpad * 7 * 4 + 72 * 4 + (a.nm_m > 0 ? (size_t)dpad : 0), 16));

    // ---- set-up: private copy of H^-1, the row, the diagonal, the live list
    const float *Hinv = a.Hinv;
    for (size_t e = tid; e < (size_t)d * d; e += nthr) A[e] = Hinv[e];
    for (int j = tid; j < d; j += nthr) {
        bool alive = (MODE == MODE_QUANT && a.live_in) ? (a.live_in[(size_t)row * d + j] != 0) : true;
        w[j] = alive ? a.W[(size_t)row * d + j] : 0.f;
        diag[j] = Hinv[(size_t)j * d + j];
        pos[j] = alive ? 0 : -1;
        if (MODE == MODE_QUANT) a.codes[(size_t)row * d + j] = -1;
    }
    if (a.nm_m > 0)
        for (int b = tid; b < d / a.nm_m; b += nthr) blk[b] = 0;
    __syncthreads();
    if (tid == 0) {
        int m = 0, nd = 0;
        for (int j = 0; j < d; ++j) {
            if (pos[j] == 0) { lidx[m] = j; pos[j] = m; ++m; }
            else dead[nd++] = j;
        }
        misc[0] = m;
        misc[1] = nd;
    }
    __syncthreads();
    const int n_dead = misc[1];
    int m = misc[0];   // live count, tracked in a register by every thread

    int steps = a.k_steps;
    if (MODE == MODE_QUANT) steps = m;
    if (a.stop_counts) {
        int sc = a.stop_counts[row];
        sc = sc < 0 ? 0 : sc;
        steps = sc < steps ? sc : steps;
    }
    float qd = 1.f, qo = 0.f;
    const float qmax = (float)a.maxq;
    if (MODE == MODE_QUANT) { qd = a.delta[row]; qo = a.offset[row]; }

    const bool vec4 = (d % 4 == 0);
    bool failed = false;

    // dead indices are eliminated first, in ascending order, with no weight change; they are
    // kept on a separate list, so the live list only ever holds survivors
    for (int t = -n_dead; t < steps; ++t) {
        int p;
        float target = 0.f, wp = 0.f, app;
        if (t < 0) {
            p = dead[t + n_dead];
            app = diag[p];
        } else {
            // ---- (1) selection
            Cand c;
            c.s = __builtin_inff();
            c.j = 0x7fffffff;
            for (int q = tid; q < m; q += nthr) {
                int j = lidx[q];
                if (a.nm_m > 0 && blk[j / a.nm_m] >= a.nm_m - a.nm_n) continue;
                float wj = w[j];
                float tj = (MODE == MODE_QUANT) ? dequant(quant_code(wj, qd, qo, qmax), qd, qo) : 0.f;
                float s = score_of(wj, tj, diag[j]);
                if (cand_less(s, j, c.s, c.j)) { c.s = s; c.j = j; }
            }
            c = block_argmin(c, red_s, red_j);
            p = c.j;
            if (p == 0x7fffffff) { failed = true; break; }
            app = diag[p];
            wp = w[p];
            float code = 0.f;
            if (MODE == MODE_QUANT) {
                code = quant_code(wp, qd, qo, qmax);
                target = dequant(code, qd, qo);
            }
            if (tid == 0) {
                float e = __fsub_rn(target, wp);
                a.order[(size_t)row * a.out_ld + t] = p;
                a.loss[(size_t)row * a.out_ld + t] = __fdiv_rn(__fmul_rn(e, e), __fmul_rn(2.f, app));
                if (MODE == MODE_QUANT) a.codes[(size_t)row * d + p] = (int)code;
            }
        }
        if (!(app > 0.f) || !(app < __builtin_inff())) { failed = true; break; }

        // ---- (2) row p of A (= column p), and the multipliers A[i,p] / A_pp
        const float *Ap = A + (size_t)p * d;
        for (int j = tid; j < d; j += nthr) {
            float v = Ap[j];
            colp[j] = v;
            fcol[j] = __fdiv_rn(v, app);
        }
        __syncthreads();

        // During the up-front phase the not-yet-eliminated dead indices still belong to the
        // matrix being reduced: their rows and diagonal entries are updated like live ones.
        const int dnext = t + n_dead + 1;
        const int rem = (t < 0) ? n_dead - dnext : 0;
        const int mtot = m + rem;

        // ---- (3) compensation of the live weights, maintained diagonal
        const float g = __fdiv_rn(__fsub_rn(wp, target), app);
        for (int q = tid; q < mtot; q += nthr) {
            int j = (q < m) ? lidx[q] : dead[dnext + q - m];
            if (j == p) continue;
            if (q < m) w[j] = fmaf(-colp[j], g, w[j]);
            diag[j] = fmaf(-fcol[j], colp[j], diag[j]);
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
                lidx[qp] = last;
                pos[last] = qp;
                pos[p] = -1;
                if (a.nm_m > 0) blk[p / a.nm_m] += 1;
            }
            m -= 1;
        }
        __syncthreads();
        if (t >= 0 && a.trace) {
            float *tr = a.trace + ((size_t)row * a.out_ld + t) * d;
            for (int j = tid; j < d; j += nthr) tr[j] = w[j];
        }
    }

    if (failed && tid == 0) obc_latch(a.status, OBC_ERR_NUMERIC);
    __syncthreads();
    for (int j = tid; j < d; j += nthr) a.W_out[(size_t)row * d + j] = w[j];
}

inline size_t rank1_vec_lds(int d, int nm_m)
{
    size_t dpad = (size_t)((d + 3) & ~3);
    return obc_align_up(dpad * 7 * 4 + 72 * 4 + (nm_m > 0 ? dpad : 0), 16);
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
                 int nm_n, int nm_m, const int32_t *stop_counts, const float *delta,
                 const float *offset, int maxq, const uint8_t *live, int32_t *order, float *loss,
                 int32_t *codes, float *W_out, float *trace, int out_ld, void *ws, size_t ws_bytes)
{
    Rank1Args a;
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
    for (int t = 0; t < k_steps; ++t) mm += (double)(d - t) * (double)(d - t);
    obc_scope sc(ctx, OBC_KERNEL_RANK1, resident ? 0.0 : (double)R * 8.0 * mm, (double)R * 2.0 * mm);
    if (mode == MODE_PRUNE) {
        OBC_HIP(ctx, hipFuncSetAttribute((const void *)rows_rank1_kernel<MODE_PRUNE>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        rows_rank1_kernel<MODE_PRUNE><<<R, threads, lds, ctx->stream>>>(a);
    } else {
        OBC_HIP(ctx, hipFuncSetAttribute((const void *)rows_rank1_kernel<MODE_QUANT>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        rows_rank1_kernel<MODE_QUANT><<<R, threads, lds, ctx->stream>>>(a);
    }
    OBC_LAUNCH_CHECK(ctx, "rows_rank1_kernel");
    return OBC_OK;
}

}  // namespace obc_rows
