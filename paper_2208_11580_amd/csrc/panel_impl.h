// The panel kernel of the blocked row solver (see rows_blocked.hip for the scheme).  Included by
// one small translation unit per (threads, elements per thread, block size) variant.
#pragma once

#include "rows_blocked.h"

namespace obc_blocked {

// Per-thread state of the panel: everything indexed by the owned element e (compact index
// tid + e*T) or by the step r inside the block.  All indices are compile-time constants once the
// step loop is unrolled (panel_steps below), so the arrays live in registers.
template <int EPT, int B>
struct PanelRegs {
    double w[EPT], dg[EPT];
    int og[EPT];
    bool alive[EPT];
    float u[B][EPT];
};

struct PanelShared {
    double red_s[2][16];
    int red_j[2][16];
    float cvec[BMAX];
    float invd_s[BMAX];
    int pivs[BMAX];
    double bc_wp, bc_app;
    int bc_o;
};

struct PanelRow {
    const float *Acur;
    float *gU;
    int ld, d, m, done, total, ndead, row;
    double qd, qo, qmax;
};

// One greedy step, S-th of the block.  Returns 0 to continue, 1 when the row has no step left,
// 2 on a numeric failure.  Every thread of the workgroup returns the same value.
template <int MODE, int T, int EPT, int B, int S>
__device__ __forceinline__ int panel_step(const PanelArgs &a, const PanelRow &pr, PanelRegs<EPT, B> &st,
                                          PanelShared &sh, uint8_t *blk)
{
    constexpr int NW = T / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (pr.done + S >= pr.total) return 1;

    // ---- (1) selection: fp64 score of every owned live index, workgroup argmin
    double bs = __builtin_inf();
    int bj = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        if (!st.alive[e]) continue;
        double sc;
        if (st.og[e] < 0) {
            sc = -1.0;
        } else {
            if (a.nm_m > 0 && blk[st.og[e] / a.nm_m] >= a.nm_m - a.nm_n) continue;
            double tq = 0.0;
            if (MODE == MODE_QUANT) {
                double c = rint((st.w[e] - pr.qo) / pr.qd);
                c = fmin(fmax(c, 0.0), pr.qmax);
                tq = pr.qo + pr.qd * c;
            }
            double er = tq - st.w[e];
            sc = er * er / st.dg[e];
        }
        if (sc < bs) { bs = sc; bj = tid + e * T; }   // own indices ascend: strict '<' keeps the lowest
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        double os = __shfl_xor(bs, off, 64);
        int oj = __shfl_xor(bj, off, 64);
        if (os < bs || (os == bs && oj < bj)) { bs = os; bj = oj; }
    }
    if (lane == 0) { sh.red_s[S & 1][wave] = bs; sh.red_j[S & 1][wave] = bj; }
    __syncthreads();
    bs = sh.red_s[S & 1][0];
    bj = sh.red_j[S & 1][0];
#pragma unroll
    for (int wv = 1; wv < NW; ++wv) {
        double os = sh.red_s[S & 1][wv];
        int oj = sh.red_j[S & 1][wv];
        if (os < bs || (os == bs && oj < bj)) { bs = os; bj = oj; }
    }
    const int p = bj;
    if (p == 0x7fffffff) return 2;

    // ---- (2) fetch the owned part of A0[p,:]; the owner of p publishes what everyone needs
    float col[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        int j = tid + e * T;
        col[e] = (j < pr.m) ? pr.Acur[(size_t)p * pr.ld + j] : 0.f;
    }
    const bool owner = (tid == p % T);
    if (owner) {
        const int ep = p / T;
        double wp = 0.0, ap = 1.0;
        int op = 0;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (e == ep) { wp = st.w[e]; ap = st.dg[e]; op = st.og[e]; }
        sh.bc_wp = wp;
        sh.bc_app = ap;
        sh.bc_o = op;
        sh.pivs[S] = p;
#pragma unroll
        for (int r = 0; r < S; ++r) {
            float ur = 0.f;
#pragma unroll
            for (int e = 0; e < EPT; ++e)
                if (e == ep) ur = st.u[r][e];
            sh.cvec[r] = __fmul_rn(ur, sh.invd_s[r]);
        }
        if (a.nm_m > 0 && op >= 0) blk[op / a.nm_m] += 1;
    }
    __syncthreads();
    const double app = sh.bc_app, wp = sh.bc_wp;
    const int op = sh.bc_o;
    if (!(app > 0.0) || !(app < __builtin_inf())) return 2;

    // ---- (3) target, compensation factor
    const bool isdead = op < 0;
    double target = 0.0, code = 0.0;
    if (isdead) target = wp;
    else if (MODE == MODE_QUANT) {
        code = rint((wp - pr.qo) / pr.qd);
        code = fmin(fmax(code, 0.0), pr.qmax);
        target = pr.qo + pr.qd * code;
    }
    const double g = (wp - target) / app;
    const double invapp = 1.0 / app;

    // ---- (4) bring the fetched row up to date, keep it, update w and the diagonal
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        float c = col[e];
#pragma unroll
        for (int r = 0; r < S; ++r) c = fmaf(-sh.cvec[r], st.u[r][e], c);
        st.u[S][e] = c;
        int j = tid + e * T;
        if (st.alive[e]) {
            if (j == p) {
                st.alive[e] = false;
            } else {
                double cd = (double)c;
                st.w[e] -= cd * g;
                st.dg[e] -= cd * cd * invapp;
            }
        }
    }
    if (owner) {
        sh.invd_s[S] = (float)invapp;
        if (!isdead) {
            const int t = pr.done + S - pr.ndead;
            const double er = target - wp;
            a.order[(size_t)pr.row * a.out_ld + t] = op;
            a.loss[(size_t)pr.row * a.out_ld + t] = (float)(er * er / (2.0 * app));
            a.W_out[(size_t)pr.row * pr.d + op] = (float)target;
            if (MODE == MODE_QUANT) a.codes[(size_t)pr.row * pr.d + op] = (int)code;
        }
    }
    if (MODE == MODE_PRUNE && a.trace && !isdead) {
        float *tr = a.trace + ((size_t)pr.row * a.out_ld + (pr.done + S - pr.ndead)) * pr.d;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (st.alive[e] && st.og[e] >= 0) tr[st.og[e]] = (float)st.w[e];
    }
    return 0;
}

// Compile-time unrolled step loop; returns the number of steps done and sets *failed.
template <int MODE, int T, int EPT, int B, int S>
__device__ __forceinline__ int panel_steps(const PanelArgs &a, const PanelRow &pr, PanelRegs<EPT, B> &st,
                                           PanelShared &sh, uint8_t *blk, bool *failed)
{
    if constexpr (S < B) {
        int rc = panel_step<MODE, T, EPT, B, S>(a, pr, st, sh, blk);
        if (rc != 0) {
            *failed = (rc == 2);
            return S;
        }
        return panel_steps<MODE, T, EPT, B, S + 1>(a, pr, st, sh, blk, failed);
    } else {
        return B;
    }
}

template <int MODE, int T, int EPT, int B>
__global__ __launch_bounds__(T) void panel_kernel(PanelArgs a)
{
    __shared__ PanelShared sh;
    extern __shared__ uint8_t blk[];   // N:M counters (d / M bytes), only when nm_m > 0

    const int row = blockIdx.x, tid = threadIdx.x;
    PanelRow pr;
    pr.row = row;
    pr.d = a.d;
    pr.m = a.ws.m[row];
    pr.done = a.ws.done[row];
    pr.total = a.ws.total[row];
    pr.ndead = a.ws.ndead[row];
    if (pr.done >= pr.total) {
        if (tid == 0) a.ws.nb[row] = 0;
        return;
    }
    const int d = a.d, m = pr.m;
    pr.Acur = a.A_cur + (size_t)row * a.a_row_stride;
    pr.ld = a.ld;
    pr.gU = a.ws.U + (size_t)row * BMAX * d;
    double *gw = a.ws.w + (size_t)row * d;
    double *gd = a.ws.diag + (size_t)row * d;
    int *go = a.ws.orig + (size_t)row * d;

    PanelRegs<EPT, B> st;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        int j = tid + e * T;
        st.alive[e] = j < m;
        st.w[e] = st.alive[e] ? gw[j] : 0.0;
        st.dg[e] = st.alive[e] ? gd[j] : 1.0;
        st.og[e] = st.alive[e] ? go[j] : 0;
    }
    const int nmb = a.nm_m > 0 ? d / a.nm_m : 0;
    for (int b = tid; b < nmb; b += T) blk[b] = a.ws.blk[(size_t)row * d + b];
    pr.qd = 1.0;
    pr.qo = 0.0;
    pr.qmax = (double)a.maxq;
    if (MODE == MODE_QUANT) { pr.qd = (double)a.delta[row]; pr.qo = (double)a.offset[row]; }
    __syncthreads();

    bool failed = false;
    const int nbv = panel_steps<MODE, T, EPT, B, 0>(a, pr, st, sh, blk, &failed);
    __syncthreads();

    // ---- block epilogue: drop this block's pivots from the compact index space
    for (int r = tid; r < nbv; r += T) {
        a.ws.invd[(size_t)row * BMAX + r] = sh.invd_s[r];
        a.ws.piv[(size_t)row * BMAX + r] = sh.pivs[r];
    }
    int *gmap = a.ws.map + (size_t)row * d;
    float *Wo = a.W_out + (size_t)row * d;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        int j = tid + e * T;
        if (j < m && st.alive[e]) {
            int below = 0;
            for (int r = 0; r < nbv; ++r) below += (sh.pivs[r] < j) ? 1 : 0;
            int jn = j - below;
            gw[jn] = st.w[e];
            gd[jn] = st.dg[e];
            go[jn] = st.og[e];
            gmap[jn] = j;
            if (st.og[e] >= 0) Wo[st.og[e]] = (float)st.w[e];
            // this block's vectors u_r, already in the new compact order, for the flush
#pragma unroll
            for (int r = 0; r < B; ++r)
                if (r < nbv) pr.gU[(size_t)r * d + jn] = st.u[r][e];
        }
    }
    for (int b = tid; b < nmb; b += T) a.ws.blk[(size_t)row * d + b] = blk[b];
    if (tid == 0) {
        a.ws.m[row] = m - nbv;
        a.ws.done[row] = pr.done + nbv;
        a.ws.nb[row] = nbv;
        if (failed) {
            a.ws.total[row] = pr.done + nbv;   // the row stops here
            obc_latch(a.status, OBC_ERR_NUMERIC);
        }
    }
}


#define OBC_DEFINE_PANEL(T, EPT, B)                                                                 \
    void launch_panel_##T##_##EPT##_##B(int mode, int R, size_t lds, hipStream_t st,                \
                                        const PanelArgs &a)                                         \
    {                                                                                               \
        if (mode == MODE_PRUNE)                                                                     \
            hipLaunchKernelGGL((panel_kernel<MODE_PRUNE, T, EPT, B>), dim3(R), dim3(T), lds, st, a); \
        else                                                                                        \
            hipLaunchKernelGGL((panel_kernel<MODE_QUANT, T, EPT, B>), dim3(R), dim3(T), lds, st, a); \
    }

}  // namespace obc_blocked
