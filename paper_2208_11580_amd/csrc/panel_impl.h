// The panel kernel of the blocked row solver (see rows_blocked.hip for the scheme).  Included by
// one small translation unit per (threads, elements per thread, block size) variant.
#pragma once

#include <atomic>

#include "rows_blocked.h"

namespace obc_blocked {

// Per-thread state of the panel: everything indexed by the owned element e (compact index
// tid + e*T) or by the step r inside the block.  All indices are compile-time constants once the
// step loop is unrolled (panel_steps below), so the arrays live in registers.
template <int EPT, int BR>
struct PanelRegs {
    double w[EPT], dg[EPT];
    int og[EPT];
    bool alive[EPT];
    float u[BR][EPT];   // u_r for the first BR steps of the block; later ones live in LDS
    // block pruning only: row j of the 4 x 4 diagonal block of the current inverse that element j
    // belongs to (entry k = A[j][4 (j / 4) + k]; the element's own slot is not used), and the first
    // position of the block being eliminated
    float ob[EPT][4];
    int p0;
};

struct PanelShared {
    unsigned long long red_k[2][16];
    __attribute__((aligned(16))) float cvec[BMAX];
    float invd_s[BMAX];
    int pivs[BMAX];
    double bc_g, bc_invapp;
    int bc_o, bc_ok;
    float bc_loss, bc_target;   // the step's records, written out after the barrier
    int bc_code;
    double blk_loss;   // block pruning: loss of the block being eliminated, summed over its weights
};

// order-preserving map of a float onto unsigned integers
__device__ __forceinline__ unsigned score_bits(float f)
{
    unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// value of lane K of the caller's group of four lanes (DPP quad_perm broadcast); must be called
// with all four lanes active
template <int K>
__device__ __forceinline__ float quad_bcast(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), K * 0x55, 0xf, 0xf, false));
}
template <int K>
__device__ __forceinline__ double quad_bcast(double v)
{
    long long b = __double_as_longlong(v);
    unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)b, K * 0x55, 0xf, 0xf, false);
    unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(b >> 32), K * 0x55, 0xf, 0xf, false);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Block pruning (Sec. 4 "Block-Sparsity", eq. (5)), blocks of 4: the score w_P^T ((H^-1)_P)^-1 w_P of
// the block that the calling lane's element belongs to.  The block's four elements sit on four
// neighbouring lanes (positions 4b .. 4b+3 of the compact index space); every lane gathers the
// block's weights and its 4 x 4 piece of the inverse and runs the same elimination, so the four
// lanes get bit-identical scores.  NaN when a pivot is not positive.
__device__ __forceinline__ double quad_block_score(double w, double dg, const float (&ob)[4])
{
    double v[4], M[4][4];
    v[0] = quad_bcast<0>(w); v[1] = quad_bcast<1>(w); v[2] = quad_bcast<2>(w); v[3] = quad_bcast<3>(w);
    M[0][0] = quad_bcast<0>(dg); M[1][1] = quad_bcast<1>(dg);
    M[2][2] = quad_bcast<2>(dg); M[3][3] = quad_bcast<3>(dg);
    M[1][0] = (double)quad_bcast<1>(ob[0]);
    M[2][0] = (double)quad_bcast<2>(ob[0]); M[2][1] = (double)quad_bcast<2>(ob[1]);
    M[3][0] = (double)quad_bcast<3>(ob[0]); M[3][1] = (double)quad_bcast<3>(ob[1]);
    M[3][2] = (double)quad_bcast<3>(ob[2]);
    double s = 0.0;
    bool bad = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const double piv = M[k][k];
        bad = bad || !(piv > 0.0);
        const double ip = 1.0 / piv;
        s += v[k] * v[k] * ip;
#pragma unroll
        for (int i = k + 1; i < 4; ++i) {
            const double f = M[i][k] * ip;
            v[i] -= f * v[k];
#pragma unroll
            for (int j = k + 1; j <= i; ++j) M[i][j] -= f * M[j][k];
        }
    }
    return bad ? __builtin_nan("") : s;
}

// One DPP stage of an unsigned minimum: combine with the lane `row_shr` positions down the
// 16-lane row (lanes shifted in from outside the row contribute the identity).
template <int CTRL>
__device__ __forceinline__ unsigned dpp_umin_stage(unsigned v)
{
    const unsigned o = (unsigned)__builtin_amdgcn_update_dpp(-1, (int)v, CTRL, 0xf, 0xf, false);
    return o < v ? o : v;
}

// minimum over each 16-lane row, valid in the row's last lane
__device__ __forceinline__ unsigned row16_umin(unsigned v)
{
    v = dpp_umin_stage<0x111>(v);   // row_shr:1
    v = dpp_umin_stage<0x112>(v);   // row_shr:2
    v = dpp_umin_stage<0x114>(v);   // row_shr:4
    v = dpp_umin_stage<0x118>(v);   // row_shr:8
    return v;
}

// minimum over the wavefront (uniform result)
__device__ __forceinline__ unsigned wave_umin(unsigned v)
{
    v = row16_umin(v);
    unsigned a0 = (unsigned)__builtin_amdgcn_readlane((int)v, 15), a1 = (unsigned)__builtin_amdgcn_readlane((int)v, 31);
    unsigned a2 = (unsigned)__builtin_amdgcn_readlane((int)v, 47), a3 = (unsigned)__builtin_amdgcn_readlane((int)v, 63);
    a0 = a1 < a0 ? a1 : a0;
    a2 = a3 < a2 ? a3 : a2;
    return a2 < a0 ? a2 : a0;
}

// minimum over the first 16 lanes' values (every row holds the same 16 values; uniform result)
__device__ __forceinline__ unsigned row16_umin_all(unsigned v)
{
    return (unsigned)__builtin_amdgcn_readlane((int)row16_umin(v), 15);
}

struct PanelRow {
    const float *Acur;
    float *gU;
    int ld, swz, d, m, done, total, ndead, row;
    double qd, qo, qmax, iqd;
};

// One greedy step, S-th of the block.  Returns 0 to continue, 1 when the row has no step left,
// 2 on a numeric failure.  Every thread of the workgroup returns the same value.
template <int MODE, int T, int EPT, int BR, int BL, int S>
__device__ __forceinline__ int panel_step(const PanelArgs &a, const PanelRow &pr, PanelRegs<EPT, BR> &st,
                                          PanelShared &sh, uint8_t *blk, float *ul)
{
    // u_r[j] for r >= BR is kept at ul[(r - BR) * (T * EPT) + j]; only the owner of j touches it
    constexpr int CAP = T * EPT;
    constexpr int NW = T / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (pr.done + S >= pr.total) return 1;

    // ---- (1) selection.  The error (target - w) is formed in fp64 (for OBQ it is a difference of
    // nearby numbers); the score itself, error^2 / a_jj, is only compared, so it is taken in fp32
    // with the hardware reciprocal (2 ulp): candidates closer than that count as tied.
    // A candidate is the pair (order-preserving bits of the score, index); the argmin with ties to
    // the lowest index is taken in two unsigned 32-bit minima: the least score, then the least
    // index among the candidates that have it.  All ones = no candidate.
    unsigned cs = ~0u, ci = ~0u;
    if constexpr (MODE == MODE_BLOCK) {
        // a block is chosen every fourth step; the three steps after it take its other weights
        if constexpr (S % 4 == 0) {
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const float sc = (float)quad_block_score(st.w[e], st.dg[e], st.ob[e]);
                if (st.alive[e] && sc == sc) {
                    const unsigned b = score_bits(sc);
                    if (b < cs) { cs = b; ci = (unsigned)((tid & ~3) + e * T); }   // (indices ascend with e)
                }
            }
        }
    } else {
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        if (!st.alive[e]) continue;
        float sc;
        if (st.og[e] < 0) {
            sc = -__builtin_inff();   // dead indices go first, before any outlier
        } else {
            if (a.nm_m > 0 && blk[st.og[e] / a.nm_m] >= a.nm_m - a.nm_n) continue;
            double tq = 0.0;
            if (MODE == MODE_QUANT) {
                double c = rint((st.w[e] - pr.qo) * pr.iqd);
                c = fmin(fmax(c, 0.0), pr.qmax);
                tq = pr.qo + pr.qd * c;
            }
            double er = tq - st.w[e];
            sc = (float)(er * er) * __builtin_amdgcn_rcpf((float)st.dg[e]);
            // outlier heuristic: a weight whose error exceeds half a grid step sorts before every
            // non-outlier
            if (MODE == MODE_QUANT && a.outliers && fabs(er) > 0.5 * pr.qd) sc = outlier_first(sc);
        }
        if (sc == sc) {   // a NaN score is no candidate
            const unsigned b = score_bits(sc);
            if (b < cs) { cs = b; ci = (unsigned)(tid + e * T); }   // (indices ascend with e)
        }
    }
    }
    int p;
    if constexpr (MODE == MODE_BLOCK && S % 4 != 0) {
        __syncthreads();   // the previous step's readers of the shared step data are done
        p = st.p0 + S % 4;
    } else {
        {
            const unsigned ws = wave_umin(cs);
            const unsigned wi = wave_umin(cs == ws ? ci : ~0u);
            if (lane == 0) sh.red_k[S & 1][wave] = ((unsigned long long)ws << 32) | wi;
        }
        __syncthreads();
        const unsigned long long wk = (lane & 15) < NW ? sh.red_k[S & 1][lane & 15] : ~0ull;
        const unsigned gs = row16_umin_all((unsigned)(wk >> 32));
        if (gs == ~0u) return 2;
        p = (int)row16_umin_all((unsigned)(wk >> 32) == gs ? (unsigned)wk : ~0u);
        if constexpr (MODE == MODE_BLOCK) st.p0 = p;
    }

    // ---- (2) fetch the owned part of row p of A0.  Only the lower triangle of A0 is kept up to
    // date (the matrix is symmetric): entry (p, j) is read as (max(p, j), min(p, j)), i.e. along
    // row p up to the diagonal and down column p below it.
    float col[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        int j = tid + e * T;
        const int hi = (j <= p) ? p : j, lo = (j <= p) ? j : p;
        // (a row's matrix has at most 4608^2 entries: 32-bit index arithmetic)
        const unsigned off = pr.swz ? (((unsigned)(hi >> 2) * (unsigned)pr.ld + (unsigned)lo) << 2) + (unsigned)(hi & 3)
                                    : (unsigned)hi * (unsigned)pr.ld + (unsigned)lo;
        col[e] = (j < pr.m) ? __builtin_nontemporal_load(&pr.Acur[off]) : 0.f;
    }
    // the owner of p publishes the pivot's data, the step's scalars and the coefficients
    // u_r[p] / a_r of the earlier steps of this block
    const bool owner = (tid == p % T);
    if (owner) {
        const int ep = p / T;
        double wp = 0.0, ap = 1.0, target = 0.0, code = 0.0;
        int op = 0;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (e == ep) { wp = st.w[e]; ap = st.dg[e]; op = st.og[e]; }
        if (op < 0) target = wp;
        else if (MODE == MODE_QUANT) {
            code = rint((wp - pr.qo) * pr.iqd);   // same expression as in the selection
            code = fmin(fmax(code, 0.0), pr.qmax);
            target = pr.qo + pr.qd * code;
        }
        const bool ok = (ap > 0.0) && (ap < __builtin_inf());
        const double invapp = 1.0 / ap;           // the step's only division
        const double er = target - wp;
        sh.bc_loss = (float)(0.5 * er * er * invapp);
        sh.bc_target = (float)target;
        sh.bc_code = (int)code;
        sh.bc_g = (wp - target) * invapp;
        sh.bc_invapp = invapp;
        sh.bc_o = op;
        sh.bc_ok = ok ? 1 : 0;
        sh.pivs[S] = p;
        sh.invd_s[S] = (float)invapp;
        // coefficients of the vectors kept in registers: only the owner has their entry p.  One
        // branch per owned element, then four coefficients per LDS read / write.
        constexpr int SREG = S < BR ? S : BR;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            if (e != ep) continue;
#pragma unroll
            for (int r4 = 0; r4 < SREG; r4 += 4) {
                const float4 iv = *reinterpret_cast<const float4 *>(&sh.invd_s[r4]);
                float4 v;
                v.x = __fmul_rn(st.u[r4][e], iv.x);
                v.y = (r4 + 1 < SREG) ? __fmul_rn(st.u[r4 + 1 < BR ? r4 + 1 : 0][e], iv.y) : 0.f;
                v.z = (r4 + 2 < SREG) ? __fmul_rn(st.u[r4 + 2 < BR ? r4 + 2 : 0][e], iv.z) : 0.f;
                v.w = (r4 + 3 < SREG) ? __fmul_rn(st.u[r4 + 3 < BR ? r4 + 3 : 0][e], iv.w) : 0.f;
                *reinterpret_cast<float4 *>(&sh.cvec[r4]) = v;
            }
        }
        if (a.nm_m > 0 && op >= 0) blk[op / a.nm_m] += 1;
    }
    // coefficients of the vectors kept in LDS: one lane each
    if constexpr (S > BR) {
        const int r = BR + tid;
        if (r < S) sh.cvec[r] = __fmul_rn(ul[(r - BR) * CAP + p], sh.invd_s[r]);
    }
    __syncthreads();
    if (!sh.bc_ok) return 2;
    // the step's records are written here, while everybody waits for the fetched row anyway
    if (owner) {
        const int op = sh.bc_o;
        if (MODE == MODE_BLOCK) {
            // the block's loss is the sum of its four single losses (owners of consecutive steps
            // are separated by the step's barriers)
            const double acc = (S % 4 == 0) ? (double)sh.bc_loss : sh.blk_loss + (double)sh.bc_loss;
            sh.blk_loss = acc;
            a.W_out[(size_t)pr.row * pr.d + op] = 0.f;
            if (S % 4 == 3) {
                const int t = (pr.done + S) / 4;
                a.order[(size_t)pr.row * a.out_ld + t] = op / 4;
                a.loss[(size_t)pr.row * a.out_ld + t] = (float)acc;
            }
        } else if (op >= 0) {
            const int t = pr.done + S - pr.ndead;
            a.order[(size_t)pr.row * a.out_ld + t] = op;
            a.loss[(size_t)pr.row * a.out_ld + t] = sh.bc_loss;
            a.W_out[(size_t)pr.row * pr.d + op] = sh.bc_target;
            if (MODE == MODE_QUANT) a.codes[(size_t)pr.row * pr.d + op] = sh.bc_code;
        }
    }
    const double g = sh.bc_g, invapp = sh.bc_invapp;
    const bool isdead = sh.bc_o < 0;
    // coefficients of this step, once, into scalar registers (they are the same for every lane;
    // as vector registers they would take up to B of them next to the block vectors)
    float cv[S > 0 ? S : 1];
    auto uni = [](float x) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x))); };
#pragma unroll
    for (int r4 = 0; r4 < S; r4 += 4) {
        float4 c4 = *reinterpret_cast<const float4 *>(&sh.cvec[r4]);
        cv[r4] = uni(c4.x);
        if (r4 + 1 < S) cv[r4 + 1] = uni(c4.y);
        if (r4 + 2 < S) cv[r4 + 2] = uni(c4.z);
        if (r4 + 3 < S) cv[r4 + 3] = uni(c4.w);
    }

    // ---- (3) bring the fetched row up to date, keep it, update w and the diagonal
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        int j = tid + e * T;
        // the correction is summed on its own and subtracted once: its roundings are then relative
        // to the (small) correction instead of to the matrix entry, and the sum does not wait for
        // the fetched row
        float corr = 0.f;
#pragma unroll
        for (int r = 0; r < S; ++r) {
            float ur = (r < BR) ? st.u[r < BR ? r : 0][e] : ul[(r - BR) * CAP + j];
            corr = fmaf(cv[r], ur, corr);
        }
        float c = __fsub_rn(col[e], corr);
        if constexpr (S < BR) st.u[S < BR ? S : 0][e] = c;
        else ul[(S - BR) * CAP + j] = c;
        if constexpr (MODE == MODE_BLOCK) {
            // Lemma 1 on the element's row of its own 4 x 4 block: A[j][j'] -= u[j] u[j'] / a
            const float cs = c * (float)invapp;
            st.ob[e][0] = fmaf(-cs, quad_bcast<0>(c), st.ob[e][0]);
            st.ob[e][1] = fmaf(-cs, quad_bcast<1>(c), st.ob[e][1]);
            st.ob[e][2] = fmaf(-cs, quad_bcast<2>(c), st.ob[e][2]);
            st.ob[e][3] = fmaf(-cs, quad_bcast<3>(c), st.ob[e][3]);
        }
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
    if (MODE == MODE_BLOCK && a.trace && S % 4 == 3) {
        float *tr = a.trace + ((size_t)pr.row * a.out_ld + (pr.done + S) / 4) * pr.d;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (st.alive[e]) tr[st.og[e]] = (float)st.w[e];
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
template <int MODE, int T, int EPT, int BR, int BL, int S>
__device__ __forceinline__ int panel_steps(const PanelArgs &a, const PanelRow &pr, PanelRegs<EPT, BR> &st,
                                           PanelShared &sh, uint8_t *blk, float *ul, bool *failed)
{
    if constexpr (S < BR + BL) {
        int rc = panel_step<MODE, T, EPT, BR, BL, S>(a, pr, st, sh, blk, ul);
        if (rc != 0) {
            *failed = (rc == 2);
            return S;
        }
        return panel_steps<MODE, T, EPT, BR, BL, S + 1>(a, pr, st, sh, blk, ul, failed);
    } else {
        return BR + BL;
    }
}

template <int MODE, int T, int EPT, int BR, int BL>
__global__ __launch_bounds__(T) void panel_kernel(PanelArgs a)
{
    constexpr int B = BR + BL;
    __shared__ PanelShared sh;
    // dynamic LDS: BL vectors of T * EPT floats, then the N:M counters (d / M bytes) when nm_m > 0
    extern __shared__ __align__(16) uint8_t dyn_lds[];
    float *ul = reinterpret_cast<float *>(dyn_lds);
    uint8_t *blk = dyn_lds + (size_t)BL * T * EPT * sizeof(float);

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
    pr.swz = a.swz;
    pr.gU = a.ws.U + (size_t)row * BMAX * a.ws.ldu;
    double *gw = a.ws.w + (size_t)row * d;
    double *gd = a.ws.diag + (size_t)row * d;
    int *go = a.ws.orig + (size_t)row * d;

    PanelRegs<EPT, BR> st;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        int j = tid + e * T;
        st.alive[e] = j < m;
        st.w[e] = st.alive[e] ? gw[j] : 0.0;
        st.dg[e] = st.alive[e] ? gd[j] : 1.0;
        st.og[e] = st.alive[e] ? go[j] : 0;
    }
    if constexpr (MODE == MODE_BLOCK) {
        // the element's row of its 4 x 4 diagonal block, from the lower triangle of the matrix
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int j = tid + e * T, j0 = j & ~3;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int jj = j0 + k;
                const int hi = (jj <= j) ? j : jj, lo = (jj <= j) ? jj : j;
                const size_t off = pr.swz ? quad_index(hi, lo, pr.ld) : (size_t)hi * pr.ld + lo;
                st.ob[e][k] = (j < m) ? pr.Acur[off] : 0.f;
            }
        }
        st.p0 = 0;
    }
    const int nmb = a.nm_m > 0 ? d / a.nm_m : 0;
    for (int b = tid; b < nmb; b += T) blk[b] = a.ws.blk[(size_t)row * d + b];
    pr.qd = 1.0;
    pr.qo = 0.0;
    pr.qmax = (double)a.maxq;
    if (MODE == MODE_QUANT) { pr.qd = (double)a.delta[row]; pr.qo = (double)a.offset[row]; }
    pr.iqd = 1.0 / pr.qd;
    __syncthreads();

    bool failed = false;
    const int nbv = panel_steps<MODE, T, EPT, BR, BL, 0>(a, pr, st, sh, blk, ul, &failed);
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
                if (r < nbv)
                    pr.gU[(size_t)r * a.ws.ldu + jn] = (r < BR) ? st.u[r < BR ? r : 0][e] : ul[(r - BR) * (T * EPT) + j];
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


// A kernel's dynamic LDS limit is a per-device attribute: `done` remembers, one bit per device, where
// it has been raised for `fn`.  Safe from several host threads (raising it twice is harmless).
inline int panel_raise_lds_limit(const void *fn, std::atomic<unsigned long long> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return 0;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(160 * 1024 - 2048)) != hipSuccess)
        return -1;
    done.fetch_or(bit, std::memory_order_release);
    return 0;
}

#define OBC_DEFINE_PANEL(T, EPT, BR, BL)                                                            \
    int launch_panel_##T##_##EPT##_##BR##_##BL(int mode, int R, size_t lds_nm, hipStream_t st,      \
                                               const PanelArgs &a)                                  \
    {                                                                                               \
        const size_t lds = (size_t)(BL) * (T) * (EPT) * sizeof(float) + lds_nm;                     \
        auto kp = panel_kernel<MODE_PRUNE, T, EPT, BR, BL>;                                         \
        auto kq = panel_kernel<MODE_QUANT, T, EPT, BR, BL>;                                         \
        static std::atomic<unsigned long long> raised_p{0}, raised_q{0};                            \
        if (lds > 48 * 1024) {                                                                      \
            if (mode == MODE_PRUNE && panel_raise_lds_limit((const void *)kp, raised_p) != 0) return -1; \
            if (mode != MODE_PRUNE && panel_raise_lds_limit((const void *)kq, raised_q) != 0) return -1; \
        }                                                                                           \
        if (mode == MODE_PRUNE) hipLaunchKernelGGL(kp, dim3(R), dim3(T), lds, st, a);               \
        else hipLaunchKernelGGL(kq, dim3(R), dim3(T), lds, st, a);                                  \
        return 0;                                                                                   \
    }

// The block-pruning instance of a variant, in a translation unit of its own.
#define OBC_DEFINE_PANEL_BLOCK(T, EPT, BR, BL)                                                      \
    int launch_panel_block_##T##_##EPT##_##BR##_##BL(int, int R, size_t lds_nm, hipStream_t st,     \
                                                     const PanelArgs &a)                            \
    {                                                                                               \
        const size_t lds = (size_t)(BL) * (T) * (EPT) * sizeof(float) + lds_nm;                     \
        auto kb = panel_kernel<MODE_BLOCK, T, EPT, BR, BL>;                                         \
        static std::atomic<unsigned long long> raised{0};                                           \
        if (lds > 48 * 1024 && panel_raise_lds_limit((const void *)kb, raised) != 0) return -1;     \
        hipLaunchKernelGGL(kb, dim3(R), dim3(T), lds, st, a);                                       \
        return 0;                                                                                   \
    }

}  // namespace obc_blocked
