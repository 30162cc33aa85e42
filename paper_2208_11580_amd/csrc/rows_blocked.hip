// Row solver, blocked strategy: the greedy loops of Algorithm 1 / Algorithm 3 (arxiv 2208.11580)
// with the Lemma-1 eliminations applied to the row's private inverse in blocks of B steps.
//
// What a greedy step needs is small: the current diagonal of A, the current weights, and the
// current row p of A.  The first two are O(d) to maintain.  Row p can be formed on demand from
// the matrix as of the last block boundary, A0, and the eliminations done since:
//
//     A[p,:] = A0[p,:] - sum_r (u_r[p] / a_r) u_r        u_r = row p_r of A when p_r was chosen,
//                                                        a_r = its diagonal entry
//
// so inside a block nothing of size d^2 moves.  Every B steps the deferred eliminations are
// applied at once,  A0 <- A0 - U diag(1/a) U^T,  a dense rank-B contraction that runs on the fp32
// matrix cores and touches A once per B steps instead of once per step.  The result is the same
// sequence of exact OBS steps; only the order of fp32 roundings inside A differs from the
// rank-1 strategy.
//
// Two kernels alternate on the stream (host loop, no host synchronisation):
//
//   panel_kernel  one workgroup per row, B greedy steps.  Thread t owns the compact indices
//                 t, t+T, ...: their weights and diagonal (fp64) and the B vectors u_r live in its
//                 registers.  Per step: fp64 score + workgroup argmin (barrier 1), the owner of p
//                 publishes w_p, a_p and the coefficients u_r[p]/a_r while every thread fetches its
//                 part of A0[p,:] (barrier 2), then the row is corrected, w / diag are updated and
//                 u_s is kept (registers) and stored (HBM, for the flush).
//   flush_kernel  A0_new = compact(A0 - U diag(1/a) U^T): 128x128 tiles on v_mfma_f32_32x32x2_f32,
//                 one workgroup per strip of 128 or 256 rows of one row's matrix (only the lower
//                 triangle is kept).  The eliminated rows and columns are dropped while writing
//                 (out of place, two buffers), so the matrix shrinks with the live set and later
//                 blocks cost (m/d)^2 of the first.
//
// The first block reads the shared H^-1 directly, so no per-row copy of it is ever made.
// Already-pruned weights (quantization or pruning of survivors) are eliminated first, in index
// order, with no weight change and nothing recorded: 64 at a time by a block form of Lemma 1 as
// long as every row has that many left (see "bulk elimination" below), the rest as candidates
// with score -infinity inside the panel.
#include "rows_blocked.h"

namespace {

using namespace obc_blocked;

size_t carve(BlockedWs *ws, void *base, int R, int d)
{
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += obc_align_up(bytes, 256);
        return base ? (char *)base + o : (char *)nullptr;
    };
    size_t mat = (size_t)R * obc_align_up((size_t)d * d, 4) * sizeof(float);
    char *p0 = take(mat), *p1 = take(mat);
    const int ldu = (d + 3) & ~3;
    char *pu = take((size_t)R * BMAX * ldu * sizeof(float));
    char *pi = take((size_t)R * BMAX * sizeof(float));
    char *pp = take((size_t)R * BMAX * sizeof(int));
    char *pm = take((size_t)R * d * sizeof(int));
    char *pw = take((size_t)R * d * sizeof(double));
    char *pd = take((size_t)R * d * sizeof(double));
    char *po = take((size_t)R * d * sizeof(int));
    char *s0 = take((size_t)R * sizeof(int)), *s1 = take((size_t)R * sizeof(int));
    char *s2 = take((size_t)R * sizeof(int)), *s3 = take((size_t)R * sizeof(int));
    char *s4 = take((size_t)R * sizeof(int));
    char *pb = take((size_t)R * d);
    char *pg = take((size_t)R * BMAX * ldu * sizeof(float));
    char *pmb = take((size_t)R * BMAX * BMAX * sizeof(double));
    char *ptb = take((size_t)R * BMAX * BMAX * sizeof(double));
    char *psc = take(256);
    if (ws) {
        ws->G = (float *)pg; ws->Mb = (double *)pmb; ws->Tb = (double *)ptb; ws->scal = (int *)psc;
        ws->Abuf[0] = (float *)p0; ws->Abuf[1] = (float *)p1; ws->U = (float *)pu; ws->ldu = ldu;
        ws->invd = (float *)pi; ws->piv = (int *)pp; ws->map = (int *)pm; ws->w = (double *)pw;
        ws->diag = (double *)pd; ws->orig = (int *)po; ws->m = (int *)s0; ws->done = (int *)s1;
        ws->total = (int *)s2; ws->ndead = (int *)s3; ws->nb = (int *)s4; ws->blk = (uint8_t *)pb;
    }
    return off;
}

// ------------------------------------------------------------------------------------------ init
struct InitArgs {
    const float *W, *Hinv;
    const uint8_t *live_in;
    const int32_t *stop_counts;
    int d, k_steps, mode;
    BlockedWs ws;
    int32_t *codes;
    float *W_out;
};

__global__ __launch_bounds__(256) void blocked_init_kernel(InitArgs a)
{
    __shared__ int cnt;
    const int row = blockIdx.x, tid = threadIdx.x, d = a.d;
    if (tid == 0) cnt = 0;
    __syncthreads();
    int dead_local = 0;
    for (int j = tid; j < d; j += 256) {
        bool alive = (a.mode != MODE_BLOCK && a.live_in) ? a.live_in[(size_t)row * d + j] != 0 : true;
        a.ws.w[(size_t)row * d + j] = alive ? (double)a.W[(size_t)row * d + j] : 0.0;
        a.ws.diag[(size_t)row * d + j] = (double)a.Hinv[(size_t)j * d + j];
        a.ws.orig[(size_t)row * d + j] = alive ? j : ~j;
        a.ws.blk[(size_t)row * d + j] = 0;
        a.W_out[(size_t)row * d + j] = alive ? a.W[(size_t)row * d + j] : 0.f;   // rows that do no step keep W
        if (a.mode == MODE_QUANT) a.codes[(size_t)row * d + j] = -1;
        dead_local += alive ? 0 : 1;
    }
    atomicAdd(&cnt, dead_local);
    __syncthreads();
    if (tid == 0) {
        // steps on the survivors, in single eliminations (block pruning: 4 per block step); the
        // eliminations of the already-pruned indices come on top
        const int survivors = d - cnt;
        int steps = (a.mode == MODE_QUANT) ? survivors : (a.k_steps < survivors ? a.k_steps : survivors);
        if (a.stop_counts) {
            int sc = a.stop_counts[row];
            sc = sc < 0 ? 0 : sc;
            if (a.mode == MODE_BLOCK) sc = sc > d / 4 ? d : sc * 4;
            steps = sc < steps ? sc : steps;
        }
        const int total = cnt + steps;
        a.ws.m[row] = d;
        a.ws.done[row] = 0;
        a.ws.total[row] = total;
        a.ws.ndead[row] = cnt;
        a.ws.nb[row] = 0;
    }
}

// p[0 .. n) = v with 16-byte streaming stores; the floats before the first 16-byte boundary and
// after the last one singly (p is 4-byte aligned)
__global__ __launch_bounds__(256) void fill_f32_kernel(float *p, size_t n, float v)
{
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    size_t head = ((16 - ((uintptr_t)p & 15)) & 15) / 4;
    if (head > n) head = n;
    const floatx4 v4 = {v, v, v, v};
    floatx4 *p4 = reinterpret_cast<floatx4 *>(p + head);
    const size_t n4 = (n - head) / 4, tail = (n - head) % 4;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n4; e += (size_t)gridDim.x * 256)
        __builtin_nontemporal_store(v4, p4 + e);
    if (blockIdx.x == 0) {
        if (threadIdx.x < head) p[threadIdx.x] = v;
        if (threadIdx.x < tail) p[head + n4 * 4 + threadIdx.x] = v;
    }
}

// ------------------------------------------------------------ bulk elimination of pruned indices
// Already-pruned indices (quantization or pruning of the survivors of an earlier pass) leave the
// inverse without any choice to make: they go in index order and change no weight.  For a set P of
// BMAX of them the eliminations collapse into one block step (the block form of Lemma 1, as in
// eq. (5)):  A <- A - A[:,P] (A[P,P])^-1 A[P,:] = A - U U^T  with  U = A[:,P] L^-T,  A[P,P] = L L^T.
// That needs no vectors kept on chip, so the rank of the update is BMAX whatever the width of the
// row -- the greedy panel manages 24 at 4608 -- and the flush that follows moves that much less.
// Three kernels per block: gather A[:,P] and A[P,P]; factor A[P,P] and invert the factor (fp64,
// one wavefront per row); U = L^-1 A[P,:] with the diagonal update and the compaction.  Every row
// does the same number of such blocks (the smallest count of pruned indices over the rows decides);
// what is left goes through the panel as before.
struct DeadArgs {
    const float *A_cur;
    size_t a_row_stride;
    int ld, swz, d;
    BlockedWs ws;
};

// out[0] = smallest number of up-front eliminations over the rows, out[1] = largest number of
// eliminations (up-front + greedy) any row does
__global__ __launch_bounds__(256) void min_ndead_kernel(const int *__restrict__ ndead, const int *__restrict__ total,
                                                        int R, int *out)
{
    __shared__ int red[256], redt[256];
    int v = 0x7fffffff, t = 0;
    for (int i = threadIdx.x; i < R; i += 256) {
        v = ndead[i] < v ? ndead[i] : v;
        t = total[i] > t ? total[i] : t;
    }
    red[threadIdx.x] = v;
    redt[threadIdx.x] = t;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            red[threadIdx.x] = red[threadIdx.x + w] < red[threadIdx.x] ? red[threadIdx.x + w] : red[threadIdx.x];
            redt[threadIdx.x] = redt[threadIdx.x + w] > redt[threadIdx.x] ? redt[threadIdx.x + w] : redt[threadIdx.x];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { out[0] = red[0]; out[1] = redt[0]; }
}

// The block's pivots (the first BMAX pruned indices in compact order), the rows of the matrix at
// them (G, in the old compact order) and their principal submatrix (Mb, fp64).
__global__ __launch_bounds__(512) void dead_gather_kernel(DeadArgs a)
{
    __shared__ int pv[BMAX];
    __shared__ int wcnt[8];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = a.ws.m[row];
    const int *orig = a.ws.orig + (size_t)row * a.d;
    int found = 0;                                       // pivots found so far (uniform)
    for (int c0 = 0; c0 < m && found < BMAX; c0 += 512) {
        const int j = c0 + tid;
        const bool dead = j < m && orig[j] < 0;
        const unsigned long long bal = __ballot(dead);
        if (lane == 0) wcnt[wave] = __popcll(bal);
        __syncthreads();
        int before = found, total = 0;
        for (int w = 0; w < 8; ++w) {
            if (w < wave) before += wcnt[w];
            total += wcnt[w];
        }
        const int rank = before + __popcll(bal & ((1ull << lane) - 1ull));
        if (dead && rank < BMAX) pv[rank] = j;
        found += total;
        __syncthreads();
    }
    // (the host only launches this while every row still has BMAX pruned indices)
    const float *Acur = a.A_cur + (size_t)row * a.a_row_stride;
    float *G = a.ws.G + (size_t)row * BMAX * a.ws.ldu;
    for (int r = 0; r < BMAX; ++r) {
        const int p = pv[r];
        for (int j = tid; j < m; j += 512) {
            const int hi = (j <= p) ? p : j, lo = (j <= p) ? j : p;
            const size_t off = a.swz ? quad_index(hi, lo, a.ld) : (size_t)hi * a.ld + lo;
            G[(size_t)r * a.ws.ldu + j] = Acur[off];
        }
    }
    if (tid < BMAX) a.ws.piv[(size_t)row * BMAX + tid] = pv[tid];
    __syncthreads();                                     // G visible to the whole workgroup
    double *Mb = a.ws.Mb + (size_t)row * BMAX * BMAX;
    for (int e = tid; e < BMAX * BMAX; e += 512) {
        const int r = e / BMAX, s2 = e % BMAX;
        Mb[e] = (double)G[(size_t)r * a.ws.ldu + pv[s2]];
    }
}

// U = T G (T = L^-1 lower triangular, fp32 here), written in the new compact order; the diagonal
// loses sum_k U[k][j]^2; weights, diagonal, original indices and the index map are compacted.
// Only the owner of column j ever touches G[:, j], so once it has read the column it parks the
// column's new diagonal entry and new index there (rows 0..2) until the compaction.
__global__ __launch_bounds__(512) void dead_apply_kernel(DeadArgs a)
{
    __shared__ __align__(16) float Tl[BMAX][BMAX];       // T[k][r]
    __shared__ int pv[BMAX];
    const int row = blockIdx.x, tid = threadIdx.x, d = a.d;
    const int m = a.ws.m[row];
    const int ldu = a.ws.ldu;
    const double *Tb = a.ws.Tb + (size_t)row * BMAX * BMAX;
    for (int e = tid; e < BMAX * BMAX; e += 512) Tl[e / BMAX][e % BMAX] = (float)Tb[e];
    if (tid < BMAX) pv[tid] = a.ws.piv[(size_t)row * BMAX + tid];
    __syncthreads();
    float *G = a.ws.G + (size_t)row * BMAX * ldu;
    float *U = a.ws.U + (size_t)row * BMAX * ldu;
    double *gw = a.ws.w + (size_t)row * d;
    double *gd = a.ws.diag + (size_t)row * d;
    int *go = a.ws.orig + (size_t)row * d;
    int *gmap = a.ws.map + (size_t)row * d;

#pragma unroll 1
    for (int j = tid; j < m; j += 512) {
        int below = 0;
        bool piv = false;
        for (int s2 = 0; s2 < BMAX; ++s2) {
            below += (pv[s2] < j) ? 1 : 0;
            piv = piv || (pv[s2] == j);
        }
        int jnew = -1;
        double newd = 0.0;
        if (!piv) {
            jnew = j - below;
            float g[BMAX];
#pragma unroll
            for (int r = 0; r < BMAX; ++r) g[r] = G[(size_t)r * ldu + j];
            double dsum = 0.0;
#pragma unroll
            for (int k = 0; k < BMAX; ++k) {
                float acc = 0.f;
#pragma unroll
                for (int r = 0; r <= k; ++r) acc = fmaf(Tl[k][r], g[r], acc);
                U[(size_t)k * ldu + jnew] = acc;
                dsum += (double)acc * (double)acc;
                // one row of T at a time (otherwise its LDS reads are all issued up front)
                __builtin_amdgcn_sched_barrier(0);
            }
            newd = gd[j] - dsum;
        }
        const long long bits = __double_as_longlong(newd);
        G[j] = __int_as_float((int)(unsigned)bits);
        G[(size_t)ldu + j] = __int_as_float((int)(unsigned)((unsigned long long)bits >> 32));
        G[(size_t)2 * ldu + j] = __int_as_float(jnew);
    }
    // compaction: read the old entries, wait for everybody, write the new ones
    constexpr int EMAX = 10;                             // ceil(largest d / 512)
    double wv[EMAX], dv[EMAX];
    int ov[EMAX], jn[EMAX];
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
        const int j = tid + e * 512;
        jn[e] = -1;
        if (j >= m) continue;
        jn[e] = __float_as_int(G[(size_t)2 * ldu + j]);
        const unsigned lo = (unsigned)__float_as_int(G[j]), hi = (unsigned)__float_as_int(G[(size_t)ldu + j]);
        dv[e] = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
        wv[e] = gw[j];
        ov[e] = go[j];
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
        if (jn[e] < 0) continue;
        gw[jn[e]] = wv[e];
        gd[jn[e]] = dv[e];
        go[jn[e]] = ov[e];
        gmap[jn[e]] = tid + e * 512;
    }
    if (tid < BMAX) a.ws.invd[(size_t)row * BMAX + tid] = 1.f;
    if (tid == 0) {
        a.ws.m[row] = m - BMAX;
        a.ws.done[row] += BMAX;
        a.ws.nb[row] = BMAX;
    }
}

// ----------------------------------------------------------------------------------------- flush
struct FlushArgs {
    const float *A_old;
    size_t old_row_stride;   // 0 when every row still reads the shared H^-1
    int ld_old;
    int old_swz;             // layout of A_old: 0 plain row-major, 1 row-quad (A_new is always row-quad)
    float *A_new;
    size_t new_row_stride;
    int ld_new;
    int d, R, strips;
    BlockedWs ws;
};

// One workgroup (8 waves) per 128-row strip of one row's matrix; it walks the strip's 128-column
// tiles up to and including the diagonal one: the matrix is symmetric, so only its lower triangle
// is kept (the panel reads row p as "row part + column part").  In a diagonal tile the entries
// above the diagonal are neither read nor (except as don't-care slots of a 4-row store) written.  Wave (wm, wn) owns a 64 x 32 sub-tile = two 32x32 MFMA accumulators, which are loaded
// straight from the old matrix (one dword per lane: 32 consecutive columns of a row per half
// wave, i.e. whole 128-byte lines) and stored straight to the new one.  Accesses to the matrices
// are raw buffer loads / stores: a 32-bit byte offset per access instead of a 64-bit address
// (register pressure), and the hardware range check (offset >= size reads 0 / drops the store)
// replaces the per-element predicates.  A tile's loads are issued before its MFMAs, which do not
// depend on them.
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
constexpr unsigned kBufWord3 = 0x00020000u;   // raw buffer, 32-bit data format
constexpr int kFar = 0x40000000;              // byte offset beyond any matrix: "out of range"
// Cache policy bits of the matrix accesses (gfx950 buffer instructions: 1 = sc0, 2 = nt, 16 = sc1).
// The new matrix is written once and next read by another kernel: streaming stores keep it from
// displacing the U tiles and the old matrix's lines in L2 (flush 19.9 -> 18.9 ms on the 256 x 2304
// layer; nt, sc0+nt and sc1+nt within 1 % of each other, sc bits alone no change).  The loads stay
// cached: a lane's four rows of a column share sectors over four consecutive loads, and streaming
// loads made the kernel 25 % slower.
constexpr int kMatLoadPolicy = 0;
constexpr int kMatStorePolicy = 2 | 16;

// K is the block size: every row that still has steps to do has exactly K deferred eliminations
// (a row with fewer has finished and is skipped).  A strip is HALVES x 128 rows tall: the U tile
// of a column block, once in LDS, serves all the strip's halves (loading it is the expensive part
// of a tile next to the matrix traffic itself), and the F tile covers the whole strip.
template <int KMAX, int HALVES>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4))) void flush_kernel(FlushArgs a)
{
    constexpr int SR = HALVES * FT;          // rows per strip
    __shared__ __align__(16) float Fs[KMAX][SR + 4];
    __shared__ __align__(16) float Us[KMAX][FLD];
    __shared__ int rowoff_s[SR];   // byte offset of each strip row in the old matrix
    __shared__ int rowold_s[SR];   // its old compact index

    // Workgroups are dealt round-robin to the 8 XCDs: all strips of one row stay on one XCD, so
    // that its U panel and index map stay in that XCD's L2.  Within an XCD the rows go in groups
    // of G, and a group's workgroups run strip-major (the longest strip of each of its rows, then
    // the next longest, ...): long strips start first, and workgroups that start together take
    // equally long.  Measured against one row's strips in a run (lengths in a sawtooth): 10 % less
    // time per launch, 20 % where the strip count is a multiple of 4 (every fourth workgroup of
    // an XCD then got the long strips); G = 4, 8, 16, 32 gave 21.0, 20.3, 19.8, 20.4 ms of flush
    // time on the 256 x 2304 layer (22.2 ms before).
    const int L = blockIdx.x;
    const int nx = gridDim.x / (8 * a.strips);            // rows per XCD
    constexpr int G = 16;
    const int grp = (L / 8) / (G * a.strips), within = (L / 8) - grp * G * a.strips;
    const int rig = nx - G * grp < G ? nx - G * grp : G;  // rows in this group
    const int strip = a.strips - 1 - within / rig;
    const int row = (G * grp + within % rig) * 8 + (L % 8);
    if (row >= a.R) return;
    if (a.ws.nb[row] != KMAX || a.ws.done[row] >= a.ws.total[row]) return;
    constexpr int nb = KMAX;
    const int mn = a.ws.m[row];             // live size after the block (new compact space)
    const int i0 = strip * SR;
    if (i0 >= mn) return;

    const int d = a.d;
    const int *map = a.ws.map + (size_t)row * d;
    const int ldu = a.ws.ldu;
    const float *U = a.ws.U + (size_t)row * BMAX * ldu;    // u_k in the new compact order, 16-byte aligned rows
    const float *invd = a.ws.invd + (size_t)row * BMAX;
    const int ldo = a.ld_old, ldn = a.ld_new;
    constexpr int nbp = (nb + 1) & ~1;
    __amdgpu_buffer_rsrc_t rold = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(a.A_old + (size_t)row * a.old_row_stride), 0, (int)(((size_t)d * d + 3) / 4 * 16), kBufWord3);
    __amdgpu_buffer_rsrc_t rnew = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(a.A_new + (size_t)row * a.new_row_stride), 0, ((mn + 3) >> 2) * ldn * 16, kBufWord3);
    const int swz = a.old_swz;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int jl = wn * 32 + (lane & 31);
    const int lrow = 4 * (lane >> 5);        // the lane-dependent part of the accumulator row

    // F tile: F[k][i] = -u_k[i] / a_k for the strip's rows (four rows per 16-byte load; rows
    // beyond mn only reach outputs that are never stored); byte offsets of the strip's old rows
    for (int idx = tid; idx < nbp * (SR / 4); idx += 512) {
        int k = idx / (SR / 4), i = (idx % (SR / 4)) * 4;
        int ii = i0 + i;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k < nb && ii < mn) {
            v = *reinterpret_cast<const float4 *>(U + (size_t)k * ldu + ii);
            const float s = -invd[k];
            v.x = __fmul_rn(v.x, s); v.y = __fmul_rn(v.y, s); v.z = __fmul_rn(v.z, s); v.w = __fmul_rn(v.w, s);
        }
        *reinterpret_cast<float4 *>(&Fs[k][i]) = v;
    }
    for (int i = tid; i < SR; i += 512) {
        int o = (i0 + i < mn) ? map[i0 + i] : -1;
        rowold_s[i] = o;
        rowoff_s[i] = (o < 0) ? kFar : swz ? ((o >> 2) * ldo * 4 + (o & 3)) * 4 : o * ldo * 4;
    }

    // U tile staging: KMAX x 128 floats by 512 threads, four consecutive columns (16 bytes) each
    constexpr int UV = (KMAX * (FT / 4) + 511) / 512;
    float4 ureg[UV];
    auto fetch_u = [&](int j0) {
#pragma unroll
        for (int h = 0; h < UV; ++h) {
            int idx = tid + h * 512;
            int k = idx / (FT / 4), j = (idx % (FT / 4)) * 4;
            // a group that starts below mn may end beyond it: those columns hold old values of
            // the same buffer and only reach outputs that are never stored
            ureg[h] = (k < nb && j0 + j < mn) ? *reinterpret_cast<const float4 *>(U + (size_t)k * ldu + j0 + j)
                                               : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto stash_u = [&]() {
#pragma unroll
        for (int h = 0; h < UV; ++h) {
            int idx = tid + h * 512;
            int k = idx / (FT / 4), j = (idx % (FT / 4)) * 4;
            if (KMAX * (FT / 4) % 512 == 0 || k < KMAX) *reinterpret_cast<float4 *>(&Us[k][j]) = ureg[h];
        }
    };
    // strictly-lower tiles: element (i, j) sits at old[map i][map j]; rb = first strip row of the tile
    auto fetch_c = [&](floatx16(&c)[2], int jold, int rb) {
        const int joldB = (jold < 0) ? kFar : swz ? jold * 16 : jold * 4;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int ro = rowoff_s[rb + wm * 64 + mt * 32 + 8 * (v >> 2) + lrow + (v & 3)];
                c[mt][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rold, ro + joldB, 0, kMatLoadPolicy));
            }
    };
    // the diagonal tile: only entries on or below the diagonal exist
    auto fetch_c_diag = [&](floatx16(&c)[2], int jold, int rb) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int oi = rowold_s[rb + wm * 64 + mt * 32 + 8 * (v >> 2) + lrow + (v & 3)];
                int off = (jold < 0 || jold > oi) ? kFar
                          : swz ? (((oi >> 2) * ldo + jold) * 4 + (oi & 3)) * 4 : (oi * ldo + jold) * 4;
                c[mt][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rold, off, 0, kMatLoadPolicy));
            }
    };
    auto old_col = [&](int j) { return (j < mn) ? map[j] : -1; };
    // halves of the strip that hold rows at all
    const int nh = (mn - i0 + FT - 1) / FT < HALVES ? (mn - i0 + FT - 1) / FT : HALVES;

    // The strip's tiles in the order they are visited: column block j0 = 0, 128, ...; within a
    // column block the halves hf whose rows reach down to it (rows i0 + 128 hf .. >= j0).
    // (j0, hf) -> the next one; returns false after the last.
    auto advance = [&](int &j0, int &hf) {
        if (hf + 1 < nh) { hf += 1; return true; }
        j0 += FT;
        if (j0 >= mn) return false;
        // first half whose diagonal block is at or beyond column block j0
        int h0 = (j0 - i0) / FT;
        if (j0 <= i0) h0 = 0;
        if (h0 >= nh) return false;
        hf = h0;
        return true;
    };
    auto fetch_tile = [&](floatx16(&c)[2], int jold, int j0, int hf) {
        if (j0 == i0 + hf * FT) fetch_c_diag(c, jold, hf * FT);
        else fetch_c(c, jold, hf * FT);
    };

    // Per tile: the loads of the old entries are issued first, the rank-K update is summed on the
    // matrix cores into accumulators that start at zero while those loads are in flight, and the
    // two are added once at the end.  (Summing into the loaded entries instead would round every
    // one of the K partial sums at the magnitude of the matrix entry; this way the update, which is
    // small next to the entry, is rounded at its own magnitude, and the entry takes one rounding
    // per block.  The loads overlap with the same tile's MFMAs instead of the previous tile's.)
    int j0 = 0, hf = 0;
    int jold = old_col(jl);
    fetch_u(0);
    __syncthreads();                           // rowoff_s / rowold_s visible
    stash_u();
    __syncthreads();                           // Us and Fs visible
    floatx16 old[2], sum[2];
    for (;;) {
        fetch_tile(old, jold, j0, hf);
        int j0n = j0, hfn = hf;
        const bool more = advance(j0n, hfn);
        const bool new_col = more && j0n != j0;
        int joldn = jold;
        if (new_col) {
            fetch_u(j0n);
            joldn = old_col(j0n + jl);
        }
        const int kl = lane >> 5, il = lane & 31;
        const int rb = hf * FT;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sum[0][v] = 0.f; sum[1][v] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < nbp; kk += 2) {
            float a0 = Fs[kk + kl][rb + wm * 64 + il];
            float a1 = Fs[kk + kl][rb + wm * 64 + 32 + il];
            float b0 = Us[kk + kl][wn * 32 + il];
            sum[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, sum[0], 0, 0, 0);
            sum[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, sum[1], 0, 0, 0);
        }
        // store: a lane's registers 4q .. 4q+3 are four consecutive rows of its column = one
        // 16-byte slot of the row-quad layout
        const int jcol = j0 + jl;
        const int colB = (jcol < mn) ? jcol * 16 : kFar;
        const bool on_diag = (j0 == i0 + rb);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int qrow = i0 + rb + wm * 64 + mt * 32 + 8 * q + lrow;   // first row of the quad
                const int quad = qrow >> 2;
                if (on_diag && jcol > qrow + 3) continue;                   // wholly above the diagonal
                uintx4 v4 = {__float_as_uint(__fadd_rn(old[mt][4 * q], sum[mt][4 * q])),
                             __float_as_uint(__fadd_rn(old[mt][4 * q + 1], sum[mt][4 * q + 1])),
                             __float_as_uint(__fadd_rn(old[mt][4 * q + 2], sum[mt][4 * q + 2])),
                             __float_as_uint(__fadd_rn(old[mt][4 * q + 3], sum[mt][4 * q + 3]))};
                __builtin_amdgcn_raw_buffer_store_b128(v4, rnew, quad * ldn * 16 + colB, 0, kMatStorePolicy);
            }
        if (!more) break;
        if (new_col) {
            __syncthreads();                   // everyone is done reading Us
            stash_u();
            __syncthreads();                   // the new Us visible
        }
        j0 = j0n;
        hf = hfn;
        jold = joldn;
    }
}

// ------------------------------------------------------------------------------------- host side
struct Variant {
    int cap;   // largest live size it handles (T * EPT)
    int B;     // steps per block
    int (*launch)(int, int, size_t, hipStream_t, const PanelArgs &);
    int (*launch_block)(int, int, size_t, hipStream_t, const PanelArgs &);   // block pruning
};

#define OBC_VARIANT(T, EPT, BR, BL)                                           \
    { (T) * (EPT), (BR) + (BL), launch_panel_##T##_##EPT##_##BR##_##BL,       \
      launch_panel_block_##T##_##EPT##_##BR##_##BL }

const Variant kVariants[] = {
    OBC_VARIANT(256, 1, 64, 0),   OBC_VARIANT(1024, 1, 64, 0), OBC_VARIANT(512, 3, 48, 16),  OBC_VARIANT(512, 4, 40, 16),
    OBC_VARIANT(768, 3, 32, 16),  OBC_VARIANT(512, 6, 28, 12), OBC_VARIANT(512, 8, 20, 8),   OBC_VARIANT(512, 9, 16, 8),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

// Three of these fit on one CU (registers and LDS); with several times more rows than CUs that
// hides the per-step latency of one row behind the steps of two others (measured: a gain from
// three rows per CU on -- the 768 x 768 layer 7.6 -> 7.1 ms, its panels 3.5 -> 2.4 ms while the
// shorter blocks make its flushes 2.2 -> 2.9 ms; below that the shorter blocks cost more than the
// overlap brings).
const Variant kSharedCuVariant = OBC_VARIANT(256, 3, 32, 16);
constexpr int kSharedCuMinRows = 768;

const Variant *pick_variant(int m, int R)
{
    if (R >= kSharedCuMinRows && m <= kSharedCuVariant.cap && m > 256) return &kSharedCuVariant;
    for (int i = 0; i < kNumVariants; ++i)
        if (m <= kVariants[i].cap) return &kVariants[i];
    return nullptr;
}

}  // namespace

namespace obc_rows {

int blocked_max_d() { return kVariants[kNumVariants - 1].cap; }

size_t blocked_workspace_bytes(int R, int d) { return carve(nullptr, nullptr, R, d); }

int potrf64_batched_launch(obc_ctx *ctx, double *M, double *T, int R);   // invert.hip

int blocked_launch(obc_ctx *ctx, int mode, const float *W, const float *Hinv, int R, int d, int k_steps,
                   int nm_n, int nm_m, const int32_t *stop_counts, const float *delta,
                   const float *offset, int maxq, const uint8_t *live, int flags, int32_t *order, float *loss,
                   int32_t *codes, float *W_out, float *trace, int out_ld, void *ws, size_t ws_bytes)
{
    if (d > blocked_max_d())
        return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "row solver (blocked): d = %d exceeds the supported %d", d, blocked_max_d());
    BlockedWs bw;
    size_t need = carve(&bw, ws, R, d);
    if (!ws || ws_bytes < need)
        return obc_fail(ctx, OBC_ERR_WORKSPACE, "row solver: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    hipStream_t st = ctx->stream;
    ctx->chain_fresh = false;   // the set-up kernels below are not timed: the first timed launch records its own start

    InitArgs ia;
    ia.W = W; ia.Hinv = Hinv; ia.live_in = live; ia.stop_counts = stop_counts; ia.d = d;
    ia.k_steps = k_steps; ia.mode = mode; ia.ws = bw; ia.codes = codes; ia.W_out = W_out;
    blocked_init_kernel<<<R, 256, 0, st>>>(ia);
    OBC_LAUNCH_CHECK(ctx, "blocked_init_kernel");
    if (trace && k_steps > 0) {
        size_t n = (size_t)R * out_ld * d;
        unsigned blocks = (unsigned)((n / 4 + 256 * 8 - 1) / (256 * 8));
        if (blocks > 65535) blocks = 65535;
        if (blocks == 0) blocks = 1;
        fill_f32_kernel<<<blocks, 256, 0, st>>>(trace, n, 0.f);
        OBC_LAUNCH_CHECK(ctx, "fill_f32_kernel");
    }

    PanelArgs pa;
    pa.d = d; pa.nm_n = nm_n; pa.nm_m = nm_m; pa.delta = delta; pa.offset = offset; pa.maxq = maxq;
    pa.ws = bw; pa.order = order; pa.loss = loss; pa.codes = codes; pa.W_out = W_out; pa.trace = trace;
    pa.out_ld = out_ld; pa.status = ctx->d_status; pa.outliers = (flags & OBC_QUANT_OUTLIERS) ? 1 : 0;
    FlushArgs fa;
    fa.d = d; fa.R = R; fa.ws = bw;

    int host_total = (mode == MODE_QUANT || live) ? d : k_steps;   // upper bound over the rows
    const size_t lds_nm = nm_m > 0 ? obc_align_up((size_t)(d / nm_m), 16) : 0;
    const size_t mat_stride = obc_align_up((size_t)d * d, 4);   // floats between two rows' matrices
    int host_done = 0;
    int cur = -1;            // -1: the shared H^-1; otherwise index into Abuf
    int ld_cur = d;

    // where the rows' matrices are now, as the kernels take it
    auto cur_matrix = [&](const float **A, size_t *stride, int *swz) {
        *A = (cur < 0) ? Hinv : bw.Abuf[cur];
        *stride = (cur < 0) ? 0 : mat_stride;
        *swz = (cur < 0) ? 0 : 1;
    };
    // rank-K update and compaction of every row's matrix into the other buffer
    auto launch_flush = [&](int K) -> int {
        const int m_next = d - host_done;
        const int nxt = (cur < 0) ? 0 : 1 - cur;
        int swz;
        cur_matrix(&fa.A_old, &fa.old_row_stride, &swz);
        fa.ld_old = ld_cur;
        fa.old_swz = swz;
        fa.A_new = bw.Abuf[nxt];
        fa.new_row_stride = mat_stride;
        fa.ld_new = m_next;
        // strips of 256 rows where two workgroups' tiles fit in a CU's LDS, else 128
        const int halves = (K <= 48) ? 2 : 1;
        fa.strips = (m_next + halves * FT - 1) / (halves * FT);
        const int rows8 = (R + 7) / 8 * 8;
        {
            // one triangle of the surviving m_next x m_next part of every row's inverse is read and
            // written once
            const double tri = 0.5 * (double)m_next * (m_next + 1.0);   // entries of one triangle
            obc_scope sc(ctx, OBC_KERNEL_FLUSH, (double)R * 8.0 * tri, (double)R * 2.0 * K * tri);
            const dim3 grid(fa.strips * rows8);
            switch (K) {
            case 24: flush_kernel<24, 2><<<grid, 512, 0, st>>>(fa); break;
            case 28: flush_kernel<28, 2><<<grid, 512, 0, st>>>(fa); break;
            case 40: flush_kernel<40, 2><<<grid, 512, 0, st>>>(fa); break;
            case 48: flush_kernel<48, 2><<<grid, 512, 0, st>>>(fa); break;
            case 56: flush_kernel<56, 1><<<grid, 512, 0, st>>>(fa); break;
            case 64: flush_kernel<64, 1><<<grid, 512, 0, st>>>(fa); break;
            default: return obc_fail(ctx, OBC_ERR_BAD_ARG, "row solver: no flush kernel for block size %d", K);
            }
        }
        OBC_LAUNCH_CHECK(ctx, "flush_kernel");
        cur = nxt;
        ld_cur = fa.ld_new;
        return OBC_OK;
    };

    // ---- already-pruned indices, BMAX at a time, as long as every row has that many left.  The
    // smallest count over the rows is read back once (the only wait in this call).
    if (live && mode != MODE_BLOCK) {
        int scal[2] = {0, 0};
        min_ndead_kernel<<<1, 256, 0, st>>>(bw.ndead, bw.total, R, bw.scal);
        OBC_LAUNCH_CHECK(ctx, "min_ndead_kernel");
        OBC_HIP(ctx, hipMemcpyAsync(scal, bw.scal, sizeof(scal), hipMemcpyDeviceToHost, st));
        OBC_HIP(ctx, hipStreamSynchronize(st));
        const int min_dead = scal[0];
        if (scal[1] < host_total) host_total = scal[1];    // no launches past the longest row's last step
        int nfast = min_dead / BMAX;
        if (d - nfast * BMAX < BMAX) nfast -= 1;            // keep a matrix for the flush to write
        DeadArgs da;
        da.d = d; da.ws = bw;
        for (int it = 0; it < nfast; ++it) {
            const int m_max = d - host_done;
            cur_matrix(&da.A_cur, &da.a_row_stride, &da.swz);
            da.ld = ld_cur;
            {
                obc_scope sc(ctx, OBC_KERNEL_PANEL, (double)R * BMAX * 4.0 * m_max,
                             (double)R * BMAX * (double)BMAX * m_max);
                dead_gather_kernel<<<R, 512, 0, st>>>(da);
                OBC_LAUNCH_CHECK(ctx, "dead_gather_kernel");
                int rc = potrf64_batched_launch(ctx, bw.Mb, bw.Tb, R);
                if (rc != OBC_OK) return rc;
                dead_apply_kernel<<<R, 512, 0, st>>>(da);
                OBC_LAUNCH_CHECK(ctx, "dead_apply_kernel");
            }
            host_done += BMAX;
            int rc = launch_flush(BMAX);
            if (rc != OBC_OK) return rc;
        }
    }

    while (host_done < host_total) {
        const int m_max = d - host_done;
        const Variant *v = pick_variant(m_max, R);
        int swz;
        cur_matrix(&pa.A_cur, &pa.a_row_stride, &swz);
        pa.ld = ld_cur;
        pa.swz = swz;
        {
            // a panel reads one (corrected) matrix row per step: 4 m bytes, and does ~B m flops on it
            const int steps = (host_total - host_done < v->B) ? host_total - host_done : v->B;
            obc_scope sc(ctx, OBC_KERNEL_PANEL, (double)R * steps * 4.0 * m_max,
                         (double)R * steps * (double)steps * m_max);
            if ((mode == MODE_BLOCK ? v->launch_block : v->launch)(mode, R, lds_nm, st, pa) != 0)
                return obc_fail(ctx, OBC_ERR_HIP, "panel kernel: cannot set its dynamic LDS size");
        }
        OBC_LAUNCH_CHECK(ctx, "panel_kernel");
        host_done += v->B;
        if (host_done >= host_total) break;
        int rc = launch_flush(v->B);
        if (rc != OBC_OK) return rc;
    }
    return OBC_OK;
}

}  // namespace obc_rows
