// Device helpers shared by the per-row greedy solvers (Algorithm 1 / Algorithm 3 of
// arxiv 2208.11580): the quantizer, the candidate score and the lexicographic
// (score, index) argmin over a workgroup.
#pragma once

#include "common.h"

namespace obc_rows {

constexpr int MODE_PRUNE = 0;
constexpr int MODE_QUANT = 1;
constexpr int MODE_BLOCK = 2;   // pruning in blocks of c consecutive weights (Sec. 4 "Block-Sparsity")

struct Cand {
    float s;   // score; +inf when the thread saw no candidate
    int j;     // index; INT_MAX when none
};

__device__ inline bool cand_less(float s, int j, float bs, int bj)
{
    // strict order on (score, index): lowest score wins, lowest index on equal scores
    return (s < bs) || (s == bs && j < bj);
}

// grid code of Sec. 5's quant(.): clamp(rne((w - offset) / delta), 0, maxq)
__device__ inline float quant_code(float w, float delta, float offset, float maxq)
{
    float c = rintf(__fdiv_rn(__fsub_rn(w, offset), delta));
    c = fminf(fmaxf(c, 0.f), maxq);
    return c;
}

__device__ inline float dequant(float code, float delta, float offset)
{
    // the grid value in fp64, rounded once to fp32
    return (float)((double)offset + (double)delta * (double)code);
}

// eq. (3) / eq. (7): (target - w)^2 / [H^-1]_pp
__device__ inline float score_of(float w, float target, float app)
{
    float e = __fsub_rn(target, w);
    return __fdiv_rn(__fmul_rn(e, e), app);
}

// Outlier heuristic of Sec. 5: the score s >= 0 of an outlier is mapped, order-preserving and
// without loss (a reflection of its bit pattern), into the finite negative floats, so that every
// outlier sorts before every non-outlier and outliers keep their order among themselves.
__device__ inline float outlier_first(float s)
{
    unsigned u = __float_as_uint(s);
    if ((u & 0x80000000u) || s != s) return s;  // a negative or NaN score (broken diagonal) stays
    u = u < 0x7EFFFFFFu ? u : 0x7EFFFFFFu;      // keeps the image a normal number (scores above 1.7e38 tie)
    return __uint_as_float(0x80000000u | (0x7F7FFFFFu - u));
}

__device__ inline Cand wave_argmin(Cand c)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float os = __shfl_xor(c.s, off, 64);
        int oj = __shfl_xor(c.j, off, 64);
        if (cand_less(os, oj, c.s, c.j)) { c.s = os; c.j = oj; }
    }
    return c;
}

// Workgroup argmin; `red_s` / `red_j` hold one slot per wave (<= 16) plus a result slot [16].
// Every thread gets the winner.  Contains two barriers.
__device__ inline Cand block_argmin(Cand c, float *red_s, int *red_j)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwaves = (blockDim.x + 63) >> 6;
    c = wave_argmin(c);
    if (lane == 0) { red_s[wave] = c.s; red_j[wave] = c.j; }
    __syncthreads();
    if (wave == 0) {
        Cand r;
        r.s = (lane < nwaves) ? red_s[lane] : __builtin_inff();
        r.j = (lane < nwaves) ? red_j[lane] : 0x7fffffff;
        r = wave_argmin(r);
        if (lane == 0) { red_s[16] = r.s; red_j[16] = r.j; }
    }
    __syncthreads();
    Cand out;
    out.s = red_s[16];
    out.j = red_j[16];
    return out;
}

}  // namespace obc_rows
