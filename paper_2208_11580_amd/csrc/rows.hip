// C-ABI entry points of the per-row solvers (argument checks, strategy dispatch) and the two
// small per-row helpers: the min-max quantization grid and the gather from the pruning trace.
#include "rows_common.h"

namespace obc_rows {
bool rank1_lds_resident(int d, int nm_m);
size_t rank1_workspace_bytes(int R, int d);
int rank1_launch(obc_ctx *ctx, int mode, const float *W, const float *Hinv, int R, int d, int k_steps,
                 int nm_n, int nm_m, int blk_c, const int32_t *stop_counts, const float *delta,
                 const float *offset, int maxq, const uint8_t *live, int flags, int32_t *order, float *loss,
                 int32_t *codes, float *W_out, float *trace, int out_ld, void *ws, size_t ws_bytes);
size_t blocked_workspace_bytes(int R, int d);
int blocked_max_d();
int blocked_launch(obc_ctx *ctx, int mode, const float *W, const float *Hinv, int R, int d, int k_steps,
                   int nm_n, int nm_m, const int32_t *stop_counts, const float *delta,
                   const float *offset, int maxq, const uint8_t *live, int flags, int32_t *order, float *loss,
                   int32_t *codes, float *W_out, float *trace, int out_ld, void *ws, size_t ws_bytes);
}  // namespace obc_rows

namespace {

using namespace obc_rows;

int pick_strategy(int strategy, int d)
{
    if (strategy == OBC_STRATEGY_RANK1 || strategy == OBC_STRATEGY_BLOCKED) return strategy;
    if (rank1_lds_resident(d, 8)) return OBC_STRATEGY_RANK1;
    return d <= blocked_max_d() ? OBC_STRATEGY_BLOCKED : OBC_STRATEGY_RANK1;
}

// Block pruning: the deferred-update solver handles blocks of 4; -1 when it is asked for others.
int pick_block_strategy(int strategy, int d, int c)
{
    if (c == 1) return pick_strategy(strategy, d);
    if (strategy == OBC_STRATEGY_BLOCKED) return (c == 4 && d <= blocked_max_d()) ? OBC_STRATEGY_BLOCKED : -1;
    if (strategy == OBC_STRATEGY_RANK1 || c != 4) return OBC_STRATEGY_RANK1;
    return pick_strategy(OBC_STRATEGY_AUTO, d);
}

// The row's grid over its live weights (min-max, or symmetric about zero); one wave per row.
__global__ __launch_bounds__(256) void minmax_grid_kernel(const float *__restrict__ W,
                                                          const uint8_t *__restrict__ live, int R,
                                                          int d, int maxq, int symmetric,
                                                          float *__restrict__ delta,
                                                          float *__restrict__ offset)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= R) return;
    float lo = __builtin_inff(), hi = -__builtin_inff();
    for (int j = lane; j < d; j += 64) {
        if (live && !live[(size_t)row * d + j]) continue;
        float v = W[(size_t)row * d + j];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, 64));
        hi = fmaxf(hi, __shfl_xor(hi, off, 64));
    }
    if (lane == 0) {
        if (symmetric) {
            float m = (lo <= hi) ? fmaxf(fabsf(lo), fabsf(hi)) : 0.f;
            bool ok = (m > 0.f) && maxq > 0;
            delta[row] = ok ? __fdiv_rn(__fmul_rn(2.f, m), (float)maxq) : 1.f;
            offset[row] = -m;
        } else {
            bool ok = (hi > lo) && maxq > 0;
            delta[row] = ok ? __fdiv_rn(__fsub_rn(hi, lo), (float)maxq) : 1.f;
            offset[row] = (lo <= hi) ? lo : 0.f;
        }
    }
}

__global__ __launch_bounds__(256) void gather_trace_kernel(const float *__restrict__ W,
                                                           const float *__restrict__ trace,
                                                           const int32_t *__restrict__ counts, int d,
                                                           int k_steps, float *__restrict__ W_out)
{
    const int row = blockIdx.x;
    int c = counts[row];
    if (c > k_steps) c = k_steps;
    const float *src = (c <= 0) ? W + (size_t)row * d : trace + ((size_t)row * k_steps + (c - 1)) * d;
    for (int j = threadIdx.x; j < d; j += blockDim.x) W_out[(size_t)row * d + j] = src[j];
}

}  // namespace

extern "C" {

int obc_rows_workspace_bytes(int R, int d, int strategy, size_t *bytes)
{
    if (!bytes || R < 0 || d <= 0) return OBC_ERR_BAD_ARG;
    if (strategy < OBC_STRATEGY_AUTO || strategy > OBC_STRATEGY_BLOCKED) return OBC_ERR_BAD_ARG;
    int s = pick_strategy(strategy, d);
    *bytes = (s == OBC_STRATEGY_RANK1) ? rank1_workspace_bytes(R, d) : blocked_workspace_bytes(R, d);
    return OBC_OK;
}

int obc_prune_rows(obc_ctx *ctx, const float *W, const float *Hinv, int R, int d, int k_steps,
                   int nm_n, int nm_m, const int32_t *stop_counts, const uint8_t *live, int32_t *order,
                   float *loss, float *W_out, float *trace, int strategy, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (R < 0 || d <= 0 || k_steps < 0)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_rows: negative size");
    if (R > 0 && (!W || !Hinv || !W_out || (k_steps > 0 && (!order || !loss))))
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_rows: null W, Hinv, order, loss or W_out");
    if (strategy < OBC_STRATEGY_AUTO || strategy > OBC_STRATEGY_BLOCKED)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_rows: unknown strategy %d", strategy);
    if (k_steps > d)
        return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "obc_prune_rows: k_steps (%d) > d (%d)", k_steps, d);
    if (nm_m < 0 || nm_n < 0 || (nm_m > 0 && nm_n > nm_m) || nm_m > 255)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_rows: bad N:M pattern %d:%d", nm_n, nm_m);
    if (nm_m > 0 && live)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_rows: the N:M rule applies to dense rows (live must be null)");
    if (nm_m > 0) {
        if (d % nm_m != 0)
            return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "obc_prune_rows: d (%d) is not a multiple of M (%d)", d, nm_m);
        if ((int64_t)k_steps > (int64_t)(d / nm_m) * (nm_m - nm_n))
            return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "obc_prune_rows: k_steps (%d) exceeds what %d:%d allows", k_steps, nm_n, nm_m);
    }
    if (R == 0) return OBC_OK;
    int s = pick_strategy(strategy, d);
    if (s == OBC_STRATEGY_RANK1)
        return rank1_launch(ctx, MODE_PRUNE, W, Hinv, R, d, k_steps, nm_n, nm_m, 0, stop_counts, nullptr,
                            nullptr, 0, live, 0, order, loss, nullptr, W_out, trace, k_steps, ws, ws_bytes);
    return blocked_launch(ctx, MODE_PRUNE, W, Hinv, R, d, k_steps, nm_n, nm_m, stop_counts, nullptr,
                          nullptr, 0, live, 0, order, loss, nullptr, W_out, trace, k_steps, ws, ws_bytes);
}

int obc_prune_blocks(obc_ctx *ctx, const float *W, const float *Hinv, int R, int d, int c, int k_blocks,
                     const int32_t *stop_counts, int32_t *order, float *loss, float *W_out, float *trace,
                     int strategy, void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (R < 0 || d <= 0 || k_blocks < 0)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_blocks: negative size");
    if (c < 1 || c > 8)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_blocks: block size %d outside 1..8", c);
    if (d % c != 0)
        return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "obc_prune_blocks: d (%d) is not a multiple of the block size (%d)", d, c);
    if (k_blocks > d / c)
        return obc_fail(ctx, OBC_ERR_BAD_SHAPE, "obc_prune_blocks: k_blocks (%d) > d / c (%d)", k_blocks, d / c);
    if (R > 0 && (!W || !Hinv || !W_out || (k_blocks > 0 && (!order || !loss))))
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_blocks: null W, Hinv, order, loss or W_out");
    if (strategy < OBC_STRATEGY_AUTO || strategy > OBC_STRATEGY_BLOCKED)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_blocks: unknown strategy %d", strategy);
    if (c == 1)   // blocks of one weight: Algorithm 1 itself
        return obc_prune_rows(ctx, W, Hinv, R, d, k_blocks, 0, 0, stop_counts, nullptr, order, loss, W_out, trace,
                              strategy, ws, ws_bytes);
    const int s = pick_block_strategy(strategy, d, c);
    if (s < 0)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_prune_blocks: the deferred-update solver handles blocks of 4 only");
    if (R == 0) return OBC_OK;
    if (s == OBC_STRATEGY_RANK1)
        return rank1_launch(ctx, MODE_BLOCK, W, Hinv, R, d, k_blocks, 0, 0, c, stop_counts, nullptr, nullptr, 0,
                            nullptr, 0, order, loss, nullptr, W_out, trace, k_blocks, ws, ws_bytes);
    return blocked_launch(ctx, MODE_BLOCK, W, Hinv, R, d, k_blocks * 4, 0, 0, stop_counts, nullptr, nullptr, 0,
                          nullptr, 0, order, loss, nullptr, W_out, trace, k_blocks, ws, ws_bytes);
}

int obc_blocks_workspace_bytes(int R, int d, int c, int strategy, size_t *bytes)
{
    if (!bytes || R < 0 || d <= 0 || c < 1 || c > 8) return OBC_ERR_BAD_ARG;
    if (strategy < OBC_STRATEGY_AUTO || strategy > OBC_STRATEGY_BLOCKED) return OBC_ERR_BAD_ARG;
    const int s = pick_block_strategy(strategy, d, c);
    if (s < 0) return OBC_ERR_BAD_ARG;
    *bytes = (s == OBC_STRATEGY_RANK1) ? rank1_workspace_bytes(R, d) : blocked_workspace_bytes(R, d);
    return OBC_OK;
}

int obc_quant_rows(obc_ctx *ctx, const float *W, const float *Hinv, int R, int d,
                   const float *delta, const float *offset, int maxq, const uint8_t *live, int flags,
                   int32_t *order, float *loss, int32_t *codes, float *W_out, int strategy,
                   void *ws, size_t ws_bytes)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (R < 0 || d <= 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_quant_rows: negative size");
    if (R > 0 && (!W || !Hinv || !delta || !offset || !order || !loss || !codes || !W_out))
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_quant_rows: null argument");
    if (maxq < 0 || maxq > (1 << 16))
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_quant_rows: maxq (%d) out of range", maxq);
    if (flags & ~OBC_QUANT_OUTLIERS)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_quant_rows: unknown flags 0x%x", flags);
    if (strategy < OBC_STRATEGY_AUTO || strategy > OBC_STRATEGY_BLOCKED)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_quant_rows: unknown strategy %d", strategy);
    if (R == 0) return OBC_OK;
    int s = pick_strategy(strategy, d);
    if (s == OBC_STRATEGY_RANK1)
        return rank1_launch(ctx, MODE_QUANT, W, Hinv, R, d, d, 0, 0, 0, nullptr, delta, offset, maxq, live,
                            flags, order, loss, codes, W_out, nullptr, d, ws, ws_bytes);
    return blocked_launch(ctx, MODE_QUANT, W, Hinv, R, d, d, 0, 0, nullptr, delta, offset, maxq, live,
                          flags, order, loss, codes, W_out, nullptr, d, ws, ws_bytes);
}

int obc_minmax_grid(obc_ctx *ctx, const float *W, const uint8_t *live, int R, int d, int maxq,
                    int symmetric, float *delta, float *offset)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!W || !delta || !offset) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_minmax_grid: null argument");
    if (R < 0 || d <= 0 || maxq < 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_minmax_grid: bad size");
    if (R == 0) return OBC_OK;
    minmax_grid_kernel<<<(R + 3) / 4, 256, 0, ctx->stream>>>(W, live, R, d, maxq, symmetric, delta, offset);
    OBC_LAUNCH_CHECK(ctx, "minmax_grid_kernel");
    return OBC_OK;
}

int obc_gather_trace(obc_ctx *ctx, const float *W, const float *trace, const int32_t *counts, int R,
                     int d, int k_steps, float *W_out)
{
    if (!ctx) return OBC_ERR_BAD_ARG;
    if (!W || !trace || !counts || !W_out)
        return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_gather_trace: null argument");
    if (R < 0 || d <= 0 || k_steps < 0) return obc_fail(ctx, OBC_ERR_BAD_ARG, "obc_gather_trace: bad size");
    if (R == 0) return OBC_OK;
    gather_trace_kernel<<<R, 256, 0, ctx->stream>>>(W, trace, counts, d, k_steps, W_out);
    OBC_LAUNCH_CHECK(ctx, "gather_trace_kernel");
    return OBC_OK;
}

}  // extern "C"
