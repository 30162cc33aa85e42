// Row solver, blocked strategy (placeholder: forwards to the rank-1 solver until the blocked
// kernels land).
#include "rows_common.h"

namespace obc_rows {
size_t rank1_workspace_bytes(int R, int d);
int rank1_launch(obc_ctx *ctx, int mode, const float *W, const float *Hinv, int R, int d, int k_steps,
                 int nm_n, int nm_m, const int32_t *stop_counts, const float *delta,
                 const float *offset, int maxq, const uint8_t *live, int32_t *order, float *loss,
                 int32_t *codes, float *W_out, float *trace, int out_ld, void *ws, size_t ws_bytes);

size_t blocked_workspace_bytes(int R, int d) { return obc_align_up((size_t)R * d * d * sizeof(float), 256); }

int blocked_launch(obc_ctx *ctx, int mode, const float *W, const float *Hinv, int R, int d, int k_steps,
                   int nm_n, int nm_m, const int32_t *stop_counts, const float *delta,
                   const float *offset, int maxq, const uint8_t *live, int32_t *order, float *loss,
                   int32_t *codes, float *W_out, float *trace, int out_ld, void *ws, size_t ws_bytes)
{
    return rank1_launch(ctx, mode, W, Hinv, R, d, k_steps, nm_n, nm_m, stop_counts, delta, offset, maxq,
                        live, order, loss, codes, W_out, trace, out_ld, ws, ws_bytes);
}
}  // namespace obc_rows
