/*
 * libobc -- the layer-wise ExactOBS / OBQ solver of "Optimal Brain Compression"
 * (arxiv 2208.11580) for one AMD MI355X (gfx950).
 *
 * Problem (Sec. 3, eq. (2)): for a layer with weights W (d_row x d_col) and calibration
 * inputs X (d_col x N) find compressed weights W^ minimising ||W X - W^ X||^2 under a
 * sparsity or quantization constraint.  The path is
 *
 *     X --obc_hessian--> H = 2 X X^T + lambda I --obc_invert--> H^-1
 *       --obc_prune_rows / obc_quant_rows--> per-row order P, loss changes L, weights
 *       --obc_global_select--> per-row counts and layer mask
 *       --obc_gather_trace (from the pruning trace) or obc_reconstruct_rows (closed form)--> W^
 *
 * Conventions
 *  - Every array argument is a DEVICE pointer owned by the caller, row-major and
 *    contiguous unless a leading dimension is given.  `const` inputs are never written.
 *    The library allocates no large memory: scratch is a caller-provided workspace whose
 *    size comes from the matching *_workspace_bytes query (host call, no GPU work).
 *  - All work is enqueued on the HIP stream given to obc_create and is asynchronous with
 *    respect to the host, except obc_invert, obc_refit and obc_check, which wait for the stream,
 *    and obc_prune_rows / obc_quant_rows when given a live mask, which wait once at their start
 *    (the smallest number of already-pruned weights over the rows is read back).
 *  - Every call returns 0 (OBC_OK) or a negative OBC_ERR_* code; nothing throws or aborts
 *    across this boundary.  obc_last_error gives a text for the last failure on a context.
 *    Conditions only a kernel can see (a non-positive or non-finite pivot [H^-1]_pp) are
 *    latched on the device and reported by obc_check.
 *  - Results are deterministic: the same inputs give bit-identical outputs.
 *  - Matrices and results are fp32.  obc_invert, obc_refit and obc_reconstruct_rows factorise in fp64
 *    internally and round the result; the row solvers keep a row's weights and the diagonal of its
 *    inverse in fp64 and the matrix itself in fp32.
 */
#ifndef OBC_H
#define OBC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OBC_OK 0
#define OBC_ERR_BAD_ARG (-1)   /* null pointer, negative size, value out of range */
#define OBC_ERR_BAD_SHAPE (-2) /* sizes inconsistent with each other (d % M != 0, k > d, ...) */
#define OBC_ERR_NOT_SPD (-3)   /* obc_invert met a non-positive Cholesky pivot */
#define OBC_ERR_WORKSPACE (-4) /* workspace missing or smaller than the query says (or than a row needs) */
#define OBC_ERR_NUMERIC (-5)   /* a row solver met a non-positive / non-finite [H^-1]_pp */
#define OBC_ERR_HIP (-6)       /* a HIP runtime call failed */

/* Row-solver strategies (argument `strategy` below).  AUTO picks the rank-1 solver with the
 * row's matrix resident in LDS for d_col <= 192, the blocked solver up to d_col = 4608 and the
 * streamed rank-1 solver beyond (as far as its per-row vectors fit in LDS, d_col <= ~5600;
 * larger d_col returns OBC_ERR_BAD_SHAPE). */
#define OBC_STRATEGY_AUTO 0
#define OBC_STRATEGY_RANK1 1   /* literal Algorithm 1: one rank-1 elimination per step */
#define OBC_STRATEGY_BLOCKED 2 /* same arithmetic result, eliminations applied in blocks */

typedef struct obc_ctx obc_ctx;

/* Create a context bound to `hip_stream` (a hipStream_t; NULL = the default stream) on the
 * current device.  The context owns only a few bytes of device memory (the error latch). */
int obc_create(obc_ctx **ctx, void *hip_stream);
int obc_destroy(obc_ctx *ctx);
const char *obc_last_error(const obc_ctx *ctx);
const char *obc_version(void);

/* Wait for the context's stream and return the first error a kernel latched since the last
 * obc_check (OBC_ERR_NUMERIC, OBC_ERR_NOT_SPD) or OBC_OK; clears the latch. */
int obc_check(obc_ctx *ctx);

/* ---- Measurement support (not part of the method) ---------------------------------------
 * Between obc_profile_begin and obc_profile_end every launch of the row solvers' kernels is
 * bracketed by HIP events on the context's stream.  obc_profile_end waits for the stream and
 * fills one obc_kernel_stat per kernel class: launches, summed duration, and the algorithmic
 * bytes / flops of those launches (what the method needs moved / computed under the schedule
 * the kernel implements: the flush reads and writes one triangle of the surviving m x m part of
 * each row's (symmetric) inverse once per block of B steps, 8 m(m+1)/2 bytes and B m(m+1) flops
 * per row; a panel reads one matrix row per step; the rank-1 kernel moves 8 m^2 bytes per step). */
#define OBC_KERNEL_PANEL 0
#define OBC_KERNEL_FLUSH 1
#define OBC_KERNEL_RANK1 2
#define OBC_KERNEL_CLASSES 3
typedef struct obc_kernel_stat {
    int launches;
    double ms;
    double bytes;
    double flops;
} obc_kernel_stat;
int obc_profile_begin(obc_ctx *ctx);
int obc_profile_end(obc_ctx *ctx, obc_kernel_stat stats[OBC_KERNEL_CLASSES]);

/* What this GPU's memory system gives the plainest kernels (16-byte accesses, every compute unit
 * busy): kind 0 reads `bytes` from src, 1 writes `bytes` to dst, 2 copies src to dst; streaming != 0
 * makes the stores non-temporal (as the row solver's matrix stores are).  Runs one warm-up pass and
 * `reps` timed passes on the context's stream, waits, and returns the mean milliseconds per pass:
 * the measured ceiling that HBM-bound kernels are compared with.  bytes must be a multiple of 16,
 * the buffers 16-byte aligned; for kind 0 the buffer must hold words whose lowest bit is clear
 * (e.g. all zero).  Synchronous. */
int obc_membench(obc_ctx *ctx, int kind, int streaming, const void *src, void *dst, size_t bytes,
                 int reps, double *ms_per_pass);

/* What the matrix cores of this GPU sustain on nothing but independent MFMA instructions, four
 * wavefronts on every SIMD: kind 0 = v_mfma_f32_32x32x2_f32 (the Hessian's instruction), kind 1 =
 * v_mfma_f64_16x16x4_f64 (the factorisation's).  Every wavefront issues 4 * iters instructions per
 * pass; one warm-up pass and `reps` timed ones on the context's stream.  Returns the mean
 * milliseconds per pass and the flops of a pass.  Synchronous. */
int obc_mfmabench(obc_ctx *ctx, int kind, int iters, int reps, double *ms_per_pass, double *flops_per_pass);

/* ---- Sec. 4: H = 2 X X^T, "Implementation Details": dampening -------------------------
 * X: d x N fp32 with leading dimension ldx >= N (element (j, n) at X[j*ldx + n]).
 * H: d x d fp32.  accumulate == 0: H = 2 X X^T;  accumulate != 0: H += 2 X X^T (calibration
 * data arriving in batches; samples only ever need to be accumulated once).
 * damp_rel >= 0: after the product, add damp_rel * mean(diag(H)) to the diagonal (call with
 * damp_rel < 0 for all batches but the last).  The sum over samples is not divided by N. */
int obc_hessian_workspace_bytes(int d, int64_t N, size_t *bytes);
int obc_hessian(obc_ctx *ctx, const float *X, int d, int64_t N, int64_t ldx, float damp_rel,
                int accumulate, float *H, void *ws, size_t ws_bytes);

/* ---- Sec. 4 Step 1: the inverse every row starts from ---------------------------------
 * In-place inverse of the symmetric positive definite d x d matrix H through its Cholesky
 * factor (fp64 inside, result rounded to fp32 and exactly symmetric).  Synchronous.
 * Returns OBC_ERR_NOT_SPD (H is then undefined) when a pivot is not positive. */
int obc_invert_workspace_bytes(int d, size_t *bytes);
int obc_invert(obc_ctx *ctx, float *H_inout, int d, void *ws, size_t ws_bytes);

/* ---- Algorithm 1 (+ N:M rule of Sec. 4) and Algorithm 3 --------------------------------
 * Workspace for obc_prune_rows / obc_quant_rows on R rows of width d. */
int obc_rows_workspace_bytes(int R, int d, int strategy, size_t *bytes);

/* Prune every row of W independently with Algorithm 1, each on a private copy of Hinv.
 *   W        R x d   weights (input)
 *   Hinv     d x d   symmetric inverse Hessian shared by all rows (input)
 *   k_steps  greedy steps per row, 0 <= k_steps <= d (N:M: <= d (M-N)/M)
 *   nm_n, nm_m   N:M pattern: a weight is eligible while its block of nm_m consecutive
 *            indices has fewer than nm_m - nm_n pruned weights; nm_m == 0: unstructured
 *   stop_counts  nullable, R: row i stops after min(k_steps, stop_counts[i]) steps (replay of
 *            the counts chosen by obc_global_select); entries of order/loss beyond are untouched
 *   live     nullable, R x d: 0 marks a weight that is already pruned (Sec. 4 "Implementation
 *            Details": an already sparse matrix is handled on the dense sub-problem of its
 *            non-zeros).  Those indices are first removed from the row's inverse (Lemma 1, no
 *            weight change, nothing recorded), keep weight 0, and the k_steps greedy steps run
 *            on the survivors (a row with fewer survivors stops when none is left; entries of
 *            order / loss beyond are untouched).  Not combined with the N:M rule.
 *   order    R x k_steps int32 out: index pruned at each step
 *   loss     R x k_steps fp32 out: loss change w_p^2 / (2 [H^-1]_pp) of each step
 *   W_out    R x d out: the row after its last step (pruned weights exactly 0)
 *   trace    nullable, R x k_steps x d out: the row after every step (the "pruning trace" of
 *            Sec. 4 Step 2, kept in HBM here); entries of steps a row does not take (stop_counts,
 *            fewer survivors than k_steps) are zero
 * Ties in the argmin go to the lowest index. */
int obc_prune_rows(obc_ctx *ctx, const float *W, const float *Hinv, int R, int d, int k_steps,
                   int nm_n, int nm_m, const int32_t *stop_counts, const uint8_t *live, int32_t *order,
                   float *loss, float *W_out, float *trace, int strategy, void *ws, size_t ws_bytes);

/* Block pruning (Sec. 4 "Block-Sparsity", eq. (5)): Algorithm 1 on blocks of c consecutive
 * weights (block b = indices b c .. b c + c - 1; d must be a multiple of c, 1 <= c <= 8).  Each
 * step takes the live block P with the smallest w_P^T ((H^-1)_P)^-1 w_P, moves the remaining
 * weights by -H^-1[:,P] ((H^-1)_P)^-1 w_P and removes P from the inverse (Lemma 1 for every p in
 * P).  Arguments as obc_prune_rows, counted in blocks:
 *   k_blocks     steps per row (<= d / c); stop_counts nullable, per-row step limits in blocks
 *   order, loss  R x k_blocks out: block index per step and its loss change
 *                w_P^T ((H^-1)_P)^-1 w_P / 2
 *   trace        nullable, R x k_blocks x d out: the row after every block step
 * The traces feed obc_global_select (with d := k_blocks) and obc_gather_trace unchanged.
 * Workspace: obc_blocks_workspace_bytes.  strategy: OBC_STRATEGY_BLOCKED handles c = 4 (and
 * c = 1, which is obc_prune_rows) and returns OBC_ERR_BAD_ARG otherwise; OBC_STRATEGY_AUTO uses
 * it for those and the rank-1 solver for every other block size. */
int obc_blocks_workspace_bytes(int R, int d, int c, int strategy, size_t *bytes);
int obc_prune_blocks(obc_ctx *ctx, const float *W, const float *Hinv, int R, int d, int c, int k_blocks,
                     const int32_t *stop_counts, int32_t *order, float *loss, float *W_out, float *trace,
                     int strategy, void *ws, size_t ws_bytes);

/* Flags of obc_quant_rows. */
#define OBC_QUANT_OUTLIERS 1   /* Sec. 5 "Quantization Outliers": while any live weight of the row has
                                  a quantization error |q(w) - w| > delta / 2, the greedy choice runs
                                  over those weights only (same score, same tie rule) */

/* Quantize every row with Algorithm 3 on the caller's per-row uniform grid
 *   q(w) = offset[i] + delta[i] * clamp(rne((w - offset[i]) / delta[i]), 0, maxq)
 * (rne = round half to even; the kernels evaluate the quotient in fp64 as a product with the fp64
 * reciprocal of delta[i], in the candidate scores and when the chosen weight is written alike).
 *   flags    0 or OBC_QUANT_OUTLIERS
 *   live     nullable, R x d: 0 marks an already pruned weight; those are first removed from the
 *            row's inverse (Lemma 1, no weight change) so that OBQ runs on the dense sub-problem
 *            of the survivors; they keep weight 0 and get code -1.
 *   order, loss   R x d: entries [0, #live_i) are written for row i
 *   codes    R x d int32 out: grid code of each weight at the moment it was chosen
 *   W_out    R x d out: dequantized weights offset + delta * code */
int obc_quant_rows(obc_ctx *ctx, const float *W, const float *Hinv, int R, int d,
                   const float *delta, const float *offset, int maxq, const uint8_t *live, int flags,
                   int32_t *order, float *loss, int32_t *codes, float *W_out, int strategy,
                   void *ws, size_t ws_bytes);

/* Per-row grid over the live weights (live nullable = all live).
 *   symmetric == 0: asymmetric min-max grid, offset = min, delta = (max - min) / maxq
 *   symmetric != 0: grid symmetric about zero, offset = -max|w|, delta = 2 max|w| / maxq
 * delta = 1 when the range is empty (constant row, all-zero row, no live weight). */
int obc_minmax_grid(obc_ctx *ctx, const float *W, const uint8_t *live, int R, int d, int maxq,
                    int symmetric, float *delta, float *offset);

/* ---- Appendix "Sequential Quantization with OBQ": re-fit of the dense weights ------------
 * When the layer's inputs X come from the already compressed model, the dense weights are first
 * re-optimised for them by the closed form of linear regression, W^T = (X X^T)^-1 X Y^T (Y = the
 * dense model's outputs of this layer, d_row x N); then their gradient is zero again and OBQ
 * applies.  With H = 2 X X^T (+ dampening, as obc_hessian forms it) and C = 2 Y X^T this is
 * W = C H^-1: the minimiser of the quadratic whose Hessian the row solvers use.  C is accumulated
 * over batches like H. */

/* Workspace of obc_cross. */
int obc_cross_workspace_bytes(int d_row, int d_col, int64_t N, size_t *bytes);

/* C (d_row x d_col, device, row-major) = 2 Y X^T, or C += 2 Y X^T when accumulate != 0.
 *   X  device, d_col x N, leading dimension ldx >= N;  Y  device, d_row x N, ldy >= N.
 * fp32 matrix cores, fixed summation order (deterministic).  Errors as obc_hessian. */
int obc_cross(obc_ctx *ctx, const float *X, const float *Y, int d_col, int d_row, int64_t N, int64_t ldx,
              int64_t ldy, int accumulate, float *C, void *ws, size_t ws_bytes);

/* Workspace of obc_refit. */
int obc_refit_workspace_bytes(int d_col, int d_row, size_t *bytes);

/* W_out (d_row x d_col, device) = C H^-1 through the fp64 Cholesky factor of H (H^-1 itself is
 * never rounded to fp32 on the way).
 *   H   device, d_col x d_col, the dampened Hessian; left untouched when invert_in_place == 0,
 *       replaced by its inverse exactly as obc_invert does otherwise (the factorisation is shared)
 *   C   device, d_row x d_col, from obc_cross
 * Synchronises.  OBC_ERR_NOT_SPD as obc_invert. */
int obc_refit(obc_ctx *ctx, float *H, int d_col, const float *C, int d_row, float *W_out,
              int invert_in_place, void *ws, size_t ws_bytes);

/* ---- Appendix Algorithm 2: the global step ---------------------------------------------
 * From the per-row loss traces (loss, order: R x d as written by obc_prune_rows with
 * k_steps == d) find how many weights each row gives up when k weights are pruned from the
 * layer: k times, the row whose next loss change is smallest advances (lowest row on ties).
 *   counts   R int32 out;  mask  R x d uint8 out, 1 = pruned. */
int obc_global_select_workspace_bytes(int R, int d, size_t *bytes);
int obc_global_select(obc_ctx *ctx, const float *loss, const int32_t *order, int R, int d,
                      int64_t k, int32_t *counts, uint8_t *mask, void *ws, size_t ws_bytes);

/* The same global step for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid allocation): the
 * scratch is a device array built into the library, OBC_SELECT_STATIC_SCRATCH_BYTES per GPU, held
 * from the library's load to the end of the process.  Arguments, results and errors as
 * obc_global_select; layers beyond OBC_SELECT_STATIC_MAX_WEIGHTS weights or
 * OBC_SELECT_STATIC_MAX_ROWS rows are refused with OBC_ERR_WORKSPACE.  The call allocates and
 * frees nothing, waits for nothing and clears its scratch with kernels.  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (two streams, two contexts) race;
 * calls on one stream are ordered and safe. */
#define OBC_SELECT_STATIC_MAX_WEIGHTS 2359296 /* R * d, e.g. 512 x 4608, 768 x 3072, 3072 x 768 */
#define OBC_SELECT_STATIC_MAX_ROWS 8192
#define OBC_SELECT_STATIC_SCRATCH_BYTES (4 * OBC_SELECT_STATIC_MAX_WEIGHTS + 2 * 4 * OBC_SELECT_STATIC_MAX_ROWS + 2048)
int obc_global_select_static(obc_ctx *ctx, const float *loss, const int32_t *order, int R, int d,
                             int64_t k, int32_t *counts, uint8_t *mask);

/* ---- Sec. 4 Step 2: weights of the chosen mask from the pruning trace -------------------
 * W_out[i] = trace[i][counts[i]-1] (the row after counts[i] steps), or W[i] when counts[i] == 0.
 * trace is R x k_steps x d with k_steps >= max counts. */
int obc_gather_trace(obc_ctx *ctx, const float *W, const float *trace, const int32_t *counts,
                     int R, int d, int k_steps, float *W_out);

/* ---- Sec. 4 Step 2: weights of a mask by the group-OBS closed form ------------------------
 * For every row, with P the indices the mask marks as pruned,
 *     W_out = w - H^-1[:, P] ((H^-1)[P, P])^-1 w_P,    W_out[P] = 0 exactly
 * (the sign as in eq. (5)), from the ORIGINAL weights W and inverse Hessian Hinv: neither a trace nor a
 * second run of the greedy loop is needed (the paper's cheaper way to a row's weights once the global
 * step has fixed its mask).  The solve runs in fp64 through a Cholesky factorisation per row.
 *   mask        R x d uint8, non-zero = pruned (as obc_global_select writes it)
 *   max_pruned  upper bound on the pruned weights of any row, 0 <= max_pruned <= d; it sizes the
 *               workspace (8 max_pruned^2 bytes per row, roughly).  A row with more pruned weights
 *               than that is returned unchanged (a copy of W) and OBC_ERR_WORKSPACE is latched for
 *               obc_check; a non-positive pivot latches OBC_ERR_NUMERIC.
 * Asynchronous. */
int obc_reconstruct_workspace_bytes(int R, int d, int max_pruned, size_t *bytes);
int obc_reconstruct_rows(obc_ctx *ctx, const float *W, const float *Hinv, const uint8_t *mask, int R, int d,
                         int max_pruned, float *W_out, void *ws, size_t ws_bytes);

#ifdef __cplusplus
}
#endif
#endif /* OBC_H */
