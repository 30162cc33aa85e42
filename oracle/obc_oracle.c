/*
 * ExactOBS / OBQ oracle: a plain, slow, fp64 CPU implementation of the layer-wise
 * solver of "Optimal Brain Compression" (arxiv 2208.11580).
 *
 * THIS IS TEST INFRASTRUCTURE.  Only the test-suite, the smoke check and the
 * benchmark's cpu-baseline leg may call it.  It shares no code with the HIP
 * library and the HIP library never calls it.
 *
 * Everything is written as the paper states it, one step after another, with
 * no blocking, fusion or reordering:
 *   - Sec. 4 "Step 1", Algorithm 1   : prune one row (orc_row_solve, mode 0)
 *   - Sec. 4 "N:M Sparsity"          : eligibility filter in the same loop
 *   - Sec. 5 eq. (7), Appendix Alg. 3: quantize one row (orc_row_solve, mode 1)
 *   - Lemma 1                        : the rank-1 row/column removal inside the loop
 *   - Sec. 4 "Block-Sparsity", eq. (5): prune one row in blocks of c (orc_block_row_solve)
 *   - Appendix Algorithm 2           : global mask selection (orc_global_select)
 *   - Sec. 4 "Implementation Details": inverse of the dampened Hessian (orc_spd_inverse)
 *
 * Readings of points the paper leaves open (all listed in the design notes):
 *   - recorded loss change is w_p^2 / (2 [H^-1]_pp): with H = 2 X X^T this is the
 *     true change of the squared error; the selection score omits the 1/2.
 *   - ties in an argmin go to the lowest index (strict '<' scan).
 *   - an eliminated index is never read again (explicit live flags); the chosen
 *     weight is written exactly (0 or its grid value).
 *   - N:M: p is eligible iff its block of M consecutive indices has fewer than
 *     M - N pruned weights so far.
 *   - quantizer: code = clamp(rne((w - offset) / delta), 0, maxq),
 *     q(w) = offset + delta * code, round-half-to-even.
 *   - outlier heuristic of Sec. 5 ("Quantization Outliers"), optional: before each argmin, if any
 *     live weight has a quantization error |q(w_p) - w_p| > delta / 2 (possible only outside the
 *     clamped range of the grid), the argmin runs over those weights only; same score, same tie
 *     rule.  The paper gives the threshold as an example and does not say when it is tested;
 *     this reading is ours.
 *
 * Parity pins live in tests/test_oracle_pins.py (closed-form least squares,
 * loss identity, brute force, Lemma 1 against direct inversion, diagonal-H
 * special cases, invariances, literal whole-matrix OBS for Algorithm 2).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_BAD_ARG (-1)
#define ORC_NOT_SPD (-3)
#define ORC_NUMERIC (-5)

/* ---------------------------------------------------------------------------
 * Inverse of a symmetric positive definite matrix through its Cholesky factor.
 * H (d x d, row-major) is overwritten by H^-1.  Returns ORC_NOT_SPD when a
 * pivot is not positive.
 * ------------------------------------------------------------------------- */
int orc_spd_inverse(double *H, int d)
{
    if (!H || d <= 0) return ORC_BAD_ARG;
    double *L = (double *)calloc((size_t)d * d, sizeof(double));
    double *Li = (double *)calloc((size_t)d * d, sizeof(double));
    if (!L || !Li) { free(L); free(Li); return ORC_BAD_ARG; }

    /* H = L L^T, L lower triangular */
    for (int j = 0; j < d; ++j) {
        double s = H[(size_t)j * d + j];
        for (int k = 0; k < j; ++k) s -= L[(size_t)j * d + k] * L[(size_t)j * d + k];
        if (!(s > 0.0) || !isfinite(s)) { free(L); free(Li); return ORC_NOT_SPD; }
        double ljj = sqrt(s);
        L[(size_t)j * d + j] = ljj;
        for (int i = j + 1; i < d; ++i) {
            double t = H[(size_t)i * d + j];
            for (int k = 0; k < j; ++k) t -= L[(size_t)i * d + k] * L[(size_t)j * d + k];
            L[(size_t)i * d + j] = t / ljj;
        }
    }
    /* Li = L^-1 (lower triangular), column by column by forward substitution */
    for (int c = 0; c < d; ++c) {
        Li[(size_t)c * d + c] = 1.0 / L[(size_t)c * d + c];
        for (int i = c + 1; i < d; ++i) {
            double t = 0.0;
            for (int k = c; k < i; ++k) t -= L[(size_t)i * d + k] * Li[(size_t)k * d + c];
            Li[(size_t)i * d + c] = t / L[(size_t)i * d + i];
        }
    }
    /* H^-1 = L^-T L^-1 : entry (i,j) = sum_k Li[k][i] * Li[k][j], k >= max(i,j) */
    for (int i = 0; i < d; ++i) {
        for (int j = 0; j <= i; ++j) {
            double t = 0.0;
            for (int k = i; k < d; ++k) t += Li[(size_t)k * d + i] * Li[(size_t)k * d + j];
            H[(size_t)i * d + j] = t;
            H[(size_t)j * d + i] = t;
        }
    }
    free(L);
    free(Li);
    return ORC_OK;
}

/* Quantizer of Sec. 5 on a uniform grid of width delta starting at offset. */
static int orc_code(double w, double delta, double offset, int maxq)
{
    double c = nearbyint((w - offset) / delta); /* default rounding mode: half to even */
    if (c < 0.0) c = 0.0;
    if (c > (double)maxq) c = (double)maxq;
    return (int)c;
}

int orc_quant_code(double w, double delta, double offset, int maxq)
{
    return orc_code(w, delta, offset, maxq);
}

/* ---------------------------------------------------------------------------
 * One row of Algorithm 1 (mode 0, pruning) or Algorithm 3 (mode 1, OBQ).
 *
 *   Hinv     d x d row-major inverse Hessian, not modified
 *   w_in     the row's d weights, not modified
 *   k_steps  number of greedy steps (<= d; N:M: <= d (M-N)/M)
 *   nm_n/m   N:M pattern for pruning; nm_m == 0 means unstructured
 *   outlier  mode 1 only: non-zero switches on the outlier heuristic of Sec. 5
 *   delta, offset, maxq  the row's quantization grid (mode 1)
 *   forced   nullable: take p = forced[t] at step t instead of the argmin
 *            (used to replay another implementation's order); scores are still
 *            reported so that the caller can judge the forced pick
 *   order    out, k_steps: chosen index per step
 *   loss     out, k_steps: (target - w_p)^2 / (2 A_pp)
 *   codes    out, d, nullable (mode 1): grid code of each chosen weight at the
 *            moment it was chosen; -1 for weights never chosen
 *   w_out    out, d: the row after the last step
 *   trace    out, nullable, k_steps x d: the row after every step
 *   min_score / pick_score  out, nullable, k_steps: smallest eligible score
 *            in this state / the score of the index actually taken
 *   pre_round out, nullable, k_steps (mode 1): (w_p - offset)/delta before rounding
 *   A        scratch d x d; on return holds the reduced inverse (valid only on
 *            still-live rows and columns)
 *   live     scratch d bytes; on return 1 for indices never chosen
 * ------------------------------------------------------------------------- */
int orc_row_solve(int mode, const double *Hinv, int d, const double *w_in, int k_steps,
                  int nm_n, int nm_m, int outlier, double delta, double offset, int maxq,
                  const int32_t *forced, int32_t *order, double *loss, int32_t *codes,
                  double *w_out, double *trace, double *min_score, double *pick_score,
                  double *pre_round, double *A, uint8_t *live)
{
    if (!Hinv || !w_in || !order || !loss || !w_out || !A || !live) return ORC_BAD_ARG;
    if (d <= 0 || k_steps < 0 || k_steps > d) return ORC_BAD_ARG;
    if (mode != 0 && mode != 1) return ORC_BAD_ARG;
    int use_nm = (mode == 0 && nm_m > 0);
    if (use_nm && (nm_n < 0 || nm_n > nm_m || d % nm_m != 0)) return ORC_BAD_ARG;
    if (use_nm && (long)k_steps > (long)(d / nm_m) * (nm_m - nm_n)) return ORC_BAD_ARG;
    if (mode == 1 && (!(delta > 0.0) || maxq < 0)) return ORC_BAD_ARG;

    memcpy(A, Hinv, (size_t)d * d * sizeof(double));
    double *w = w_out;
    memcpy(w, w_in, (size_t)d * sizeof(double));
    for (int j = 0; j < d; ++j) live[j] = 1;
    if (codes) for (int j = 0; j < d; ++j) codes[j] = -1;
    int *blk_pruned = NULL;
    if (use_nm) blk_pruned = (int *)calloc((size_t)(d / nm_m), sizeof(int));

    int rc = ORC_OK;
    for (int t = 0; t < k_steps; ++t) {
        /* outlier heuristic: are there live weights whose quantization error exceeds delta / 2 ? */
        int any_outlier = 0;
        if (mode == 1 && outlier) {
            for (int j = 0; j < d && !any_outlier; ++j) {
                if (!live[j]) continue;
                double e = offset + delta * orc_code(w[j], delta, offset, maxq) - w[j];
                if (fabs(e) > 0.5 * delta) any_outlier = 1;
            }
        }
        /* selection: argmin over the live, eligible set */
        int best = -1;
        double best_s = 0.0;
        for (int j = 0; j < d; ++j) {
            if (!live[j]) continue;
            if (use_nm && blk_pruned[j / nm_m] >= nm_m - nm_n) continue;
            double target = (mode == 0) ? 0.0 : offset + delta * orc_code(w[j], delta, offset, maxq);
            double e = target - w[j];
            if (any_outlier && !(fabs(e) > 0.5 * delta)) continue;
            double s = e * e / A[(size_t)j * d + j];
            if (best < 0 || s < best_s) { best = j; best_s = s; }
        }
        if (best < 0) { rc = ORC_BAD_ARG; break; }
        int p = best;
        if (forced) {
            p = forced[t];
            if (p < 0 || p >= d || !live[p]) { rc = ORC_BAD_ARG; break; }
        }
        double app = A[(size_t)p * d + p];
        if (!(app > 0.0) || !isfinite(app)) { rc = ORC_NUMERIC; break; }
        int code = 0;
        double target = 0.0;
        if (mode == 1) {
            code = orc_code(w[p], delta, offset, maxq);
            target = offset + delta * code;
            if (pre_round) pre_round[t] = (w[p] - offset) / delta;
        }
        double e = target - w[p];
        if (min_score) min_score[t] = best_s;
        if (pick_score) pick_score[t] = e * e / app;
        order[t] = p;
        loss[t] = e * e / (2.0 * app);
        if (codes && mode == 1) codes[p] = code;

        /* compensation: w <- w - A[:,p] (w_p - target) / A_pp on the live set */
        double g = (w[p] - target) / app;
        for (int j = 0; j < d; ++j)
            if (live[j] && j != p) w[j] -= A[(size_t)j * d + p] * g;
        w[p] = target;

        /* Lemma 1: remove p from the inverse (live rows and columns only) */
        for (int i = 0; i < d; ++i) {
            if (!live[i] || i == p) continue;
            double f = A[(size_t)i * d + p] / app;
            for (int j = 0; j < d; ++j) {
                if (!live[j] || j == p) continue;
                A[(size_t)i * d + j] -= f * A[(size_t)p * d + j];
            }
        }
        live[p] = 0;
        if (use_nm) blk_pruned[p / nm_m] += 1;
        if (trace) memcpy(trace + (size_t)t * d, w, (size_t)d * sizeof(double));
    }
    free(blk_pruned);
    return rc;
}

/* Solve the c x c symmetric positive definite system M z = b by Gaussian elimination without
 * pivoting (M, b are overwritten; z returned in b).  Returns 0, or ORC_NUMERIC on a bad pivot. */
static int orc_small_solve(double *M, double *b, int c)
{
    for (int k = 0; k < c; ++k) {
        double piv = M[k * c + k];
        if (!(piv > 0.0) || !isfinite(piv)) return ORC_NUMERIC;
        for (int i = k + 1; i < c; ++i) {
            double f = M[i * c + k] / piv;
            for (int j = k; j < c; ++j) M[i * c + j] -= f * M[k * c + j];
            b[i] -= f * b[k];
        }
    }
    for (int k = c - 1; k >= 0; --k) {
        double v = b[k];
        for (int j = k + 1; j < c; ++j) v -= M[k * c + j] * b[j];
        b[k] = v / M[k * c + k];
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------------
 * One row of the block-pruning variant (Sec. 4 "Block-Sparsity", eq. (5)): Algorithm 1 on
 * blocks P of c consecutive indices (block b = indices b c .. b c + c - 1; d must be a
 * multiple of c).  Per step: the live block with the smallest w_P^T ((H^-1)_P)^-1 w_P is
 * chosen (ties to the lowest block), all weights move by -H^-1[:,P] ((H^-1)_P)^-1 w_P (the
 * block itself to exactly zero), and the block's indices are removed from the inverse one
 * after another with Lemma 1, in ascending order.
 *
 *   c         block size (1 <= c <= 16); c = 1 is Algorithm 1
 *   k_blocks  number of steps (<= d / c)
 *   forced    nullable: block index to take at each step
 *   order     out, k_blocks: chosen block per step
 *   loss      out, k_blocks: w_P^T ((H^-1)_P)^-1 w_P / 2 (the 1/2 as for single weights)
 *   w_out     out, d;  trace out, nullable, k_blocks x d
 *   min_score / pick_score out, nullable, k_blocks (scores without the 1/2)
 *   A         scratch d x d;  live scratch d bytes
 * ------------------------------------------------------------------------- */
int orc_block_row_solve(const double *Hinv, int d, const double *w_in, int c, int k_blocks,
                        const int32_t *forced, int32_t *order, double *loss, double *w_out,
                        double *trace, double *min_score, double *pick_score, double *A,
                        uint8_t *live)
{
    if (!Hinv || !w_in || !order || !loss || !w_out || !A || !live) return ORC_BAD_ARG;
    if (d <= 0 || c < 1 || c > 16 || d % c != 0) return ORC_BAD_ARG;
    int nb = d / c;
    if (k_blocks < 0 || k_blocks > nb) return ORC_BAD_ARG;
    double *w = w_out;
    memcpy(A, Hinv, (size_t)d * d * sizeof(double));
    memcpy(w, w_in, (size_t)d * sizeof(double));
    for (int j = 0; j < d; ++j) live[j] = 1;
    double M[16 * 16], z[16];

    for (int t = 0; t < k_blocks; ++t) {
        int best = -1;
        double best_s = 0.0;
        for (int b = 0; b < nb; ++b) {
            if (!live[b * c]) continue;
            for (int i = 0; i < c; ++i) {
                for (int j = 0; j < c; ++j) M[i * c + j] = A[(size_t)(b * c + i) * d + (b * c + j)];
                z[i] = w[b * c + i];
            }
            if (orc_small_solve(M, z, c) != ORC_OK) return ORC_NUMERIC;
            double s = 0.0;
            for (int i = 0; i < c; ++i) s += w[b * c + i] * z[i];
            if (best < 0 || s < best_s) { best = b; best_s = s; }
        }
        if (best < 0) return ORC_BAD_ARG;
        int bp = best;
        if (forced) {
            bp = forced[t];
            if (bp < 0 || bp >= nb || !live[bp * c]) return ORC_BAD_ARG;
        }
        /* z = ((H^-1)_P)^-1 w_P for the block taken */
        for (int i = 0; i < c; ++i) {
            for (int j = 0; j < c; ++j) M[i * c + j] = A[(size_t)(bp * c + i) * d + (bp * c + j)];
            z[i] = w[bp * c + i];
        }
        if (orc_small_solve(M, z, c) != ORC_OK) return ORC_NUMERIC;
        double s = 0.0;
        for (int i = 0; i < c; ++i) s += w[bp * c + i] * z[i];
        if (min_score) min_score[t] = best_s;
        if (pick_score) pick_score[t] = s;
        order[t] = bp;
        loss[t] = 0.5 * s;

        /* weight update: w <- w - H^-1[:,P] z on the live set, the block itself to zero */
        for (int j = 0; j < d; ++j) {
            if (!live[j]) continue;
            double dj = 0.0;
            for (int i = 0; i < c; ++i) dj += A[(size_t)j * d + (bp * c + i)] * z[i];
            w[j] -= dj;
        }
        for (int i = 0; i < c; ++i) w[bp * c + i] = 0.0;

        /* Lemma 1 for every index of the block, one after another */
        for (int q = 0; q < c; ++q) {
            int p = bp * c + q;
            double app = A[(size_t)p * d + p];
            if (!(app > 0.0) || !isfinite(app)) return ORC_NUMERIC;
            for (int i = 0; i < d; ++i) {
                if (!live[i] || i == p) continue;
                double f = A[(size_t)i * d + p] / app;
                for (int j = 0; j < d; ++j) {
                    if (!live[j] || j == p) continue;
                    A[(size_t)i * d + j] -= f * A[(size_t)p * d + j];
                }
            }
            live[p] = 0;
        }
        if (trace) memcpy(trace + (size_t)t * d, w, (size_t)d * sizeof(double));
    }
    return ORC_OK;
}

/* Several rows of the block variant over OpenMP threads (arrays stacked along R). */
int orc_block_rows_solve(const double *Hinv, int R, int d, const double *W, int c, int k_blocks,
                         int32_t *order, double *loss, double *W_out, int n_threads, int *threads_used)
{
    if (R < 0 || d <= 0) return ORC_BAD_ARG;
    int rc_all = ORC_OK;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel
    {
        double *A = (double *)malloc((size_t)d * d * sizeof(double));
        uint8_t *live = (uint8_t *)malloc((size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < R; ++i) {
            int rc = (A && live) ? orc_block_row_solve(Hinv, d, W + (size_t)i * d, c, k_blocks, NULL,
                                                       order + (size_t)i * k_blocks,
                                                       loss + (size_t)i * k_blocks, W_out + (size_t)i * d,
                                                       NULL, NULL, NULL, A, live)
                                : ORC_BAD_ARG;
            if (rc != ORC_OK) {
#pragma omp critical
                if (rc_all == ORC_OK) rc_all = rc;
            }
        }
        free(A);
        free(live);
    }
    if (threads_used) *threads_used = used;
    return rc_all;
}

/* ---------------------------------------------------------------------------
 * Several rows with the same inverse Hessian, spread over OpenMP threads.
 * Arrays are the per-row arrays of orc_row_solve stacked along a leading
 * dimension R (order/loss: R x k_steps, codes/w: R x d, trace: R x k_steps x d).
 * delta/offset are per-row arrays in mode 1 (ignored in mode 0).
 * Returns the first non-zero row status, and the number of threads used in
 * *threads_used.
 * ------------------------------------------------------------------------- */
int orc_rows_solve(int mode, const double *Hinv, int R, int d, const double *W, int k_steps,
                   int nm_n, int nm_m, int outlier, const double *delta, const double *offset, int maxq,
                   int32_t *order, double *loss, int32_t *codes, double *W_out, double *trace,
                   int n_threads, int *threads_used)
{
    if (R < 0 || d <= 0) return ORC_BAD_ARG;
    int rc_all = ORC_OK;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel
    {
        double *A = (double *)malloc((size_t)d * d * sizeof(double));
        uint8_t *live = (uint8_t *)malloc((size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < R; ++i) {
            int rc = (A && live) ? orc_row_solve(
                mode, Hinv, d, W + (size_t)i * d, k_steps, nm_n, nm_m, outlier,
                mode == 1 ? delta[i] : 1.0, mode == 1 ? offset[i] : 0.0, maxq, NULL,
                order + (size_t)i * k_steps, loss + (size_t)i * k_steps,
                codes ? codes + (size_t)i * d : NULL, W_out + (size_t)i * d,
                trace ? trace + (size_t)i * k_steps * d : NULL, NULL, NULL, NULL, A, live)
                                : ORC_BAD_ARG;
            if (rc != ORC_OK) {
#pragma omp critical
                if (rc_all == ORC_OK) rc_all = rc;
            }
        }
        free(A);
        free(live);
    }
    if (threads_used) *threads_used = used;
    return rc_all;
}

/* ---------------------------------------------------------------------------
 * Appendix Algorithm 2: from the per-row loss traces L (R x d, row i holds the
 * loss changes of row i in the order its weights were pruned) find how many
 * weights each row gives up when k weights are pruned from the whole layer.
 * The frontier holds one entry (row, count) per row; k times the row whose
 * next loss change is smallest advances by one (an exhausted row counts as
 * +infinity).  Ties go to the lowest row index.
 * ------------------------------------------------------------------------- */
int orc_global_select(const double *L, int R, int d, int64_t k, int32_t *counts)
{
    if (!L || !counts || R <= 0 || d <= 0 || k < 0 || k > (int64_t)R * d) return ORC_BAD_ARG;
    for (int i = 0; i < R; ++i) counts[i] = 0;
    for (int64_t step = 0; step < k; ++step) {
        int best = -1;
        double best_v = 0.0;
        for (int i = 0; i < R; ++i) {
            if (counts[i] >= d) continue; /* infinity */
            double v = L[(size_t)i * d + counts[i]];
            if (best < 0 || v < best_v) { best = i; best_v = v; }
        }
        if (best < 0) return ORC_BAD_ARG;
        counts[best] += 1;
    }
    return ORC_OK;
}
