/* Driver for a sanitizer build (-fsanitize=address,undefined) of the CPU oracle: calls every
 * exported function on small problems whose buffers are heap blocks of exactly the documented
 * sizes, so that any read or write beyond them, and any undefined arithmetic, stops the run.
 * Values are not checked here (the pins do that); exit status 0 = clean run. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int orc_spd_inverse(double *H, int d);
int orc_quant_code(double w, double delta, double offset, int maxq);
int orc_row_solve(int mode, const double *Hinv, int d, const double *w_in, int k_steps, int nm_n, int nm_m,
                  int outlier, double delta, double offset, int maxq, const int32_t *forced, int32_t *order,
                  double *loss, int32_t *codes, double *w_out, double *trace, double *min_score,
                  double *pick_score, double *pre_round, double *A, uint8_t *live);
int orc_block_row_solve(const double *Hinv, int d, const double *w_in, int c, int k_blocks, const int32_t *forced,
                        int32_t *order, double *loss, double *w_out, double *trace, double *min_score,
                        double *pick_score, double *A, uint8_t *live);
int orc_block_rows_solve(const double *Hinv, int R, int d, const double *W, int c, int k_blocks, int32_t *order,
                         double *loss, double *W_out, int n_threads, int *threads_used);
int orc_rows_solve(int mode, const double *Hinv, int R, int d, const double *W, int k_steps, int nm_n, int nm_m,
                   int outlier, const double *delta, const double *offset, int maxq, int32_t *order, double *loss,
                   int32_t *codes, double *W_out, double *trace, int n_threads, int *threads_used);
int orc_global_select(const double *L, int R, int d, int64_t k, int32_t *counts);

static unsigned long long rng_state = 88172645463325252ull;
static double rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 - 0.5;
}

#define NEW(type, n) ((type *)malloc(sizeof(type) * (size_t)((n) > 0 ? (n) : 1)))
#define CHECK(call) do { int rc__ = (call); if (rc__ != 0) { fprintf(stderr, "%s -> %d\n", #call, rc__); return 1; } } while (0)

static int one_size(int d, int R, int c)
{
    const int n = 3 * d;
    double *X = NEW(double, d * n), *H = NEW(double, d * d), *W = NEW(double, R * d);
    for (int i = 0; i < d * n; ++i) X[i] = rnd();
    for (int i = 0; i < R * d; ++i) W[i] = 0.2 * rnd();
    for (int i = 0; i < d; ++i)
        for (int j = 0; j < d; ++j) {
            double s = 0.0;
            for (int t = 0; t < n; ++t) s += X[i * n + t] * X[j * n + t];
            H[i * d + j] = 2.0 * s + (i == j ? 0.05 : 0.0);
        }
    CHECK(orc_spd_inverse(H, d));
    /* one row: pruning with trace and diagnostics, N:M, OBQ with and without the outlier rule, forced order */
    int32_t *order = NEW(int32_t, d), *codes = NEW(int32_t, d), *forced = NEW(int32_t, d);
    double *loss = NEW(double, d), *w_out = NEW(double, d), *trace = NEW(double, d * d), *mins = NEW(double, d);
    double *pick = NEW(double, d), *pre = NEW(double, d), *A = NEW(double, d * d);
    uint8_t *live = NEW(uint8_t, d);
    CHECK(orc_row_solve(0, H, d, W, d, 0, 0, 0, 1.0, 0.0, 0, NULL, order, loss, NULL, w_out, trace, mins, pick, NULL, A, live));
    memcpy(forced, order, sizeof(int32_t) * (size_t)d);
    CHECK(orc_row_solve(0, H, d, W, d / 2, 0, 0, 0, 1.0, 0.0, 0, forced, order, loss, NULL, w_out, NULL, mins, pick, NULL, A, live));
    if (d % 4 == 0)
        CHECK(orc_row_solve(0, H, d, W, d / 2, 2, 4, 0, 1.0, 0.0, 0, NULL, order, loss, NULL, w_out, trace, NULL, NULL, NULL, A, live));
    CHECK(orc_row_solve(1, H, d, W, d, 0, 0, 0, 0.013, -0.1, 15, NULL, order, loss, codes, w_out, trace, mins, pick, pre, A, live));
    CHECK(orc_row_solve(1, H, d, W, d, 0, 0, 1, 0.004, -0.03, 7, NULL, order, loss, codes, w_out, NULL, NULL, NULL, NULL, A, live));
    CHECK(orc_row_solve(0, H, d, W, 0, 0, 0, 0, 1.0, 0.0, 0, NULL, order, loss, NULL, w_out, NULL, NULL, NULL, NULL, A, live));
    if (d % c == 0) {
        CHECK(orc_block_row_solve(H, d, W, c, d / c, NULL, order, loss, w_out, trace, mins, pick, A, live));
        memcpy(forced, order, sizeof(int32_t) * (size_t)(d / c));
        CHECK(orc_block_row_solve(H, d, W, c, d / c / 2, forced, order, loss, w_out, NULL, NULL, NULL, A, live));
    }
    /* several rows over threads */
    int32_t *orders = NEW(int32_t, R * d), *codes2 = NEW(int32_t, R * d), *counts = NEW(int32_t, R);
    double *losses = NEW(double, R * d), *W_out = NEW(double, R * d), *traces = NEW(double, R * d * d);
    double *delta = NEW(double, R), *offset = NEW(double, R);
    for (int i = 0; i < R; ++i) { delta[i] = 0.01 + 0.001 * i; offset[i] = -0.1; }
    int used = 0;
    CHECK(orc_rows_solve(0, H, R, d, W, d, 0, 0, 0, NULL, NULL, 0, orders, losses, NULL, W_out, traces, 3, &used));
    CHECK(orc_global_select(losses, R, d, (int64_t)R * d / 2, counts));
    CHECK(orc_global_select(losses, R, d, 0, counts));
    CHECK(orc_global_select(losses, R, d, (int64_t)R * d, counts));
    CHECK(orc_rows_solve(1, H, R, d, W, d, 0, 0, 0, delta, offset, 15, orders, losses, codes2, W_out, NULL, 0, &used));
    if (d % c == 0) CHECK(orc_block_rows_solve(H, R, d, W, c, d / c, orders, losses, W_out, 2, &used));
    /* error paths must not touch anything */
    if (orc_spd_inverse(NULL, d) == 0 || orc_global_select(losses, R, d, (int64_t)R * d + 1, counts) == 0) return 1;
    double bad[4] = {1.0, 2.0, 2.0, 1.0};
    if (orc_spd_inverse(bad, 2) == 0) return 1;
    free(X); free(H); free(W); free(order); free(codes); free(forced); free(loss); free(w_out); free(trace);
    free(mins); free(pick); free(pre); free(A); free(live); free(orders); free(codes2); free(counts);
    free(losses); free(W_out); free(traces); free(delta); free(offset);
    return 0;
}

int main(void)
{
    if (orc_quant_code(0.26, 0.1, 0.0, 15) != 3 || orc_quant_code(0.25, 0.1, -0.1, 15) < 0) return 1;
    if (orc_quant_code(99.0, 0.1, 0.0, 15) != 15 || orc_quant_code(-99.0, 0.1, 0.0, 15) != 0) return 1;
    if (one_size(1, 1, 1) || one_size(7, 3, 1) || one_size(12, 4, 4) || one_size(33, 2, 3) || one_size(40, 5, 8)) return 1;
    puts("oracle sanitizer run clean");
    return 0;
}
