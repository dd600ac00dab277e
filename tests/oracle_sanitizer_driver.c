/* Host sanitizer run of the oracle (test infrastructure): every entry point on small random inputs, linked with
 * oracle/laa_oracle.c under -fsanitize=address,undefined by tests/test_oracle_sanitizers.py.  Checks memory safety
 * and undefined behaviour only; what the oracle computes is pinned elsewhere. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
typedef double real;
typedef struct ora_ctx ora_ctx;
ora_ctx *ora_create(int64_t, int32_t, int32_t, double, double, double);
void ora_destroy(ora_ctx *);
int ora_set_columns(ora_ctx *, const int64_t *);
int ora_set_warmup(ora_ctx *, int64_t);
int ora_init_state(ora_ctx *, const real *);
int ora_local_step_dense(ora_ctx *, const real *);
int ora_sync(ora_ctx *);
int ora_set_generator(ora_ctx *, int, uint64_t, const real *, const real *, const real *, int, double, double);
int ora_gradient(const ora_ctx *, int64_t, real *);
int ora_local_step_gen(ora_ctx *);
int ora_local_step_sparse(ora_ctx *, const int32_t *, const real *, int32_t, int32_t);
int64_t ora_dirty_rows(const ora_ctx *, int32_t *, int64_t);
int ora_diagnostics(const ora_ctx *, double out[3]);
int ora_step_dense(ora_ctx *, const real *);
int ora_step_gen(ora_ctx *);
int ora_step_sparse(ora_ctx *, const int32_t *, const real *, int32_t, int32_t);
int ora_adagrad_step_dense(ora_ctx *, const real *);
int ora_localsgd_step_dense(ora_ctx *, const real *);
static double rnd(void) { return (double)rand() / RAND_MAX - 0.5; }
int main(void)
{
    for (int trial = 0; trial < 20; ++trial) {
        const int W = 1 + rand() % 5, H = 1 + rand() % 4, rows = 1 + rand() % 9, row_len = 4 * (1 + rand() % 3);
        const int64_t d = (int64_t)rows * row_len;
        ora_ctx *c = ora_create(d, W, H, 0.5, 1.0, 1.0);
        real *x0 = malloc(sizeof(real) * d), *a = malloc(sizeof(real) * d), *xs = malloc(sizeof(real) * d);
        real *off = malloc(sizeof(real) * W * d), *G = malloc(sizeof(real) * W * d);
        int64_t *col = malloc(sizeof(int64_t) * d);
        for (int64_t j = 0; j < d; ++j) { x0[j] = rnd(); a[j] = 1 + rnd(); xs[j] = rnd(); col[j] = 7 * j + ((int64_t)1 << 34); }
        for (int64_t j = 0; j < W * d; ++j) off[j] = rnd();
        if (trial & 1) ora_set_columns(c, col);
        if (trial & 2) ora_set_warmup(c, 5);
        ora_init_state(c, trial & 4 ? x0 : NULL);
        ora_set_generator(c, 1, 42, a, xs, off, trial % 3, 0.1, 0.1);
        for (int t = 0; t < 3 * H + 1; ++t) {
            for (int64_t j = 0; j < W * d; ++j) G[j] = rnd();
            const int k = rand() % (rows + 1);
            int32_t *idx = malloc(sizeof(int32_t) * W * (k ? k : 1));
            real *vals = malloc(sizeof(real) * W * (k ? k : 1) * row_len);
            for (int i = 0; i < W * k; ++i) idx[i] = rand() % rows;
            for (int i = 0; i < W * k * row_len; ++i) vals[i] = rnd();
            switch (rand() % 5) {
            case 0: ora_step_dense(c, G); break;
            case 1: ora_step_gen(c); break;
            case 2: ora_step_sparse(c, idx, vals, k, row_len); break;
            case 3: if (ora_local_step_gen(c) != 0) ora_sync(c); break;
            default: if (ora_local_step_sparse(c, idx, vals, k, row_len) != 0) ora_sync(c); break;
            }
            int32_t list[16]; ora_dirty_rows(c, list, 16);
            double dg[3]; ora_diagnostics(c, dg);
            ora_gradient(c, t + 1, G);
            free(idx); free(vals);
        }
        ora_sync(c);
        ora_destroy(c);
        c = ora_create(d, W, 1, 0.3, 0.1, 0.0);
        ora_init_state(c, x0);
        for (int64_t j = 0; j < W * d; ++j) G[j] = rnd();
        ora_adagrad_step_dense(c, G); ora_localsgd_step_dense(c, G);
        ora_destroy(c);
        free(x0); free(a); free(xs); free(off); free(G); free(col);
    }
    puts("oracle sanitizer run: ok");
    return 0;
}
