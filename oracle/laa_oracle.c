/*
 * Local AdaAlter — reference oracle (TEST INFRASTRUCTURE, not the product).
 *
 * A plain, single-threaded, obviously-correct CPU implementation of what the
 * GPU library computes, written from the paper (arXiv 1911.09030).  Only the
 * tests, the smoke check and the benchmark's CPU-baseline leg may call it; the
 * product path never does, and the two share no code.
 *
 * Arithmetic type: `real`, double by default (the paper fixes no precision, so
 * the oracle is the exact method up to fp64 rounding).  Compiling with
 * -DORA_REAL=float gives the same statements in fp32; that build is used only
 * to measure how far a straightforward fp32 evaluation drifts from the fp64
 * one, which is what the GPU tolerance is derived from.
 *
 * What follows the paper, statement by statement:
 *   - state and initialisation ........ Algorithm 3, "Initialize" line
 *   - t' ............................... Algorithm 3, first line of the loop body
 *   - parameter update y ............... Algorithm 3, update with the lazily
 *                                        updated denominator B^2_{i,t-t'} + t' eps^2
 *   - accumulator update A^2 ........... Algorithm 3, second half of the same line
 *   - synchronisation .................. Algorithm 3, "Synchronize" branch
 *   - lazy denominator (one value shared by all workers between syncs)
 *                                        Section 4.2, "Lazy update of the denominators"
 *   - warm-up learning rate ............ Section 6.2, "Warm-up Learning Rates"
 *   - Distributed AdaGrad .............. Algorithm 1
 *   - Local SGD ........................ Algorithm 2
 *
 * The synthetic gradient (a stand-in for the stochastic gradient of Algorithm 3
 * evaluated at the worker's own iterate) is not the paper's; it is specified in
 * the comment above ora_gradient() and implemented independently on the GPU.
 *
 * Pins (tests/test_oracle_pins.py): H=1 reduction, W=1 reduction, closed-form
 * constant-gradient trajectory, the Notation-table definition of B^2_t, a
 * literal full-history evaluation of Algorithm 3 in 50-digit decimal arithmetic
 * on tiny inputs, Philox known-answer vectors, normal-sample statistics, and
 * planted-mistake builds (ORA_PLANT_*) that each must fail a pin.
 * Unpinned: nothing in the method.  The statistical quality of the synthetic
 * gradient beyond the moments/KS checks is the workload's, not the paper's.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORA_REAL
#define ORA_REAL double
#endif
typedef ORA_REAL real;

#define ORA_OK 0
#define ORA_EINVAL (-1)
#define ORA_ESYNCDUE (-3)
#define ORA_EMODE (-5)

enum { ORA_GEN_NONE = 0, ORA_GEN_QUADRATIC = 1, ORA_GEN_NOISE = 2 };
enum { ORA_OFF_NONE = 0, ORA_OFF_ARRAY = 1, ORA_OFF_PHILOX = 2 };
enum { ORA_STREAM_OFFSET = 2, ORA_STREAM_NOISE = 3 };

typedef struct ora_ctx {
    int64_t d;
    int32_t W, H;
    real eta, eps2, b0sq;
    real *x;      /* [W][d]  x_{i,t}: each worker's parameters                       */
    real *acc;    /* [W][d]  B^2_{i,t}: each worker's running accumulator            */
    real *snap;   /* [d]     B^2_{i,t-t'}: accumulator as of the last sync (same on all i) */
    int64_t *col; /* [d]     absolute coordinate of local column (generator counters) */
    int32_t s;    /* local steps taken since the last synchronisation (= t'-1 before a step) */
    int64_t t;    /* iterations done                                                  */
    int64_t warmup_steps; /* 0 = constant eta                                         */
    /* synthetic gradient */
    int gen_mode, off_mode;
    uint64_t seed;
    real *a, *xstar, *off; /* [d], [d], [W][d] (own copies) */
    real noise_scale, off_scale;
    /* sparse bookkeeping: rows touched since last sync */
    uint8_t *dirty;
    int64_t n_rows;
    real *G; /* scratch gradient [W][d] */
} ora_ctx;

int ora_real_bytes(void) { return (int)sizeof(real); }

ora_ctx *ora_create(int64_t d, int32_t W, int32_t H, double eta, double eps, double b0)
{
    if (d <= 0 || W <= 0 || H <= 0 || !(eps >= 0.0) || !isfinite(eta) || !(b0 >= 0.0)) return NULL;
    ora_ctx *c = (ora_ctx *)calloc(1, sizeof(ora_ctx));
    if (!c) return NULL;
    c->d = d; c->W = W; c->H = H;
    c->eta = (real)eta;
    c->eps2 = (real)(eps * eps);
    c->b0sq = (real)(b0 * b0);
    size_t n = (size_t)W * (size_t)d;
    c->x = (real *)malloc(n * sizeof(real));
    c->acc = (real *)malloc(n * sizeof(real));
    c->G = (real *)malloc(n * sizeof(real));
    c->snap = (real *)malloc((size_t)d * sizeof(real));
    c->col = (int64_t *)malloc((size_t)d * sizeof(int64_t));
    if (!c->x || !c->acc || !c->G || !c->snap || !c->col) return NULL;
    for (int64_t j = 0; j < d; ++j) c->col[j] = j;
    /* Algorithm 3, Initialize: x_{i,0} = x_0 (zero until ora_init_state says otherwise), B^2_{i,0} = b0^2 */
    for (size_t k = 0; k < n; ++k) { c->x[k] = 0; c->acc[k] = c->b0sq; }
    for (int64_t j = 0; j < d; ++j) c->snap[j] = c->b0sq;
    return c;
}

void ora_destroy(ora_ctx *c)
{
    if (!c) return;
    free(c->x); free(c->acc); free(c->snap); free(c->col); free(c->G);
    free(c->a); free(c->xstar); free(c->off); free(c->dirty);
    free(c);
}

int ora_set_columns(ora_ctx *c, const int64_t *col)
{
    if (!c || !col) return ORA_EINVAL;
    memcpy(c->col, col, (size_t)c->d * sizeof(int64_t));
    return ORA_OK;
}

int ora_set_warmup(ora_ctx *c, int64_t warmup_steps)
{
    if (!c || warmup_steps < 0) return ORA_EINVAL;
    c->warmup_steps = warmup_steps;
    return ORA_OK;
}

/* Algorithm 3, Initialize. */
int ora_init_state(ora_ctx *c, const real *x0)
{
    if (!c) return ORA_EINVAL;
    for (int32_t w = 0; w < c->W; ++w)
        for (int64_t j = 0; j < c->d; ++j) {
            c->x[(size_t)w * c->d + j] = x0 ? x0[j] : (real)0;
            c->acc[(size_t)w * c->d + j] = c->b0sq;
        }
    for (int64_t j = 0; j < c->d; ++j) c->snap[j] = c->b0sq;
    c->s = 0; c->t = 0;
    if (c->dirty) memset(c->dirty, 0, (size_t)c->n_rows);
    return ORA_OK;
}

/* Section 6.2: eta_t = eta * min(1, t / warm_up_steps), t the 1-based iteration. */
static real ora_eta_at(const ora_ctx *c, int64_t t)
{
    if (c->warmup_steps <= 0) return c->eta;
    real r = (real)t / (real)c->warmup_steps;
    return c->eta * (r < (real)1 ? r : (real)1);
}

/*
 * One local iteration of Algorithm 3 for every worker, given this iteration's
 * gradients G[w][j] (already evaluated at x_{w,t-1}).
 */
int ora_local_step_dense(ora_ctx *c, const real *G)
{
    if (!c || !G) return ORA_EINVAL;
    if (c->s >= c->H) return ORA_ESYNCDUE;
    const int64_t t = c->t + 1;              /* this iteration                          */
    const int32_t tp = c->s + 1;             /* t' = mod(t-1, H) + 1 when syncs are on time */
    const real eta = ora_eta_at(c, t);
    const real pad = (real)tp * c->eps2;     /* t' eps^2, the placeholder               */
    for (int32_t w = 0; w < c->W; ++w) {
        for (int64_t j = 0; j < c->d; ++j) {
            const size_t k = (size_t)w * c->d + j;
            const real g = G[k];
#if defined(ORA_PLANT_RUNNING_DENOM)
            const real den = sqrt(c->acc[k] + pad);              /* planted: B^2_{t-1} instead of B^2_{t-t'} */
#elif defined(ORA_PLANT_NO_SQRT)
            const real den = c->snap[j] + pad;                   /* planted: square root dropped */
#elif defined(ORA_PLANT_PAD_ONE)
            const real den = sqrt(c->snap[j] + c->eps2);         /* planted: eps^2 instead of t' eps^2 */
#elif defined(ORA_PLANT_PAD_OFF_BY_ONE)
            const real den = sqrt(c->snap[j] + (real)(tp - 1) * c->eps2); /* planted: (t'-1) eps^2 */
#else
            const real den = sqrt(c->snap[j] + pad);             /* sqrt(B^2_{i,t-t'} + t' eps^2) */
#endif
#if defined(ORA_PLANT_PLUS)
            c->x[k] = c->x[k] + eta * g / den;                   /* planted: wrong sign */
#else
            c->x[k] = c->x[k] - eta * g / den;                   /* y_{i,t} */
#endif
#if defined(ORA_PLANT_ACC_ABS)
            c->acc[k] = c->acc[k] + fabs(g);                     /* planted: |g| instead of g^2 */
#else
            c->acc[k] = c->acc[k] + g * g;                       /* A^2_{i,t} = B^2_{i,t-1} + G o G */
#endif
        }
    }
    c->s += 1; c->t += 1;
    return ORA_OK;
}

/*
 * Algorithm 3, Synchronize: every worker's x and B^2 become the mean over
 * workers of y and A^2; the value under the square root for the next period
 * is that mean B^2.
 */
int ora_sync(ora_ctx *c)
{
    if (!c) return ORA_EINVAL;
    if (c->s == 0) return ORA_OK;
    for (int64_t j = 0; j < c->d; ++j) {
        real sx = 0, sb = 0;
        for (int32_t w = 0; w < c->W; ++w) {
            sx += c->x[(size_t)w * c->d + j];
            sb += c->acc[(size_t)w * c->d + j];
        }
        const real mx = sx / (real)c->W;
#if defined(ORA_PLANT_SYNC_NO_ACC)
        (void)sb;
        for (int32_t w = 0; w < c->W; ++w) c->x[(size_t)w * c->d + j] = mx;
        c->snap[j] = c->acc[j];                                  /* planted: accumulators not averaged */
#else
        const real mb = sb / (real)c->W;
        for (int32_t w = 0; w < c->W; ++w) {
            c->x[(size_t)w * c->d + j] = mx;
            c->acc[(size_t)w * c->d + j] = mb;
        }
        c->snap[j] = mb;
#endif
    }
    c->s = 0;
    if (c->dirty) memset(c->dirty, 0, (size_t)c->n_rows);
    return ORA_OK;
}

/* ------------------------------------------------------------------------- */
/* Synthetic gradient.
 *
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter (c0..c3), key
 * (k0,k1); per round  hi0:lo0 = M0*c0, hi1:lo1 = M1*c2,
 * (c0,c1,c2,c3) <- (hi1^c1^k0, lo1, hi0^c3^k1, lo0), then k0 += W0, k1 += W1.
 *
 * One Philox call serves the four coordinates j = 4q .. 4q+3:
 *   counter = (q mod 2^32, worker, t mod 2^32, stream + (q >> 32) * 16), key = (seed lo, seed hi)
 *   u_i = ((r_i >> 9) + 0.5) * 2^-23      in (0,1), exactly representable in fp32
 *   Box-Muller: (n0,n1) = sqrt(-2 ln u0) * (cos 2 pi u1, sin 2 pi u1); (n2,n3) likewise from (u2,u3)
 * stream 3 (noise) uses the iteration number t >= 1; stream 2 (per-worker
 * offset of the optimum) uses t = 0.
 *
 *   quadratic:  g = a_j * (x_{w,j} - (xstar_j + off_{w,j})) + noise_scale * n
 *   noise    :  g = a_j * n            (a_j plays the role of a per-coordinate sigma)
 */
void ora_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static real ora_uniform(uint32_t r) { return ((real)(r >> 9) + (real)0.5) * (real)(1.0 / 8388608.0); }

/* four standard normals for coordinates 4q..4q+3 of worker w at iteration t on a stream */
void ora_normals4(uint64_t seed, uint32_t stream, uint64_t q, uint32_t w, uint64_t t, real n[4])
{
    const double two_pi = 6.283185307179586476925286766559;
    uint32_t ctr[4] = { (uint32_t)q, w, (uint32_t)t, stream + (uint32_t)(q >> 32) * 16u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    ora_philox4x32_10(ctr, key, r);
    for (int p = 0; p < 2; ++p) {
        const real u0 = ora_uniform(r[2 * p]), u1 = ora_uniform(r[2 * p + 1]);
        const real rad = sqrt((real)-2 * log(u0));
        const real ang = (real)two_pi * u1;
#if defined(ORA_PLANT_SINCOS_SWAPPED)
        n[2 * p] = rad * sin(ang);                               /* planted */
        n[2 * p + 1] = rad * cos(ang);
#else
        n[2 * p] = rad * cos(ang);
        n[2 * p + 1] = rad * sin(ang);
#endif
    }
}

int ora_set_generator(ora_ctx *c, int mode, uint64_t seed, const real *a, const real *xstar,
                      const real *off, int off_mode, double noise_scale, double off_scale)
{
    if (!c || !a) return ORA_EINVAL;
    if (mode != ORA_GEN_QUADRATIC && mode != ORA_GEN_NOISE) return ORA_EINVAL;
    if (mode == ORA_GEN_QUADRATIC && !xstar) return ORA_EINVAL;
    if (off_mode == ORA_OFF_ARRAY && !off) return ORA_EINVAL;
    free(c->a); free(c->xstar); free(c->off);
    c->a = c->xstar = c->off = NULL;
    c->a = (real *)malloc((size_t)c->d * sizeof(real));
    memcpy(c->a, a, (size_t)c->d * sizeof(real));
    if (xstar) {
        c->xstar = (real *)malloc((size_t)c->d * sizeof(real));
        memcpy(c->xstar, xstar, (size_t)c->d * sizeof(real));
    }
    if (off_mode == ORA_OFF_ARRAY) {
        c->off = (real *)malloc((size_t)c->W * c->d * sizeof(real));
        memcpy(c->off, off, (size_t)c->W * c->d * sizeof(real));
    }
    c->gen_mode = mode; c->off_mode = off_mode; c->seed = seed;
    c->noise_scale = (real)noise_scale; c->off_scale = (real)off_scale;
    return ORA_OK;
}

/* G[w][j] for iteration t (1-based), evaluated at the current x (= x_{w,t-1}). */
int ora_gradient(const ora_ctx *c, int64_t t, real *G)
{
    if (!c || !G) return ORA_EINVAL;
    if (c->gen_mode == ORA_GEN_NONE) return ORA_EMODE;
    for (int32_t w = 0; w < c->W; ++w) {
        for (int64_t j = 0; j < c->d; ++j) {
            const size_t k = (size_t)w * c->d + j;
            const uint64_t ja = (uint64_t)c->col[j];
            real n[4];
            ora_normals4(c->seed, ORA_STREAM_NOISE, ja >> 2, (uint32_t)w, (uint64_t)t, n);
            const real nz = n[ja & 3];
            if (c->gen_mode == ORA_GEN_NOISE) {
                G[k] = c->a[j] * nz;
            } else {
                real o = 0;
                if (c->off_mode == ORA_OFF_ARRAY) o = c->off[k];
                else if (c->off_mode == ORA_OFF_PHILOX) {
                    real m[4];
                    ora_normals4(c->seed, ORA_STREAM_OFFSET, ja >> 2, (uint32_t)w, 0, m);
                    o = c->off_scale * m[ja & 3];
                }
#if defined(ORA_PLANT_GRAD_OFFSET_SIGN)
                G[k] = c->a[j] * (c->x[k] - (c->xstar[j] - o)) + c->noise_scale * nz; /* planted */
#else
                G[k] = c->a[j] * (c->x[k] - (c->xstar[j] + o)) + c->noise_scale * nz;
#endif
            }
        }
    }
    return ORA_OK;
}

int ora_local_step_gen(ora_ctx *c)
{
    if (!c) return ORA_EINVAL;
    if (c->gen_mode == ORA_GEN_NONE) return ORA_EMODE;
    if (c->s >= c->H) return ORA_ESYNCDUE;
    int rc = ora_gradient(c, c->t + 1, c->G);
    if (rc != ORA_OK) return rc;
    return ora_local_step_dense(c, c->G);
}

/*
 * Row-sparse gradient: the dense step applied to the gradient that is zero
 * outside the listed rows.  A zero gradient coordinate leaves y = x and
 * A^2 = B^2 in Algorithm 3, so nothing else is needed.  idx[w][k] are row
 * numbers, vals[w][k][row_len]; a row listed twice by one worker adds up.
 */
int ora_local_step_sparse(ora_ctx *c, const int32_t *idx, const real *vals, int32_t k, int32_t row_len)
{
    if (!c || k < 0 || row_len <= 0 || c->d % row_len != 0) return ORA_EINVAL;
    if (k > 0 && (!idx || !vals)) return ORA_EINVAL;
    if (c->s >= c->H) return ORA_ESYNCDUE;
    const int64_t n_rows = c->d / row_len;
    if (!c->dirty || c->n_rows != n_rows) {
        free(c->dirty);
        c->dirty = (uint8_t *)calloc((size_t)n_rows, 1);
        c->n_rows = n_rows;
    }
    for (int32_t w = 0; w < c->W; ++w)
        for (int32_t i = 0; i < k; ++i) {
            const int32_t r = idx[(size_t)w * k + i];
            if (r < 0 || r >= n_rows) return ORA_EINVAL;
        }
    memset(c->G, 0, (size_t)c->W * c->d * sizeof(real));
    for (int32_t w = 0; w < c->W; ++w)
        for (int32_t i = 0; i < k; ++i) {
            const int64_t r = idx[(size_t)w * k + i];
            for (int32_t e = 0; e < row_len; ++e)
#if defined(ORA_PLANT_SPARSE_LAST_WINS)
                c->G[(size_t)w * c->d + r * row_len + e] = vals[((size_t)w * k + i) * row_len + e];  /* planted */
#else
                c->G[(size_t)w * c->d + r * row_len + e] += vals[((size_t)w * k + i) * row_len + e];
#endif
            c->dirty[r] = 1;
        }
    return ora_local_step_dense(c, c->G);
}

/* rows touched by any worker since the last sync, ascending */
int64_t ora_dirty_rows(const ora_ctx *c, int32_t *out, int64_t cap)
{
    if (!c || !c->dirty) return 0;
    int64_t n = 0;
    for (int64_t r = 0; r < c->n_rows; ++r)
        if (c->dirty[r]) { if (out && n < cap) out[n] = (int32_t)r; ++n; }
    return n;
}

/* Diagnostics at the mean iterate xbar = (1/n) sum_i x_i (Section 5, auxiliary variable) for the quadratic
 * objective F(x) = (1/n) sum_i (1/2) sum_j a_j (x_j - xstar_j - off_ij)^2:
 *   out[0] = ||xbar - xstar||^2, out[1] = ||grad F(xbar)||^2, out[2] = (1/n) sum_i ||x_i - xbar||^2. */
int ora_diagnostics(const ora_ctx *c, double out[3])
{
    if (!c || !out) return ORA_EINVAL;
    if (c->gen_mode != ORA_GEN_QUADRATIC) return ORA_EMODE;
    double s0 = 0, s1 = 0, s2 = 0;
    for (int64_t j = 0; j < c->d; ++j) {
        double xbar = 0, moff = 0, dev = 0;
        for (int32_t w = 0; w < c->W; ++w) xbar += (double)c->x[(size_t)w * c->d + j];
        xbar /= (double)c->W;
        for (int32_t w = 0; w < c->W; ++w) {
            const double t = (double)c->x[(size_t)w * c->d + j] - xbar;
            dev += t * t;
            if (c->off_mode == ORA_OFF_ARRAY) moff += (double)c->off[(size_t)w * c->d + j];
            else if (c->off_mode == ORA_OFF_PHILOX) {
                real m[4];
                const uint64_t ja = (uint64_t)c->col[j];
                ora_normals4(c->seed, ORA_STREAM_OFFSET, ja >> 2, (uint32_t)w, 0, m);
                moff += (double)c->off_scale * (double)m[ja & 3];
            }
        }
        moff /= (double)c->W;
        const double dx = xbar - (double)c->xstar[j];
        const double g = (double)c->a[j] * (dx - moff);
        s0 += dx * dx; s1 += g * g; s2 += dev / (double)c->W;
    }
    out[0] = s0; out[1] = s1; out[2] = s2;
    return ORA_OK;
}

/* One whole iteration t of Algorithm 3: the local update, then the averaging when mod(t,H)=0. */
int ora_step_dense(ora_ctx *c, const real *G)
{
    int rc = ora_local_step_dense(c, G);
    if (rc == ORA_OK && c->s == c->H) rc = ora_sync(c);
    return rc;
}
int ora_step_gen(ora_ctx *c)
{
    int rc = ora_local_step_gen(c);
    if (rc == ORA_OK && c->s == c->H) rc = ora_sync(c);
    return rc;
}
int ora_step_sparse(ora_ctx *c, const int32_t *idx, const real *vals, int32_t k, int32_t row_len)
{
    int rc = ora_local_step_sparse(c, idx, vals, k, row_len);
    if (rc == ORA_OK && c->s == c->H) rc = ora_sync(c);
    return rc;
}

real *ora_x(ora_ctx *c) { return c->x; }
real *ora_acc(ora_ctx *c) { return c->acc; }
real *ora_snap(ora_ctx *c) { return c->snap; }
int64_t ora_t(const ora_ctx *c) { return c->t; }
int32_t ora_steps_since_sync(const ora_ctx *c) { return c->s; }

/* ------------------------------------------------------------------------- */
/* The paper's two comparison methods on the same state arrays (one shared
 * iterate for AdaGrad, kept in every worker's row so the layout is the same). */

/* Algorithm 1, Distributed AdaGrad: G = mean_i G_i; B^2 += G o G; x -= eta G / sqrt(B^2 + eps^2)
 * with the freshly updated B^2 and B^2_0 = 0 (the caller creates the context with b0 = 0). */
int ora_adagrad_step_dense(ora_ctx *c, const real *G)
{
    if (!c || !G) return ORA_EINVAL;
    const real eta = ora_eta_at(c, c->t + 1);
    for (int64_t j = 0; j < c->d; ++j) {
        real sg = 0;
        for (int32_t w = 0; w < c->W; ++w) sg += G[(size_t)w * c->d + j];
        const real g = sg / (real)c->W;
        const real b2 = c->snap[j] + g * g;
#if defined(ORA_PLANT_ADAGRAD_OLD_B2)
        const real xn = c->x[j] - eta * g / sqrt(c->snap[j] + c->eps2);  /* planted: B^2_{t-1} */
#else
        const real xn = c->x[j] - eta * g / sqrt(b2 + c->eps2);
#endif
        c->snap[j] = b2;
        for (int32_t w = 0; w < c->W; ++w) {
            c->x[(size_t)w * c->d + j] = xn;
            c->acc[(size_t)w * c->d + j] = b2;
        }
    }
    c->t += 1;
    return ORA_OK;
}

/* Algorithm 2, Local SGD: y = x - eta G on each worker; x averaged when mod(t,H)=0. */
int ora_localsgd_step_dense(ora_ctx *c, const real *G)
{
    if (!c || !G) return ORA_EINVAL;
    const real eta = ora_eta_at(c, c->t + 1);
    for (int32_t w = 0; w < c->W; ++w)
        for (int64_t j = 0; j < c->d; ++j) {
            const size_t k = (size_t)w * c->d + j;
            c->x[k] = c->x[k] - eta * G[k];
        }
    c->s += 1; c->t += 1;
    if (c->s == c->H) {
        for (int64_t j = 0; j < c->d; ++j) {
            real sx = 0;
            for (int32_t w = 0; w < c->W; ++w) sx += c->x[(size_t)w * c->d + j];
            const real mx = sx / (real)c->W;
            for (int32_t w = 0; w < c->W; ++w) c->x[(size_t)w * c->d + j] = mx;
        }
        c->s = 0;
    }
    return ORA_OK;
}
