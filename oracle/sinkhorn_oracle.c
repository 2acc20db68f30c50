/*
 * CPU oracle for log-domain Sinkhorn (entropic optimal transport).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * statement of what the hot path computes.  It is used by the test-suite, by
 * the smoke check and by the benchmark's cpu_baseline leg; the product (the
 * HIP library) never calls it, links it or shares any code with it.
 *
 * Every routine is the paper's definition written out in the paper's order and
 * notation (alpha -> f, beta -> g, mu -> a, nu -> b, pi -> P):
 *   - plan            P_ij = a_i b_j exp((f_i + g_j - C_ij)/eps)          (Eq. 5)
 *   - LogSumExp       max + log sum exp(x - max)                          (Eq. 8)
 *   - f-update        f_i = -eps LSE_j((g_j - C_ij)/eps + log b_j)        (Eq. 9)
 *   - g-update        g_j = -eps LSE_i((f_i - C_ij)/eps + log a_i)        (Eq. 10)
 *   - row marginal    log r_i = log a_i + LSE_j((f_i+g_j-C_ij)/eps + log b_j)   (Sec. 4.5)
 *   - marginal error  err = sum_i |r_i - a_i|                             (Alg. 1)
 *   - driver loop     f then g (g uses the new f), check every c iterations,
 *                     stop when err < tol                                 (Alg. 1, Eqs. 6-7)
 *   - transport cost  sum_ij C_ij P_ij                                    (Alg. 1, last step)
 *   - objectives      <C,P> + eps KL(P | a x b) with the paper's KL       (Eqs. 3-4)
 *
 * Arithmetic is IEEE double (or long double when built with
 * -DFSO_LONG_DOUBLE, used only to show that double is itself converged).
 * Inputs are the fp32 arrays the GPU gets, promoted value by value.  There is
 * no blocking, no fusion and no reordering: each row / column is reduced
 * serially in index order, so results do not depend on the thread count
 * (OpenMP only spreads independent rows / columns over cores).
 *
 * Readings where the paper is silent:
 *   - a weight of zero has log = -inf and contributes nothing; if every term
 *     of an LSE is -inf the LSE is -inf and the potential is +inf (no floor).
 *   - point-cloud cost is the squared Euclidean distance in difference form.
 *   - the dual objective is D = <a,f> + <b,g> - eps sum_ij P_ij + eps, which
 *     follows from Eqs. 3-4 and the Lagrangian of Appendix A.1.
 *
 * Parity pins for this file live in tests/test_oracle_pins.py.  The paper's
 * printed timings / iteration counts / costs (Tables 1-3) cannot pin it: their
 * inputs are unseeded and unspecified.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef FSO_LONG_DOUBLE
typedef long double real;
#define R_EXP expl
#define R_LOG logl
#define R_FABS fabsl
#else
typedef double real;
#define R_EXP exp
#define R_LOG log
#define R_FABS fabs
#endif

#define R_NEG_INF (-(real)INFINITY)

typedef struct {
    const float *C;      /* dense n x m row-major cost, or NULL */
    const float *X;      /* n x d row-major points, or NULL     */
    const float *Y;      /* m x d row-major points, or NULL     */
    const float *a;      /* n source weights (mu)               */
    const float *b;      /* m target weights (nu)               */
    int32_t d, n, m;
    real eps;
} fso_problem;

/* C_ij: the stored fp32 entry, or ||x_i - y_j||^2 from the fp32 coordinates. */
static inline real cost_ij(const fso_problem *p, int64_t i, int64_t j) {
    if (p->C) return (real)p->C[i * p->m + j];
    real s = 0;
    for (int t = 0; t < p->d; ++t) {
        real df = (real)p->X[i * p->d + t] - (real)p->Y[j * p->d + t];
        s += df * df;
    }
    return s;
}

static inline real log_weight(float w) { return w > 0.0f ? R_LOG((real)w) : R_NEG_INF; }

static void fill_problem(fso_problem *p, const float *C, const float *X, const float *Y, int d,
                         const float *a, const float *b, int n, int m, double eps) {
    p->C = C; p->X = X; p->Y = Y; p->d = d; p->a = a; p->b = b; p->n = n; p->m = m;
    p->eps = (real)eps;
}

/* LSE_j( (shift + g_j - C_ij)/eps + log b_j ), Eq. 8 applied to row i. */
static real row_lse(const fso_problem *p, int64_t i, const real *g, real shift) {
    real M = R_NEG_INF;
    for (int64_t j = 0; j < p->m; ++j) {
        real x = (shift + g[j] - cost_ij(p, i, j)) / p->eps + log_weight(p->b[j]);
        if (x > M) M = x;
    }
    if (M == R_NEG_INF) return R_NEG_INF;
    real s = 0;
    for (int64_t j = 0; j < p->m; ++j) {
        real x = (shift + g[j] - cost_ij(p, i, j)) / p->eps + log_weight(p->b[j]);
        s += R_EXP(x - M);
    }
    return M + R_LOG(s);
}

/* LSE_i( (shift + f_i - C_ij)/eps + log a_i ), Eq. 8 applied to column j. */
static real col_lse(const fso_problem *p, int64_t j, const real *f, real shift) {
    real M = R_NEG_INF;
    for (int64_t i = 0; i < p->n; ++i) {
        real y = (shift + f[i] - cost_ij(p, i, j)) / p->eps + log_weight(p->a[i]);
        if (y > M) M = y;
    }
    if (M == R_NEG_INF) return R_NEG_INF;
    real s = 0;
    for (int64_t i = 0; i < p->n; ++i) {
        real y = (shift + f[i] - cost_ij(p, i, j)) / p->eps + log_weight(p->a[i]);
        s += R_EXP(y - M);
    }
    return M + R_LOG(s);
}

static void update_f(const fso_problem *p, const real *g, real *f) {      /* Eq. 9 */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < p->n; ++i) f[i] = -p->eps * row_lse(p, i, g, 0);
}

static void update_g(const fso_problem *p, const real *f, real *g) {      /* Eq. 10 */
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < p->m; ++j) g[j] = -p->eps * col_lse(p, j, f, 0);
}

/* r_i = exp(log a_i + LSE_j((f_i + g_j - C_ij)/eps + log b_j)), Sec. 4.5. */
static void row_marginals(const fso_problem *p, const real *f, const real *g, real *r) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < p->n; ++i) {
        real l = row_lse(p, i, g, f[i]);
        r[i] = (p->a[i] > 0.0f && l > R_NEG_INF) ? R_EXP(log_weight(p->a[i]) + l) : 0;
    }
}

static void col_marginals(const fso_problem *p, const real *f, const real *g, real *c) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < p->m; ++j) {
        real l = col_lse(p, j, f, g[j]);
        c[j] = (p->b[j] > 0.0f && l > R_NEG_INF) ? R_EXP(log_weight(p->b[j]) + l) : 0;
    }
}

/* err = sum_i |r_i - a_i| (Alg. 1), its own pass over the costs. */
static real marginal_err(const fso_problem *p, const real *f, const real *g, real *r_scratch) {
    row_marginals(p, f, g, r_scratch);
    real e = 0;
    for (int64_t i = 0; i < p->n; ++i) e += R_FABS(r_scratch[i] - (real)p->a[i]);
    return e;
}

/* P_ij of Eq. 5 with the weights inside the exponent as in Alg. 1's last step. */
static inline real plan_ij(const fso_problem *p, const real *f, const real *g, int64_t i, int64_t j) {
    if (!(p->a[i] > 0.0f) || !(p->b[j] > 0.0f)) return 0;
    return R_EXP((f[i] + g[j] - cost_ij(p, i, j)) / p->eps + log_weight(p->a[i]) + log_weight(p->b[j]));
}

/* Three sums over the plan, each row summed in index order, then rows in index order:
 * mass = sum P, cost = sum C P, ent = sum P (log(P/(a b)) - 1). */
static void plan_sums(const fso_problem *p, const real *f, const real *g,
                      real *mass, real *cost, real *ent) {
    real *rm = (real *)malloc(sizeof(real) * 3 * (size_t)p->n);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < p->n; ++i) {
        real sm = 0, sc = 0, se = 0;
        for (int64_t j = 0; j < p->m; ++j) {
            real pij = plan_ij(p, f, g, i, j);
            if (pij > 0) {
                real lr = (f[i] + g[j] - cost_ij(p, i, j)) / p->eps;   /* log(P/(a b)) */
                sm += pij;
                sc += cost_ij(p, i, j) * pij;
                se += pij * (lr - 1);
            }
        }
        rm[3 * i] = sm; rm[3 * i + 1] = sc; rm[3 * i + 2] = se;
    }
    real tm = 0, tc = 0, te = 0;
    for (int64_t i = 0; i < p->n; ++i) { tm += rm[3 * i]; tc += rm[3 * i + 1]; te += rm[3 * i + 2]; }
    free(rm);
    *mass = tm; *cost = tc; *ent = te;
}

/* D(f,g) = <a,f> + <b,g> - eps sum_ij P_ij + eps  (zero-weight entries skipped). */
static real dual_objective(const fso_problem *p, const real *f, const real *g) {
    real mass, cost, ent;
    plan_sums(p, f, g, &mass, &cost, &ent);
    real d = 0;
    for (int64_t i = 0; i < p->n; ++i) if (p->a[i] > 0.0f) d += (real)p->a[i] * f[i];
    for (int64_t j = 0; j < p->m; ++j) if (p->b[j] > 0.0f) d += (real)p->b[j] * g[j];
    return d - p->eps * mass + p->eps;
}

/* ------------------------------------------------------------------ C interface
 * All pointers are host pointers owned by the caller.  Exactly one of C or
 * (X, Y, d>0) is non-NULL.  Potentials and outputs are arrays of `real`
 * (double, or long double in the FSO_LONG_DOUBLE build).                        */

int fso_real_bytes(void) { return (int)sizeof(real); }

void fso_update_f(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                  int n, int m, double eps, const real *g, real *f_out) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
    update_f(&p, g, f_out);
}

void fso_update_g(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                  int n, int m, double eps, const real *f, real *g_out) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
    update_g(&p, f, g_out);
}

void fso_marginals(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                   int n, int m, double eps, const real *f, const real *g, real *r_out, real *c_out) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
    if (r_out) row_marginals(&p, f, g, r_out);
    if (c_out) col_marginals(&p, f, g, c_out);
}

real fso_marginal_err(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, double eps, const real *f, const real *g) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
    real *r = (real *)malloc(sizeof(real) * (size_t)n);
    real e = marginal_err(&p, f, g, r);
    free(r);
    return e;
}

void fso_plan(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
              int n, int m, double eps, const real *f, const real *g, real *P_out) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j) P_out[i * m + j] = plan_ij(&p, f, g, i, j);
}

/* Barycentric projection of the plan (the "barycentric mapping" of Sec. 5.6):
 * T[i][t] = sum_j P_ij Z[j][t] / sum_j P_ij; a row without mass gives 0.
 * Z: m x dz, T_out: n x dz, both row-major. */
void fso_barycentric(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                     int n, int m, double eps, const real *f, const real *g, const real *Z, int dz,
                     real *T_out) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        real den = 0;
        for (int t = 0; t < dz; ++t) T_out[i * dz + t] = 0;
        for (int64_t j = 0; j < m; ++j) {
            real pij = plan_ij(&p, f, g, i, j);
            den += pij;
            for (int t = 0; t < dz; ++t) T_out[i * dz + t] += pij * Z[j * dz + t];
        }
        for (int t = 0; t < dz; ++t) T_out[i * dz + t] = den > 0 ? T_out[i * dz + t] / den : 0;
    }
}

/* out[0] = <C,P>, out[1] = sum P, out[2] = KL(P | a x b) of Eq. 4,
 * out[3] = primal objective of Eq. 3, out[4] = dual objective D(f,g). */
void fso_objectives(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                    int n, int m, double eps, const real *f, const real *g, real *out) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
    real mass, cost, ent;
    plan_sums(&p, f, g, &mass, &cost, &ent);
    out[0] = cost;
    out[1] = mass;
    out[2] = ent + 1;
    out[3] = cost + p.eps * (ent + 1);
    out[4] = dual_objective(&p, f, g);
}

/* Alg. 1.  f, g: in/out (used as the start iff warm_start, else zeroed).
 * err_hist (len max_iter, may be NULL): err after every iteration k (NaN where not
 * evaluated: it is evaluated at every k when err_every_iter != 0, else only at
 * the checked iterations k mod check_every == 0).
 * dual_hist (len 2*max_iter, may be NULL): D after the f half-step and after the g
 * half-step of every iteration.
 * Returns the number of iterations performed; *converged_out says whether the
 * tolerance test fired. */
int fso_solve(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
              int n, int m, double eps, int max_iter, double tol, int check_every, int warm_start,
              int err_every_iter, real *f, real *g, real *err_hist, real *dual_hist, int *converged_out) {
    fso_problem p; fill_problem(&p, C, X, Y, d, a, b, n, m, eps);
    if (check_every <= 0) check_every = 10;
    if (!warm_start) {
        for (int64_t i = 0; i < n; ++i) f[i] = 0;
        for (int64_t j = 0; j < m; ++j) g[j] = 0;
    }
    real *r = (real *)malloc(sizeof(real) * (size_t)n);
    int k = 0, converged = 0;
    while (k < max_iter) {
        update_f(&p, g, f);
        if (dual_hist) dual_hist[2 * k] = dual_objective(&p, f, g);
        update_g(&p, f, g);
        if (dual_hist) dual_hist[2 * k + 1] = dual_objective(&p, f, g);
        ++k;
        int checked = (tol > 0) && (k % check_every == 0);
        real e = (real)NAN;
        if (checked || err_every_iter) e = marginal_err(&p, f, g, r);
        if (err_hist) err_hist[k - 1] = e;
        if (checked && e < (real)tol) { converged = 1; break; }
    }
    free(r);
    if (converged_out) *converged_out = converged;
    return k;
}
