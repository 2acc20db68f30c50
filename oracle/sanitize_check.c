/*
 * Sanitizer driver of the CPU oracle (test infrastructure, CPU only): every exported routine of
 * sinkhorn_oracle.c on small seeded problems that reach its corner cases -- dense and point-cloud
 * costs, 1 x 1, zero weights (log = -inf), a row whose weights are all zero (potential +inf), early
 * stop, warm start, histories.  Built together with the oracle under -fsanitize=address,undefined
 * (oracle/build.py --sanitize); exits 0 when nothing was reported and the results are sane.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int fso_real_bytes(void);
void fso_update_f(const float *, const float *, const float *, int, const float *, const float *, int, int, double,
                  const double *, double *);
void fso_update_g(const float *, const float *, const float *, int, const float *, const float *, int, int, double,
                  const double *, double *);
void fso_marginals(const float *, const float *, const float *, int, const float *, const float *, int, int, double,
                   const double *, const double *, double *, double *);
double fso_marginal_err(const float *, const float *, const float *, int, const float *, const float *, int, int,
                        double, const double *, const double *);
void fso_plan(const float *, const float *, const float *, int, const float *, const float *, int, int, double,
              const double *, const double *, double *);
void fso_barycentric(const float *, const float *, const float *, int, const float *, const float *, int, int, double,
                     const double *, const double *, const double *, int, double *);
void fso_objectives(const float *, const float *, const float *, int, const float *, const float *, int, int, double,
                    const double *, const double *, double *);
int fso_solve(const float *, const float *, const float *, int, const float *, const float *, int, int, double, int,
              double, int, int, int, double *, double *, double *, double *, int *);

static unsigned long long rng_state = 88172645463325252ull;
static double urand(void) {            /* xorshift64: seeded, no library state */
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}

static int fails = 0;
#define CHECK(cond, msg) do { if (!(cond)) { fprintf(stderr, "sanitize_check: %s (line %d)\n", msg, __LINE__); ++fails; } } while (0)

static void one_case(int n, int m, int d, double eps, int zero_a, int zero_b) {
    float *C = NULL, *X = NULL, *Y = NULL;
    float *a = malloc(sizeof(float) * n), *b = malloc(sizeof(float) * m);
    if (d == 0) {
        C = malloc(sizeof(float) * (size_t)n * m);
        for (size_t q = 0; q < (size_t)n * m; ++q) C[q] = (float)(2.0 * urand());
    } else {
        X = malloc(sizeof(float) * (size_t)n * d); Y = malloc(sizeof(float) * (size_t)m * d);
        for (size_t q = 0; q < (size_t)n * d; ++q) X[q] = (float)urand();
        for (size_t q = 0; q < (size_t)m * d; ++q) Y[q] = (float)urand();
    }
    double sa = 0, sb = 0;
    for (int i = 0; i < n; ++i) { a[i] = (float)(0.1 + urand()); if (zero_a && i % 3 == 1) a[i] = 0; sa += a[i]; }
    for (int j = 0; j < m; ++j) { b[j] = (float)(0.1 + urand()); if (zero_b && j % 4 == 2) b[j] = 0; sb += b[j]; }
    for (int i = 0; i < n; ++i) a[i] = (float)(a[i] / sa);
    for (int j = 0; j < m; ++j) b[j] = (float)(b[j] / sb);
    double *f = calloc(n, sizeof(double)), *g = calloc(m, sizeof(double));
    double *f2 = malloc(sizeof(double) * n), *g2 = malloc(sizeof(double) * m);
    double *r = malloc(sizeof(double) * n), *c = malloc(sizeof(double) * m);
    double *P = malloc(sizeof(double) * (size_t)n * m);
    const int K = 30, dz = 3;
    double *eh = malloc(sizeof(double) * K), *dh = malloc(sizeof(double) * 2 * K);
    double *Z = malloc(sizeof(double) * (size_t)m * dz), *T = malloc(sizeof(double) * (size_t)n * dz);
    for (size_t q = 0; q < (size_t)m * dz; ++q) Z[q] = urand();
    int conv = -1;
    int it = fso_solve(C, X, Y, d, a, b, n, m, eps, K, 1e-9, 5, 0, 1, f, g, eh, dh, &conv);
    CHECK(it >= 1 && it <= K && (conv == 0 || conv == 1), "solve: iteration count / flag");
    for (int k = 1; k < 2 * it; ++k) CHECK(dh[k] >= dh[k - 1] - 1e-9 * fabs(dh[k - 1]) - 1e-12, "dual objective decreased");
    fso_update_f(C, X, Y, d, a, b, n, m, eps, g, f2);
    fso_update_g(C, X, Y, d, a, b, n, m, eps, f2, g2);
    fso_marginals(C, X, Y, d, a, b, n, m, eps, f2, g2, r, c);
    for (int j = 0; j < m; ++j) CHECK(fabs(c[j] - b[j]) <= 1e-12, "column marginal after a g-step");
    double e = fso_marginal_err(C, X, Y, d, a, b, n, m, eps, f2, g2);
    CHECK(e >= 0 && e < 2.0 + 1e-9, "marginal error out of range");
    fso_plan(C, X, Y, d, a, b, n, m, eps, f2, g2, P);
    double mass = 0;
    for (size_t q = 0; q < (size_t)n * m; ++q) { CHECK(P[q] >= 0 && P[q] <= 1 + 1e-12, "plan entry out of range"); mass += P[q]; }
    CHECK(fabs(mass - 1.0) < 1e-6 || zero_a || zero_b, "plan mass");
    fso_barycentric(C, X, Y, d, a, b, n, m, eps, f2, g2, Z, dz, T);
    for (size_t q = 0; q < (size_t)n * dz; ++q) CHECK(T[q] >= -1e-12 && T[q] <= 1 + 1e-12, "barycentre outside the hull of Z");
    double obj[5];
    fso_objectives(C, X, Y, d, a, b, n, m, eps, f2, g2, obj);
    CHECK(isfinite(obj[0]) && obj[1] > 0, "objectives");
    /* warm start from the returned potentials: one more iteration, no history buffers */
    it = fso_solve(C, X, Y, d, a, b, n, m, eps, 1, 0.0, 0, 1, 0, f, g, NULL, NULL, NULL);
    CHECK(it == 1, "warm-started solve");
    free(C); free(X); free(Y); free(a); free(b); free(f); free(g); free(f2); free(g2); free(r); free(c); free(P);
    free(eh); free(dh); free(Z); free(T);
}

int main(void) {
    if (fso_real_bytes() != 8) { fprintf(stderr, "sanitize_check wants the double-precision build\n"); return 2; }
    one_case(1, 1, 0, 0.1, 0, 0);
    one_case(7, 5, 0, 0.05, 0, 0);
    one_case(33, 40, 0, 0.01, 1, 1);
    one_case(64, 17, 0, 1e-3, 0, 1);
    one_case(1, 9, 3, 0.1, 0, 0);
    one_case(20, 31, 2, 0.02, 1, 0);
    one_case(12, 12, 7, 1e-3, 0, 0);
    /* a problem whose source weights are all zero but one: every other row has log a = -inf */
    {
        float C[6] = {0.f, 1.f, 2.f, 1.f, 0.f, 1.f}, a[2] = {1.f, 0.f}, b[3] = {0.5f, 0.25f, 0.25f};
        double f[2] = {0, 0}, g[3] = {0, 0, 0};
        int it = fso_solve(C, NULL, NULL, 0, a, b, 2, 3, 0.1, 5, 0.0, 10, 0, 0, f, g, NULL, NULL, NULL);
        CHECK(it == 5 && isfinite(f[0]) && isfinite(f[1]) && isfinite(g[0]), "zero-weight row");
    }
    if (fails) { fprintf(stderr, "sanitize_check: %d check(s) failed\n", fails); return 1; }
    printf("sanitize_check: ok\n");
    return 0;
}
