/* Sanitizer driver for the CPU oracle: built together with oracle/sparsek_oracle.c under
 * -fsanitize=address,undefined and run by tests/test_sanitizers.py.  It calls every oracle routine on small seeded
 * inputs (ragged sizes, ties, k >= n, k = 0, w = 0) and checks a few invariants, so that an out-of-bounds access, a
 * use of uninitialised heap memory that changes a result, or undefined arithmetic anywhere in the oracle stops it. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_sparsek(const float *z, int m, int k, double *tau_out, double *p, int *ustar, int *wstar);
int orc_tau_prefixes(const float *u, int n, int k, double *tau, int *ustar, int *wstar);
int orc_tau_incremental(const float *u, int n, int k, double *tau);
int orc_select_prefix(const float *u, int t, int k, int32_t *idx);
int orc_death(const float *u, int n, int k, int32_t *death);
int orc_attn_query_bydef(const float *q, const float *K, const float *V, const float *u, int n, int d, int k, int w,
                         int gate_mode, double scale, int i, double *o, double *lse);
int orc_attn_fwd(const float *q, const float *K, const float *V, const float *u, const double *tau,
                 const int32_t *death, int B, int H, int Gu, int n, int d, int k, int w, int gate_mode, double scale,
                 double *o, double *lse, int nthreads);
int orc_mask_bwd(const float *q, const float *K, const float *V, const float *u, const double *tau,
                 const int32_t *death, const float *dO, int B, int H, int Gu, int n, int d, int k, int w,
                 int gate_mode, double scale, double *du, int nthreads);
int orc_attn_bwd(const float *q, const float *K, const float *V, const float *u, const double *tau,
                 const int32_t *death, const float *dO, int B, int H, int Gu, int n, int d, int k, int w,
                 int gate_mode, double scale, double *dQ, double *dK, double *dV, int nthreads);
int orc_decode_incremental(const float *q_steps, const float *K, const float *V, const float *u, int n_ctx, int steps,
                           int d, int k, int w, int gate_mode, double scale, double *o, double *seconds);
int orc_scores(const float *X, const float *w, int B, int n, int D, double slope, int norm, double norm_eps, double *u);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void)   /* uniform in (-1, 1), xorshift */
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}
static float *vec(size_t n, double scale, int grid)
{
    float *a = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; i++) a[i] = grid ? (float)(floor(rnd() * scale * 4.0) / 4.0) : (float)(rnd() * scale);
    return a;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "oracle_san: check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int one_case(int B, int H, int Gu, int n, int d, int k, int w, int mode, int grid)
{
    const size_t rows = (size_t)B * Gu, heads = (size_t)B * H;
    float *u = vec(rows * n, 2.0, grid), *q = vec(heads * n * d, 0.5, 0), *K = vec(heads * n * d, 0.5, 0);
    float *V = vec(heads * n * d, 0.5, 0), *dO = vec(heads * n * d, 1.0, 0);
    double *tau = (double *)malloc(sizeof(double) * rows * n), *tau2 = (double *)malloc(sizeof(double) * n);
    int32_t *death = (int32_t *)malloc(sizeof(int32_t) * rows * n), *idx = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    int *us = (int *)malloc(sizeof(int) * n), *ws = (int *)malloc(sizeof(int) * n);
    double *p = (double *)malloc(sizeof(double) * n);
    for (size_t r = 0; r < rows; r++) {
        CHECK(orc_tau_prefixes(u + r * n, n, k, tau + r * n, us, ws) == 0);
        CHECK(orc_tau_incremental(u + r * n, n, k, tau2) == 0);
        for (int t = 0; t < n; t++) CHECK(fabs(tau2[t] - tau[r * n + t]) <= 1e-9 * fmax(1.0, fabs(tau2[t])));
        CHECK(orc_death(u + r * n, n, k, death + r * n) == 0);
        double tq;
        int a, b;
        CHECK(orc_sparsek(u + r * n, n, k, &tq, p, &a, &b) == 0);
        double sum = 0.0;
        for (int j = 0; j < n; j++) sum += p[j];
        CHECK(fabs(sum - (double)(k < n ? k : n)) <= 1e-9 * n);
        int cnt = orc_select_prefix(u + r * n, n - 1, k, idx);
        CHECK(cnt == (k < n ? k : n));
        for (int c = 0; c < cnt; c++) CHECK(death[r * n + idx[c]] == n);   /* selected at the end <=> still alive */
    }
    double *o = (double *)malloc(sizeof(double) * heads * n * d), *lse = (double *)malloc(sizeof(double) * heads * n);
    CHECK(orc_attn_fwd(q, K, V, u, tau, death, B, H, Gu, n, d, k, w, mode, 0.7, o, lse, 2) > 0);
    double *o1 = (double *)malloc(sizeof(double) * d), l1;
    CHECK(orc_attn_query_bydef(q, K, V, u, n, d, k, w, mode, 0.7, n - 1, o1, &l1) == 0);
    for (int c = 0; c < d; c++) CHECK(fabs(o1[c] - o[(size_t)(n - 1) * d + c]) <= 1e-9);
    double *du = (double *)malloc(sizeof(double) * rows * n);
    CHECK(orc_mask_bwd(q, K, V, u, tau, death, dO, B, H, Gu, n, d, k, w, mode, 0.7, du, 2) > 0);
    double *dQ = (double *)malloc(sizeof(double) * heads * n * d), *dK = (double *)malloc(sizeof(double) * heads * n * d);
    double *dV = (double *)malloc(sizeof(double) * heads * n * d);
    CHECK(orc_attn_bwd(q, K, V, u, tau, death, dO, B, H, Gu, n, d, k, w, mode, 0.7, dQ, dK, dV, 2) > 0);
    for (size_t i = 0; i < heads * n * d; i++) CHECK(isfinite(dQ[i]) && isfinite(dK[i]) && isfinite(dV[i]));
    if (n > 8) {   /* decode of the last 5 positions of head 0 = rows of the prefill */
        const int steps = 5, nc = n - steps;
        double *od = (double *)malloc(sizeof(double) * steps * d);
        CHECK(orc_decode_incremental(q + (size_t)nc * d, K, V, u, nc, steps, d, k, w, mode, 0.7, od, NULL) == 0);
        for (int i = 0; i < steps * d; i++) CHECK(fabs(od[i] - o[(size_t)nc * d + i]) <= 1e-9);
        free(od);
    }
    free(u); free(q); free(K); free(V); free(dO); free(tau); free(tau2); free(death); free(idx); free(us); free(ws);
    free(p); free(o); free(lse); free(o1); free(du); free(dQ); free(dK); free(dV);
    return 0;
}

int main(void)
{
    const int cases[][9] = {
        /* B  H Gu   n   d   k   w mode grid */
        {1, 1, 1, 1, 4, 1, 1, 0, 0},   {1, 2, 1, 37, 8, 5, 3, 0, 0},  {2, 2, 2, 50, 4, 7, 0, 1, 1},
        {1, 2, 2, 40, 12, 0, 6, 2, 0}, {1, 1, 1, 30, 4, 64, 2, 3, 1}, {1, 3, 1, 65, 16, 9, 70, 0, 1},
    };
    for (size_t c = 0; c < sizeof(cases) / sizeof(cases[0]); c++) {
        const int *x = cases[c];
        if (one_case(x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7], x[8])) { fprintf(stderr, "case %zu failed\n", c); return 1; }
    }
    float *X = vec(2 * 33 * 16, 1.0, 0), *w = vec(16, 0.3, 0);
    double *u = (double *)malloc(sizeof(double) * 2 * 33);
    if (orc_scores(X, w, 2, 33, 16, 0.01, 1, 1e-5, u) != 0 || fabs(u[0]) > 1e-9) { fprintf(stderr, "scores failed\n"); return 1; }
    free(X); free(w); free(u);
    printf("oracle_san ok\n");
    return 0;
}
