/*
 * Driver for the host sanitizer build of the oracle (tests/test_oracle_sanitizers.py):
 * calls every entry point of oracle/fwa_oracle.c on two small shapes with exactly sized heap
 * buffers, so that AddressSanitizer sees any access past an end and UndefinedBehaviorSanitizer any
 * signed overflow, misaligned access or bad shift.  The values are checked only for being finite
 * and for two invariants (softmax rows sum to 1 -> with V = 1 the output is 1; rows of dS sum to
 * 0 -> rows of dBias do); the arithmetic is pinned elsewhere.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int fwa_oracle_forward(const double *q, const double *k, const double *v, double *o, double *p_out, long N, int L,
                       int C, int heads, double scale, const double *bias, const double *mask, int nW, int threads,
                       int *threads_used);
int fwa_oracle_backward(const double *q, const double *k, const double *v, const double *d_o, double *dq, double *dk,
                        double *dv, double *dbias, long N, int L, int C, int heads, double scale, const double *bias,
                        const double *mask, int nW, int threads, int *threads_used);
int fwa_oracle_bias_gather(const double *table, double *bias, int heads, int k);
int fwa_oracle_bias_scatter(const double *dbias, double *dtable, int heads, int k);
int fwa_oracle_mask_from_labels(const int *labels, double *mask, int nW, int L, double value);

static unsigned long long state = 88172645463325252ULL;
static double draw(void) { /* xorshift, uniform in (-1, 1) */
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}
static double *filled(size_t n, int ones) {
    double *p = (double *)malloc(n * sizeof(double));
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = ones ? 1.0 : draw();
    return p;
}
static int finite_all(const double *p, size_t n) {
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(p[i])) return 0;
    return 1;
}

static int one_shape(long N, int k, int heads, int d, int nW, int threads) {
    const int L = k * k, C = heads * d, T = (2 * k - 1) * (2 * k - 1);
    const size_t nlc = (size_t)N * L * C, hll = (size_t)heads * L * L;
    double *q = filled(nlc, 0), *kk = filled(nlc, 0), *v = filled(nlc, 1), *g = filled(nlc, 0);
    double *o = filled(nlc, 0), *p = filled((size_t)N * heads * L * L, 0);
    double *dq = filled(nlc, 0), *dk = filled(nlc, 0), *dv = filled(nlc, 0), *db = filled(hll, 0);
    double *table = filled((size_t)heads * T, 0), *bias = filled(hll, 0), *dtable = filled((size_t)heads * T, 0);
    double *mask = filled((size_t)nW * L * L, 0);
    int *labels = (int *)malloc((size_t)nW * L * sizeof(int));
    if (!labels) exit(3);
    for (int i = 0; i < nW * L; ++i) labels[i] = (i * 7 + i / L) % 3;
    int used = 0, bad = 0;
    bad |= fwa_oracle_bias_gather(table, bias, heads, k);
    bad |= fwa_oracle_mask_from_labels(labels, mask, nW, L, -100.0);
    bad |= fwa_oracle_forward(q, kk, v, o, p, N, L, C, heads, 0.3, bias, mask, nW, threads, &used);
    for (size_t i = 0; i < nlc; ++i) bad |= fabs(o[i] - 1.0) > 1e-12; /* V = 1: every output is a row sum of P */
    bad |= fwa_oracle_forward(q, kk, g, o, NULL, N, L, C, heads, 0.3, NULL, NULL, 0, threads, NULL);
    bad |= fwa_oracle_backward(q, kk, v, g, dq, dk, dv, db, N, L, C, heads, 0.3, bias, mask, nW, threads, &used);
    for (int r = 0; r < heads * L; ++r) {
        double s = 0.0;
        for (int j = 0; j < L; ++j) s += db[(size_t)r * L + j];
        bad |= fabs(s) > 1e-9;
    }
    bad |= fwa_oracle_backward(q, kk, v, g, dq, dk, dv, NULL, N, L, C, heads, 0.3, NULL, NULL, 0, threads, NULL);
    bad |= fwa_oracle_bias_scatter(db, dtable, heads, k);
    bad |= !finite_all(o, nlc) || !finite_all(dq, nlc) || !finite_all(dk, nlc) || !finite_all(dv, nlc) ||
           !finite_all(dtable, (size_t)heads * T);
    free(q); free(kk); free(v); free(g); free(o); free(p); free(dq); free(dk); free(dv); free(db);
    free(table); free(bias); free(dtable); free(mask); free(labels);
    return bad;
}

int main(void) {
    int bad = 0;
    bad |= one_shape(6, 3, 2, 4, 3, 2);   /* L = 9, two heads of width 4, mask period 3, two threads */
    bad |= one_shape(2, 7, 3, 32, 1, 1);  /* the 7 x 7 window at head width 32, one thread */
    bad |= one_shape(0, 2, 1, 2, 1, 1);   /* an empty batch */
    printf(bad ? "FAILED\n" : "clean\n");
    return bad ? 1 : 0;
}
