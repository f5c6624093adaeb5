/*
 * fwa_oracle.c -- plain fp64 CPU oracle for window attention, forward and backward.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares
 * no code with the GPU library and must never be linked into it.
 *
 * What it computes, per window n and head h (rows q_i, k_j, v_j are the
 * d = C/heads wide channel slices X[n, i, h*d : (h+1)*d]):
 *
 *   forward  (paper Section 2.1, eq. 2-4; the feature-dimension tiling of
 *   eq. 5-6 and Algorithm 1 is an identity on top of these, so the oracle
 *   is the definition written out):
 *       s_ij = scale * <q_i, k_j> + B[h,i,j] + M[n mod nW, i, j]
 *       p_ij = exp(s_ij - max_l s_il) / sum_l exp(s_il - max_l s_il)
 *       o_i  = sum_j p_ij v_j
 *
 *   backward (paper Algorithm 2, the five assignments after the softmax
 *   recomputation; the derivation is the standard attention backward):
 *       dv_j  = sum_i p_ij do_i
 *       dp_ij = <do_i, v_j>
 *       ds_ij = p_ij (dp_ij - sum_l p_il dp_il)
 *       dq_i  = scale * sum_j ds_ij k_j
 *       dk_j  = scale * sum_i ds_ij q_i
 *       dB[h,i,j] = sum_n ds_ij^(n,h)
 *
 * Readings where the paper is silent (the equations carry no scale, bias or
 * mask): scale multiplies QK^T before B and M are added, so it also
 * multiplies dq and dk but not dB; B is indexed by head, M by n mod nW; M
 * receives no gradient; the row maximum is subtracted before exp, which
 * changes nothing mathematically.
 *
 * Everything is double precision; inputs are passed as doubles (bf16 and
 * fp32 test inputs are exactly representable).  Loops are written in the
 * order of the formulas, with no blocking or fusion.  Threads split the
 * window index n into contiguous ranges (OpenMP static schedule); dB is
 * accumulated per thread and the per-thread partial sums are added in
 * thread order, so a run is reproducible for a fixed thread count.
 *
 * Pins (tests/test_oracle_*.py): brute-force enumeration on tiny shapes,
 * closed forms (L=1, L=2, equal keys), softmax row sums, Q=0 mean of V,
 * key/value permutation invariance, score-shift invariance, linearity in
 * V, the feature-chunk identity of eq. 5-6, the block-diagonal mask limit,
 * central finite differences and the adjoint identity for the backward,
 * and a float64 library expression as a third opinion.  The label mask: a
 * case written out by hand, the equivalence-class structure, and the dense
 * shift mask of the input generator as a third opinion.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define FWA_ORACLE_OK 0
#define FWA_ORACLE_BAD_ARG 1
#define FWA_ORACLE_NO_MEM 2

static int check_shape(long N, int L, int C, int heads, int nW, const double *mask)
{
    if (N < 0 || L < 1 || C < 1 || heads < 1) return FWA_ORACLE_BAD_ARG;
    if (C % heads != 0) return FWA_ORACLE_BAD_ARG;
    if (mask != NULL && (nW < 1 || N % nW != 0)) return FWA_ORACLE_BAD_ARG;
    return FWA_ORACLE_OK;
}

/* scores and probabilities of one (window, head): s and p are L*L row-major. */
static void scores_and_probs(const double *q, const double *k, long n, int h, int L, int C, int d,
                             double scale, const double *bias, const double *mask, int nW,
                             double *s, double *p)
{
    const double *qn = q + (size_t)n * L * C + (size_t)h * d;
    const double *kn = k + (size_t)n * L * C + (size_t)h * d;
    for (int i = 0; i < L; ++i) {
        for (int j = 0; j < L; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += qn[(size_t)i * C + c] * kn[(size_t)j * C + c];
            double sij = scale * dot;
            if (bias) sij += bias[((size_t)h * L + i) * L + j];
            if (mask) sij += mask[((size_t)(n % nW) * L + i) * L + j];
            s[(size_t)i * L + j] = sij;
        }
    }
    for (int i = 0; i < L; ++i) {
        double m = s[(size_t)i * L];
        for (int j = 1; j < L; ++j)
            if (s[(size_t)i * L + j] > m) m = s[(size_t)i * L + j];
        double z = 0.0;
        for (int j = 0; j < L; ++j) {
            p[(size_t)i * L + j] = exp(s[(size_t)i * L + j] - m);
            z += p[(size_t)i * L + j];
        }
        for (int j = 0; j < L; ++j) p[(size_t)i * L + j] /= z;
    }
}

/*
 * Forward.  q,k,v,o: [N,L,C] row-major doubles.  bias: NULL or [heads,L,L].
 * mask: NULL or [nW,L,L].  p_out: NULL or [N,heads,L,L], receives P.
 * threads <= 0 means "use the OpenMP default".  Returns the number of
 * threads used through *threads_used when that pointer is not NULL.
 */
int fwa_oracle_forward(const double *q, const double *k, const double *v, double *o, double *p_out,
                       long N, int L, int C, int heads, double scale,
                       const double *bias, const double *mask, int nW,
                       int threads, int *threads_used)
{
    int rc = check_shape(N, L, C, heads, nW, mask);
    if (rc) return rc;
    if (N > 0 && (!q || !k || !v || !o)) return FWA_ORACLE_BAD_ARG;
    const int d = C / heads;
    int used = 1;
    int failed = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#endif
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        double *s = (double *)malloc(sizeof(double) * (size_t)L * L);
        double *p = (double *)malloc(sizeof(double) * (size_t)L * L);
        if (!s || !p) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (long n = 0; n < N; ++n) {
                for (int h = 0; h < heads; ++h) {
                    scores_and_probs(q, k, n, h, L, C, d, scale, bias, mask, nW, s, p);
                    const double *vn = v + (size_t)n * L * C + (size_t)h * d;
                    double *on = o + (size_t)n * L * C + (size_t)h * d;
                    for (int i = 0; i < L; ++i) {
                        for (int c = 0; c < d; ++c) {
                            double acc = 0.0;
                            for (int j = 0; j < L; ++j) acc += p[(size_t)i * L + j] * vn[(size_t)j * C + c];
                            on[(size_t)i * C + c] = acc;
                        }
                    }
                    if (p_out)
                        memcpy(p_out + ((size_t)n * heads + h) * L * L, p, sizeof(double) * (size_t)L * L);
                }
            }
        }
        free(s);
        free(p);
    }
    if (threads_used) *threads_used = used;
    return failed ? FWA_ORACLE_NO_MEM : FWA_ORACLE_OK;
}

/*
 * Backward.  q,k,v,d_o,dq,dk,dv: [N,L,C].  dbias: NULL or [heads,L,L],
 * overwritten with the sum over all N windows.  Needs nothing saved from the
 * forward: P is recomputed from q and k (Algorithm 2 takes Q,K,V,dO only).
 */
int fwa_oracle_backward(const double *q, const double *k, const double *v, const double *d_o,
                        double *dq, double *dk, double *dv, double *dbias,
                        long N, int L, int C, int heads, double scale,
                        const double *bias, const double *mask, int nW,
                        int threads, int *threads_used)
{
    int rc = check_shape(N, L, C, heads, nW, mask);
    if (rc) return rc;
    if (N > 0 && (!q || !k || !v || !d_o || !dq || !dk || !dv)) return FWA_ORACLE_BAD_ARG;
    const int d = C / heads;
    const size_t LL = (size_t)L * L;
    int used = 1;
    int failed = 0;
    int max_threads = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    max_threads = omp_get_max_threads();
#endif
    double *partial = NULL; /* [max_threads][heads][L][L] */
    if (dbias) {
        partial = (double *)calloc((size_t)max_threads * heads * LL, sizeof(double));
        if (!partial) return FWA_ORACLE_NO_MEM;
    }
#pragma omp parallel
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#pragma omp single
        used = omp_get_num_threads();
#endif
        double *s = (double *)malloc(sizeof(double) * LL);
        double *p = (double *)malloc(sizeof(double) * LL);
        double *dp = (double *)malloc(sizeof(double) * LL);
        double *ds = (double *)malloc(sizeof(double) * LL);
        if (!s || !p || !dp || !ds) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (long n = 0; n < N; ++n) {
                for (int h = 0; h < heads; ++h) {
                    const size_t base = (size_t)n * L * C + (size_t)h * d;
                    const double *qn = q + base, *kn = k + base, *vn = v + base, *gn = d_o + base;
                    double *dqn = dq + base, *dkn = dk + base, *dvn = dv + base;
                    scores_and_probs(q, k, n, h, L, C, d, scale, bias, mask, nW, s, p);
                    /* dV = P^T dO */
                    for (int j = 0; j < L; ++j)
                        for (int c = 0; c < d; ++c) {
                            double acc = 0.0;
                            for (int i = 0; i < L; ++i) acc += p[(size_t)i * L + j] * gn[(size_t)i * C + c];
                            dvn[(size_t)j * C + c] = acc;
                        }
                    /* dP = dO V^T */
                    for (int i = 0; i < L; ++i)
                        for (int j = 0; j < L; ++j) {
                            double acc = 0.0;
                            for (int c = 0; c < d; ++c) acc += gn[(size_t)i * C + c] * vn[(size_t)j * C + c];
                            dp[(size_t)i * L + j] = acc;
                        }
                    /* dS_ij = P_ij (dP_ij - sum_l P_il dP_il) */
                    for (int i = 0; i < L; ++i) {
                        double delta = 0.0;
                        for (int l = 0; l < L; ++l) delta += p[(size_t)i * L + l] * dp[(size_t)i * L + l];
                        for (int j = 0; j < L; ++j)
                            ds[(size_t)i * L + j] = p[(size_t)i * L + j] * (dp[(size_t)i * L + j] - delta);
                    }
                    /* dQ = scale dS K */
                    for (int i = 0; i < L; ++i)
                        for (int c = 0; c < d; ++c) {
                            double acc = 0.0;
                            for (int j = 0; j < L; ++j) acc += ds[(size_t)i * L + j] * kn[(size_t)j * C + c];
                            dqn[(size_t)i * C + c] = scale * acc;
                        }
                    /* dK = scale dS^T Q */
                    for (int j = 0; j < L; ++j)
                        for (int c = 0; c < d; ++c) {
                            double acc = 0.0;
                            for (int i = 0; i < L; ++i) acc += ds[(size_t)i * L + j] * qn[(size_t)i * C + c];
                            dkn[(size_t)j * C + c] = scale * acc;
                        }
                    /* dB[h] += dS */
                    if (partial) {
                        double *acc = partial + ((size_t)tid * heads + h) * LL;
                        for (size_t e = 0; e < LL; ++e) acc[e] += ds[e];
                    }
                }
            }
        }
        free(s);
        free(p);
        free(dp);
        free(ds);
    }
    if (dbias && !failed) {
        for (size_t e = 0; e < (size_t)heads * LL; ++e) {
            double acc = 0.0;
            for (int t = 0; t < max_threads; ++t) acc += partial[(size_t)t * heads * LL + e];
            dbias[e] = acc;
        }
    }
    free(partial);
    if (threads_used) *threads_used = used;
    return failed ? FWA_ORACLE_NO_MEM : FWA_ORACLE_OK;
}

/*
 * Relative-position bias of a k x k window (the paper only says the baseline
 * follows Swin Transformer; this is that published rule restated).  Token i
 * sits at (y_i, x_i) = (i / k, i % k) in the window; the pair (i, j) reads
 * table entry (y_i - y_j + k - 1) * (2k - 1) + (x_i - x_j + k - 1).
 *   table: [heads, (2k-1)^2]      bias: [heads, k*k, k*k]
 */
int fwa_oracle_bias_gather(const double *table, double *bias, int heads, int k)
{
    if (!table || !bias || heads < 1 || k < 1) return FWA_ORACLE_BAD_ARG;
    const int L = k * k, T = (2 * k - 1) * (2 * k - 1);
    for (int h = 0; h < heads; ++h)
        for (int i = 0; i < L; ++i)
            for (int j = 0; j < L; ++j) {
                int dy = i / k - j / k + k - 1;
                int dx = i % k - j % k + k - 1;
                bias[((size_t)h * L + i) * L + j] = table[(size_t)h * T + dy * (2 * k - 1) + dx];
            }
    return FWA_ORACLE_OK;
}

/* Adjoint of the gather: dtable[h, idx(i,j)] = sum over (i,j) of dbias[h,i,j]. */
int fwa_oracle_bias_scatter(const double *dbias, double *dtable, int heads, int k)
{
    if (!dbias || !dtable || heads < 1 || k < 1) return FWA_ORACLE_BAD_ARG;
    const int L = k * k, T = (2 * k - 1) * (2 * k - 1);
    for (size_t e = 0; e < (size_t)heads * T; ++e) dtable[e] = 0.0;
    for (int h = 0; h < heads; ++h)
        for (int i = 0; i < L; ++i)
            for (int j = 0; j < L; ++j) {
                int dy = i / k - j / k + k - 1;
                int dx = i % k - j % k + k - 1;
                dtable[(size_t)h * T + dy * (2 * k - 1) + dx] += dbias[((size_t)h * L + i) * L + j];
            }
    return FWA_ORACLE_OK;
}

/*
 * The shift mask written out from per-token region labels (paper Section 2.1 only
 * says that the shifted blocks mask attention between tokens that were not
 * neighbours before the cyclic shift; this is the published Swin rule restated):
 *   mask[w, i, j] = 0 when labels[w, i] == labels[w, j], else `value`.
 *   labels: [nW, L] ints      mask: [nW, L, L]
 */
int fwa_oracle_mask_from_labels(const int *labels, double *mask, int nW, int L, double value)
{
    if (!labels || !mask || nW < 1 || L < 1) return FWA_ORACLE_BAD_ARG;
    for (int w = 0; w < nW; ++w)
        for (int i = 0; i < L; ++i)
            for (int j = 0; j < L; ++j)
                mask[((size_t)w * L + i) * L + j] = labels[w * L + i] == labels[w * L + j] ? 0.0 : value;
    return FWA_ORACLE_OK;
}
