/*
 * AdaCons aggregation -- float64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP
 * path, and nothing in the product path may call it: only the test-suite, the
 * smoke check and the CPU-baseline leg of the benchmark load it.
 *
 * AdaCons (arXiv 2411.03742) is a heuristic defined by its steps, so the
 * oracle is those steps, in the paper's order, in IEEE double arithmetic on
 * exactly-widened inputs (fp32 -> fp64, bf16 -> fp64), plain loops, no
 * fast-math.  The only structuring beyond the formulas: the length-d sums are
 * taken over fixed chunks of ORACLE_CHUNK columns, each chunk summed left to
 * right, chunk results added in chunk order -- so that OpenMP threads can share
 * the chunks without the result depending on the thread count.
 *
 * Notation: G is N x d row-major, row i = worker i's gradient g_i (the paper's
 * subspace matrix P_t of Sec. 3.1, transposed, columns not yet normalised).
 * K = G G^T,  q_i = K_ii = ||g_i||^2,  r_i = sum_j K_ij = <g_i, sum_j g_j>
 * = N <g_i, gbar> with gbar the mean gradient (Sec. 3.2, Monte-Carlo mean).
 *
 * Steps of one aggregation (state: m in R^N held in sorted order, t calls):
 *   O1  K_ij = sum_k G[i,k] G[j,k]                 Eq. 7 (third line), Eq. 8 double sum
 *   O2  q_i = K_ii ; r_i = sum_j K_ij (j ascending)
 *   O3  a_i = r_i / (N sqrt(q_i))                   Eq. 7: <g_i, gbar>/||g_i||,
 *       sign taken positive for a descent direction used as w - eta*psi (Eq. 4)
 *   O4  pi = stable ascending argsort of a ; s_k = a_pi(k)      sorting operator S, Eq. 11
 *   O5  m_k <- beta m_k + (1-beta) s_k ; a~_pi(k) = m_k         Eq. 11 (S^-1 redistributes)
 *   O6  c_i = a~_i / sqrt(q_i)     second 1/||g_i|| of the column-normalised
 *       subspace matrix (Sec. 3.2) -- the ||g_i||^2 of Eq. 8 and of gamma_i under Eq. 12
 *   O7  gamma_i = c_i / sum_k c_k  (weights sum to one, Sec. 3.4, Eq. 12-13)
 *       out[k] = sum_i gamma_i G[i,k]               Eq. 12
 * Flags (the ablation columns of Table 2): momentum off skips O4-O5 (a~ = a);
 * normalise off stops at gamma_i = c_i (lambda = 1, Eq. 8).
 * Two documented variants, off by default:
 *   INDEX_EMA    O4-O5 without the sort: m_i <- beta m_i + (1-beta) a_i, a~_i = m_i -- the
 *                momentum of Eq. 10, which Sec. 3.3 then replaces by Eq. 11 because it ties a
 *                coefficient to the worker's index.
 *   LAMBDA_EQ13  O7 with lambda as Eq. 13 prints it, 1 / sum_k (a~_k): the coefficients on the
 *                column-normalised subspace matrix, gamma_i ||g_i||, then sum to one, not the
 *                weights on the raw gradients (see the first reading below).
 *
 * Readings where the paper is silent or at odds with itself:
 *   - Eq. 13 prints ||g_i|| where the weight gamma_i it normalises has
 *     ||g_i||^2; the weights applied to the raw gradients are the ones made to
 *     sum to one here (only that reading reduces identical gradients to plain
 *     averaging, as Sec. 3.2 requires).
 *   - Sort direction and ties are not stated: ascending, ties to the lower
 *     worker index first (rank by counting).
 *   - Initial state m = 0, no bias correction (a common factor, removed by O7).
 *   - Degenerate inputs: q_i = 0 gives a_i = c_i = 0; a non-finite statistic,
 *     or |sum c| <= 1e-12 sum|c|, falls back to gamma_i = 1/N (the method's own
 *     collapse limit, Sec. 5.4) and raises a flag; the EMA state is left
 *     untouched when a statistic is non-finite.
 *
 * Parity pins (tests/test_oracle_pins.py): O1-O2 against the library matmul;
 * O3 against central differences of the subspace objective (Eq. 5) on a
 * quadratic; O6 (lambda = 1) against the explicit d x d preconditioner of
 * Eq. 9; O4-O5 against the closed form of the recurrence, the step-1 identity
 * and permutation invariance with persisting state; O7 against sum-to-one, the
 * identical / orthogonal / N=1 / N=2 closed forms; the INDEX_EMA switch against the plain
 * per-index recurrence and its dependence on the worker order; the LAMBDA_EQ13 switch against
 * sum_i gamma_i ||g_i|| = 1 and the unit vector it yields for identical gradients.  No function
 * is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_CHUNK 65536

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum {
    ORACLE_FLAG_MOMENTUM = 1u,
    ORACLE_FLAG_NORMALIZE = 2u,
    ORACLE_FLAG_INDEX_EMA = 4u,   /* with MOMENTUM: the EMA of Eq. 10, coupled to the worker index */
    ORACLE_FLAG_LAMBDA_EQ13 = 8u  /* with NORMALIZE: lambda exactly as Eq. 13 prints it */
};
enum {
    ORACLE_NUM_ZERO_NORM = 1u,        /* some q_i == 0 */
    ORACLE_NUM_NONFINITE = 2u,        /* NaN/Inf reached the statistics */
    ORACLE_NUM_UNIFORM_FALLBACK = 4u  /* gamma replaced by 1/N */
};

/* Number of OpenMP threads later calls use (results do not depend on it); n < 1 is ignored. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* bf16 is the upper half of an IEEE fp32: widening is exact. */
static double bf16_to_double(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double dot_f32(const float *x, const float *y, int64_t n)
{
    double acc = 0.0;
    for (int64_t k = 0; k < n; ++k)
        acc += (double)x[k] * (double)y[k];
    return acc;
}

static double dot_bf16(const uint16_t *x, const uint16_t *y, int64_t n)
{
    double acc = 0.0;
    for (int64_t k = 0; k < n; ++k)
        acc += bf16_to_double(x[k]) * bf16_to_double(y[k]);
    return acc;
}

/* O1: K = G G^T, full N x N (both triangles written). */
int oracle_gram(const void *G, int N, int64_t d, int dtype, double *K)
{
    if (!G || !K || N < 1 || d < 1 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16))
        return 1;
    const int64_t nchunks = (d + ORACLE_CHUNK - 1) / ORACLE_CHUNK;
    const size_t nn = (size_t)N * (size_t)N;
    double *part = (double *)calloc((size_t)nchunks * nn, sizeof(double));
    if (!part)
        return 2;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t c = 0; c < nchunks; ++c) {
        const int64_t k0 = c * ORACLE_CHUNK;
        const int64_t len = (d - k0 < ORACLE_CHUNK) ? d - k0 : ORACLE_CHUNK;
        double *pc = part + (size_t)c * nn;
        for (int i = 0; i < N; ++i) {
            for (int j = i; j < N; ++j) {
                double v;
                if (dtype == ORACLE_F32) {
                    const float *g = (const float *)G;
                    v = dot_f32(g + (size_t)i * d + k0, g + (size_t)j * d + k0, len);
                } else {
                    const uint16_t *g = (const uint16_t *)G;
                    v = dot_bf16(g + (size_t)i * d + k0, g + (size_t)j * d + k0, len);
                }
                pc[(size_t)i * N + j] = v;
            }
        }
    }

    for (int i = 0; i < N; ++i) {
        for (int j = i; j < N; ++j) {
            double acc = 0.0;
            for (int64_t c = 0; c < nchunks; ++c)
                acc += part[(size_t)c * nn + (size_t)i * N + j];
            K[(size_t)i * N + j] = acc;
            K[(size_t)j * N + i] = acc;
        }
    }
    free(part);
    return 0;
}

/*
 * O3-O7 (weights) from the per-worker statistics q_i = ||g_i||^2 and r_i = <g_i, sum_j g_j>
 * (what each worker of Algorithm 1 holds after step 1 and shares in step 2), updating the
 * sorted-order EMA state m[N] and the call counter *t.  a_raw, a_smooth may be NULL.
 */
int oracle_coefficients_from_stats(const double *q, const double *r, int N, double beta, unsigned flags,
                                   double *m, int64_t *t,
                                   double *gamma, double *a_raw, double *a_smooth,
                                   unsigned *numeric_flags)
{
    if (!q || !r || !m || !t || !gamma || N < 1 || !(beta >= 0.0 && beta < 1.0))
        return 1;
    unsigned nf = 0;
    double *a = (double *)malloc(sizeof(double) * (size_t)N * 3);
    if (!a)
        return 2;
    double *as = a + N, *c = as + N;

    int finite = 1;
    for (int i = 0; i < N; ++i)
        if (!isfinite(q[i]) || !isfinite(r[i]))
            finite = 0;

    /* O3 */
    for (int i = 0; i < N; ++i) {
        if (q[i] > 0.0) {
            a[i] = r[i] / ((double)N * sqrt(q[i]));
        } else {
            a[i] = 0.0;
            if (finite)
                nf |= ORACLE_NUM_ZERO_NORM;
        }
    }

    *t += 1;

    if (!finite) {
        /* statistics poisoned: state untouched, uniform weights */
        nf |= ORACLE_NUM_NONFINITE | ORACLE_NUM_UNIFORM_FALLBACK;
        for (int i = 0; i < N; ++i) {
            gamma[i] = 1.0 / (double)N;
            if (a_raw) a_raw[i] = a[i];
            if (a_smooth) a_smooth[i] = a[i];
        }
        if (numeric_flags) *numeric_flags = nf;
        free(a);
        return 0;
    }

    /* O4-O5 */
    if ((flags & ORACLE_FLAG_MOMENTUM) && (flags & ORACLE_FLAG_INDEX_EMA)) {
        /* Eq. 10: state entry i belongs to worker i */
        for (int i = 0; i < N; ++i) {
            m[i] = beta * m[i] + (1.0 - beta) * a[i];
            as[i] = m[i];
        }
    } else if (flags & ORACLE_FLAG_MOMENTUM) {
        for (int i = 0; i < N; ++i) {
            int rank = 0; /* position of worker i in the stable ascending order */
            for (int j = 0; j < N; ++j)
                if (a[j] < a[i] || (a[j] == a[i] && j < i))
                    ++rank;
            m[rank] = beta * m[rank] + (1.0 - beta) * a[i];
            as[i] = m[rank];
        }
    } else {
        for (int i = 0; i < N; ++i)
            as[i] = a[i];
    }

    /* O6 */
    for (int i = 0; i < N; ++i)
        c[i] = (q[i] > 0.0) ? as[i] / sqrt(q[i]) : 0.0;

    /* O7 (weights) */
    if (flags & ORACLE_FLAG_NORMALIZE) {
        /* what is made to sum to one: the weights c, or (Eq. 13 as printed) the coefficients a~ */
        const double *w = (flags & ORACLE_FLAG_LAMBDA_EQ13) ? as : c;
        double s = 0.0, sabs = 0.0;
        for (int i = 0; i < N; ++i) {
            s += w[i];
            sabs += fabs(w[i]);
        }
        if (!isfinite(s) || sabs == 0.0 || fabs(s) <= 1e-12 * sabs) {
            nf |= ORACLE_NUM_UNIFORM_FALLBACK;
            for (int i = 0; i < N; ++i)
                gamma[i] = 1.0 / (double)N;
        } else {
            for (int i = 0; i < N; ++i)
                gamma[i] = c[i] / s;
        }
    } else {
        for (int i = 0; i < N; ++i)
            gamma[i] = c[i];
    }

    for (int i = 0; i < N; ++i) {
        if (a_raw) a_raw[i] = a[i];
        if (a_smooth) a_smooth[i] = as[i];
    }
    if (numeric_flags) *numeric_flags = nf;
    free(a);
    return 0;
}

/*
 * O2-O7 (coefficient part): from K to gamma.  O2 reads the statistics off the Gram matrix
 * (its diagonal and its row sums), the rest is oracle_coefficients_from_stats.
 */
int oracle_coefficients(const double *K, int N, double beta, unsigned flags,
                        double *m, int64_t *t,
                        double *gamma, double *a_raw, double *a_smooth,
                        unsigned *numeric_flags)
{
    if (!K || N < 1)
        return 1;
    double *q = (double *)malloc(sizeof(double) * (size_t)N * 2);
    if (!q)
        return 2;
    double *r = q + N;
    /* O2 */
    for (int i = 0; i < N; ++i) {
        q[i] = K[(size_t)i * N + i];
        double acc = 0.0;
        for (int j = 0; j < N; ++j)
            acc += K[(size_t)i * N + j];
        r[i] = acc;
    }
    int rc = oracle_coefficients_from_stats(q, r, N, beta, flags, m, t, gamma, a_raw, a_smooth, numeric_flags);
    free(q);
    return rc;
}

static double elem(const void *G, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)G)[idx];
    return bf16_to_double(((const uint16_t *)G)[idx]);
}

/* O7 (combination): out[k] = sum_i gamma_i G[i,k], i ascending, double out. */
int oracle_weighted_sum(const void *G, int N, int64_t d, int dtype,
                        const double *gamma, double *out)
{
    if (!G || !gamma || !out || N < 1 || d < 1 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16))
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < d; ++k) {
        double acc = 0.0;
        for (int i = 0; i < N; ++i)
            acc += gamma[i] * elem(G, dtype, (size_t)i * d + k);
        out[k] = acc;
    }
    return 0;
}

/* Same, only at the n listed columns idx[0..n) (for full-size sampled checks). */
int oracle_weighted_sum_at(const void *G, int N, int64_t d, int dtype,
                           const double *gamma, const int64_t *idx, int64_t n,
                           double *out)
{
    if (!G || !gamma || !out || !idx || N < 1 || d < 1 || n < 0 ||
        (dtype != ORACLE_F32 && dtype != ORACLE_BF16))
        return 1;
    for (int64_t s = 0; s < n; ++s) {
        const int64_t k = idx[s];
        if (k < 0 || k >= d)
            return 1;
        double acc = 0.0;
        for (int i = 0; i < N; ++i)
            acc += gamma[i] * elem(G, dtype, (size_t)i * d + k);
        out[s] = acc;
    }
    return 0;
}

/*
 * One whole aggregation, O1-O7.  K_out (N*N), a_raw, a_smooth may be NULL.
 * out may be NULL (coefficients only).
 */
int oracle_aggregate(const void *G, int N, int64_t d, int dtype,
                     double beta, unsigned flags, double *m, int64_t *t,
                     double *out, double *gamma, double *a_raw, double *a_smooth,
                     double *K_out, unsigned *numeric_flags)
{
    if (N < 1)
        return 1;
    double *K = (double *)malloc(sizeof(double) * (size_t)N * (size_t)N);
    if (!K)
        return 2;
    int rc = oracle_gram(G, N, d, dtype, K);
    if (!rc)
        rc = oracle_coefficients(K, N, beta, flags, m, t, gamma, a_raw, a_smooth, numeric_flags);
    if (!rc && out)
        rc = oracle_weighted_sum(G, N, d, dtype, gamma, out);
    if (!rc && K_out)
        memcpy(K_out, K, sizeof(double) * (size_t)N * (size_t)N);
    free(K);
    return rc;
}
