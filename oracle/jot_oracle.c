/*
 * CPU oracle for the JoT token-finalization pass -- row statistics.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  Nothing on the product path may call it;
 * it shares no code, header, table or helper with the HIP implementation.
 *
 * What it computes, per logit row (paper Section 4.1, "Confidence Metric",
 * Eq. 2 and the first two computations of Algorithm 1):
 *
 *     pi   = softmax(l)                 (no temperature)
 *     p1   = largest entry of pi,  p2 = second largest entry (of the multiset)
 *     a    = argmax_v pi_v              (smallest index among equal maxima)
 *
 * The row is widened exactly to double (fp32 and bf16 are subsets of double)
 * and everything is evaluated in double, in plain index order:
 *
 *     m1 = max_v l_v,  a = first v with l_v = m1,  m2 = max_{v != a} l_v
 *     S  = sum_v exp(l_v - m1)          =>  p1 = 1/S,  p2 = exp(m2 - m1)/S
 *
 * softmax is strictly increasing in the logit, so the top-2 of pi are the
 * top-2 of l; jot_oracle_softmax_row() returns the whole vector pi so the
 * tests can check that statement (and sum(pi) = 1) directly.
 *
 * Rows that contain NaN or +inf, or whose entries are all -inf, have no
 * softmax; they are reported with status 1 and S = NaN (the caller must not
 * finalize them).  -inf entries are ordinary: they contribute exp(-inf) = 0.
 * Every other row has a softmax, whatever the size of its entries: the
 * definition only involves differences from the row maximum.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static double widen(const void *row, int dtype, int64_t v)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)row)[v];
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t bits = (uint32_t)((const uint16_t *)row)[v] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* One row.  Returns 0 if the row has a softmax, 1 otherwise. */
static int row_stats(const void *row, int dtype, int32_t V,
                     int32_t *a, double *m1, double *m2, double *S)
{
    int bad = 0;
    double best = -INFINITY;
    int32_t arg = 0;
    for (int32_t v = 0; v < V; v++) {
        double x = widen(row, dtype, v);
        if (isnan(x) || x == INFINITY)
            bad = 1;
        if (x > best) {          /* strict: the first maximum keeps the index */
            best = x;
            arg = v;
        }
    }
    double second = -INFINITY;
    for (int32_t v = 0; v < V; v++) {
        if (v == arg)
            continue;
        double x = widen(row, dtype, v);
        if (x > second)
            second = x;
    }
    *a = arg;
    *m1 = best;
    *m2 = second;
    if (bad || best == -INFINITY) {
        *S = NAN;
        return 1;
    }
    double sum = 0.0;
    for (int32_t v = 0; v < V; v++)
        sum += exp(widen(row, dtype, v) - best);
    *S = sum;
    return 0;
}

/*
 * rows      : n_rows rows, row k starts at element k*row_stride
 * dtype     : 0 = fp32, 1 = bf16 (stored as uint16)
 * outputs   : arrays of n_rows; status[k] = 0 ok / 1 no softmax
 * n_threads : OpenMP threads over rows (<= 0: library default)
 */
void jot_oracle_row_stats(const void *rows, int dtype, int64_t n_rows,
                          int64_t row_stride, int32_t V,
                          int32_t *a, double *m1, double *m2, double *S,
                          int32_t *status, int n_threads)
{
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int64_t k = 0; k < n_rows; k++) {
        const char *row = (const char *)rows + (size_t)k * (size_t)row_stride * esz;
        status[k] = row_stats(row, dtype, V, &a[k], &m1[k], &m2[k], &S[k]);
    }
}

/* Whole probability vector of one row, pi_v = exp(l_v - m1) / S (for tests). */
int jot_oracle_softmax_row(const void *row, int dtype, int32_t V, double *pi)
{
    int32_t a;
    double m1, m2, S;
    int st = row_stats(row, dtype, V, &a, &m1, &m2, &S);
    for (int32_t v = 0; v < V; v++)
        pi[v] = st ? NAN : exp(widen(row, dtype, v) - m1) / S;
    return st;
}

/*
 * Sampling-based finalization (Section 4.1, "Early-Exit Decision": the finalized token may be
 * sampled from pi instead of taking the argmax).  Inverse-CDF sampling with a uniform number u
 * in [0, 1) supplied by the caller: the token is the first index v whose cumulative probability
 * pi_0 + ... + pi_v exceeds u.  Section 4.1 only says that the token may be sampled from pi; the
 * reading taken for the upper edge: the cumulative probability reaches 1 at the last index with a
 * non-zero probability, so that index is returned for u >= 1 (not a valid draw from [0, 1), but
 * defined -- in double the rounded running sum may or may not exceed 1.0, which must not decide),
 * and also if rounding leaves the total just below u.  Also reports the cumulative probability just below and
 * just above the chosen token (so a test can tell how far u is from either edge).
 * Returns -1 for a row without a softmax.
 */
int32_t jot_oracle_sample_row(const void *row, int dtype, int32_t V, double u,
                              double *cdf_below, double *cdf_above)
{
    int32_t a;
    double m1, m2, S;
    if (row_stats(row, dtype, V, &a, &m1, &m2, &S))
        return -1;
    double cum = 0.0;
    int32_t last = -1;
    for (int32_t v = 0; v < V; v++) {
        double pv = exp(widen(row, dtype, v) - m1) / S;
        if (pv > 0.0)
            last = v;
        if (u < 1.0 && cum + pv > u) {
            *cdf_below = cum;
            *cdf_above = cum + pv;
            return v;
        }
        cum += pv;
    }
    *cdf_below = cum;
    *cdf_above = cum;
    return last;
}

/*
 * Stability signal between consecutive steps (the per-token rule Section 2 attributes to KLASS:
 * the KL divergence between the distributions of consecutive steps identifies stable
 * predictions).  D( pi_now || pi_prev ) = sum_v pi_now(v) * ( log pi_now(v) - log pi_prev(v) ),
 * with 0 * log 0 = 0, and +inf if pi_prev(v) = 0 < pi_now(v) for some v.
 * Returns NaN if either row has no softmax.
 */
double jot_oracle_kl_row(const void *row_now, const void *row_prev, int dtype, int32_t V)
{
    int32_t a;
    double m1, m2, S, pm1, pm2, pS;
    if (row_stats(row_now, dtype, V, &a, &m1, &m2, &S) || row_stats(row_prev, dtype, V, &a, &pm1, &pm2, &pS))
        return NAN;
    const double lse = m1 + log(S), plse = pm1 + log(pS);
    double kl = 0.0;
    for (int32_t v = 0; v < V; v++) {
        const double x = widen(row_now, dtype, v), y = widen(row_prev, dtype, v);
        const double pv = exp(x - m1) / S;
        if (pv > 0.0) {
            if (y == -INFINITY)
                return INFINITY;
            kl += pv * ((x - lse) - (y - plse));
        }
    }
    return kl;
}

/* jot_oracle_kl_row over the rows selected by do_row (others get NaN); rows are independent,
 * so threads take whole rows. */
void jot_oracle_kl_rows(const void *rows_now, const void *rows_prev, int dtype, int64_t n_rows, int32_t V,
                        const uint8_t *do_row, double *out, int n_threads)
{
    const int64_t esz = dtype == 0 ? 4 : 2;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads > 0 ? n_threads : 1)
    for (int64_t k = 0; k < n_rows; k++)
        out[k] = do_row[k] ? jot_oracle_kl_row((const char *)rows_now + k * V * esz,
                                               (const char *)rows_prev + k * V * esz, dtype, V)
                           : NAN;
}
