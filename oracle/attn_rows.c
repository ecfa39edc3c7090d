/* Row-by-row causal softmax attention, forward and backward, in fp64 (plain C + OpenMP).
 *
 * TEST INFRASTRUCTURE ONLY: built and called by the tests, the smoke check and the benchmark's
 * cpu_baseline leg; never by the product.  Shares no code with the HIP path.
 *
 * Same definition as oracle/attention.py (Section 3.1, Eq. 3 of the paper and its derivative), written
 * as scalar loops so that single rows / single keys of long sequences can be evaluated one by one:
 *   s_ij = q_i.k_j / sqrt(D) for j <= i;  m_i = max_j s_ij;  l_i = sum_j exp(s_ij - m_i);
 *   p_ij = exp(s_ij - m_i) / l_i;  o_i = sum_j p_ij v_j;  lse_i = m_i + ln l_i
 *   delta_i = dO_i.o_i;  dp_ij = dO_i.v_j;  ds_ij = p_ij (dp_ij - delta_i)
 *   dq_i = (1/sqrt D) sum_{j<=i} ds_ij k_j
 *   dk_j = (1/sqrt D) sum_{h in group} sum_{i>=j} ds_ij q_i;   dv_j = sum_{h in group} sum_{i>=j} p_ij dO_i
 * Inputs are fp32 arrays (values exactly as the device sees them), layout [heads][n][D] contiguous;
 * all arithmetic is fp64.  Indices are 0-based: row i sees keys 0..i.  Query head h reads K/V head
 * h / (Hq / Hkv).
 */
#include <math.h>
#include <stdlib.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int s1f_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double dot(const float *a, const float *b, int d) {
    double s = 0.0;
    for (int t = 0; t < d; ++t) s += (double)a[t] * (double)b[t];
    return s;
}

/* lse_i and (optionally) o_i for one row of one head. p is scratch of i+1 doubles. */
static double row_forward(const float *qi, const float *k, const float *v, int64_t i, int d,
                          double *p, double *o /* may be NULL */) {
    const double scale = 1.0 / sqrt((double)d);
    double m = -INFINITY;
    for (int64_t j = 0; j <= i; ++j) {
        p[j] = dot(qi, k + j * d, d) * scale;
        if (p[j] > m) m = p[j];
    }
    double l = 0.0;
    for (int64_t j = 0; j <= i; ++j) { p[j] = exp(p[j] - m); l += p[j]; }
    for (int64_t j = 0; j <= i; ++j) p[j] /= l;
    if (o) {
        for (int t = 0; t < d; ++t) o[t] = 0.0;
        for (int64_t j = 0; j <= i; ++j)
            for (int t = 0; t < d; ++t) o[t] += p[j] * (double)v[j * d + t];
    }
    return m + log(l);
}

/* Forward for rows [r0, r1) of query head h.  out [(r1-r0)][D], lse [r1-r0]. */
void s1f_oracle_forward_rows(const float *q, const float *k, const float *v, int hq, int hkv, int64_t n,
                             int d, int h, int64_t r0, int64_t r1, double *out, double *lse) {
    const int g = h / (hq / hkv);
    const float *qh = q + (int64_t)h * n * d, *kg = k + (int64_t)g * n * d, *vg = v + (int64_t)g * n * d;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)n);
#pragma omp for schedule(dynamic, 4)
        for (int64_t i = r0; i < r1; ++i)
            lse[i - r0] = row_forward(qh + i * d, kg, vg, i, d, p, out + (i - r0) * d);
        free(p);
    }
}

/* dq for rows [r0, r1) of query head h.  dq [(r1-r0)][D]. */
void s1f_oracle_dq_rows(const float *q, const float *k, const float *v, const float *dout, int hq, int hkv,
                        int64_t n, int d, int h, int64_t r0, int64_t r1, double *dq) {
    const int g = h / (hq / hkv);
    const double scale = 1.0 / sqrt((double)d);
    const float *qh = q + (int64_t)h * n * d, *doh = dout + (int64_t)h * n * d;
    const float *kg = k + (int64_t)g * n * d, *vg = v + (int64_t)g * n * d;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)n);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
        for (int64_t i = r0; i < r1; ++i) {
            row_forward(qh + i * d, kg, vg, i, d, p, o);
            double delta = 0.0;
            for (int t = 0; t < d; ++t) delta += (double)doh[i * d + t] * o[t];
            double *dqi = dq + (i - r0) * d;
            for (int t = 0; t < d; ++t) dqi[t] = 0.0;
            for (int64_t j = 0; j <= i; ++j) {
                const double dp = dot(doh + i * d, vg + j * d, d);
                const double ds = p[j] * (dp - delta);
                for (int t = 0; t < d; ++t) dqi[t] += ds * (double)kg[j * d + t];
            }
            for (int t = 0; t < d; ++t) dqi[t] *= scale;
        }
        free(p); free(o);
    }
}

/* dk, dv for keys [j0, j1) of K/V head g, summed over the query heads of its group and over all
 * rows i >= j.  dk, dv [(j1-j0)][D].  Work: forward of every row i >= j0 of each head in the group
 * (for lse_i and delta_i), then one pass per key. */
void s1f_oracle_dkdv_keys(const float *q, const float *k, const float *v, const float *dout, int hq, int hkv,
                          int64_t n, int d, int g, int64_t j0, int64_t j1, double *dk, double *dv) {
    const int per = hq / hkv;
    const double scale = 1.0 / sqrt((double)d);
    const float *kg = k + (int64_t)g * n * d, *vg = v + (int64_t)g * n * d;
    const int64_t nrow = n - j0;
    double *lse = (double *)malloc(sizeof(double) * (size_t)(nrow * per));
    double *delta = (double *)malloc(sizeof(double) * (size_t)(nrow * per));
    for (int64_t x = 0; x < (j1 - j0) * d; ++x) { dk[x] = 0.0; dv[x] = 0.0; }
    for (int hh = 0; hh < per; ++hh) {
        const int h = g * per + hh;
        const float *qh = q + (int64_t)h * n * d, *doh = dout + (int64_t)h * n * d;
#pragma omp parallel
        {
            double *p = (double *)malloc(sizeof(double) * (size_t)n);
            double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
            for (int64_t i = j0; i < n; ++i) {
                lse[hh * nrow + (i - j0)] = row_forward(qh + i * d, kg, vg, i, d, p, o);
                double dl = 0.0;
                for (int t = 0; t < d; ++t) dl += (double)doh[i * d + t] * o[t];
                delta[hh * nrow + (i - j0)] = dl;
            }
            free(p); free(o);
        }
#pragma omp parallel for schedule(dynamic, 4)
        for (int64_t j = j0; j < j1; ++j) {
            double *dkj = dk + (j - j0) * d, *dvj = dv + (j - j0) * d;
            for (int64_t i = j; i < n; ++i) {
                const double s = dot(qh + i * d, kg + j * d, d) * scale;
                const double p = exp(s - lse[hh * nrow + (i - j0)]);
                const double dp = dot(doh + i * d, vg + j * d, d);
                const double ds = p * (dp - delta[hh * nrow + (i - j0)]);
                for (int t = 0; t < d; ++t) {
                    dvj[t] += p * (double)doh[i * d + t];
                    dkj[t] += scale * ds * (double)qh[i * d + t];
                }
            }
        }
    }
    free(lse); free(delta);
}
