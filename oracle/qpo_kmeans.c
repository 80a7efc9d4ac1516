/*
 * qpo_kmeans — code book construction by Lloyd's algorithm (k-means), plain C, binary64.
 * TEST INFRASTRUCTURE ONLY (see qpo.c).
 *
 * Appendix C.1 / C.2 / C.3.1, "Codebook construction": the scalar tables are 1-D k-means of
 * standard Gaussian samples with k = 2^b clusters, the vector tables 2-D k-means with
 * k = 2^(2b) (Lloyd's algorithm, at most 300 iterations, tolerance 1e-6), the small table of
 * the trellis quantizer 2-D k-means of 2^20 Gaussian pairs with k = 2^tlut_bits.
 *
 * One Lloyd iteration, exactly as defined:
 *   assignment  a[i] = argmin_c |x_i - m_c|^2        (ties: the lowest c)
 *   update      m_c  = mean of { x_i : a[i] = c }     (a cluster without samples keeps m_c)
 * The iteration stops after the update whose total squared movement sum_c |m_c' - m_c|^2 is
 * <= tol, or after max_iter updates.  The initial centres are an input (the paper does not
 * say how its library call was seeded; any start is a valid run of Lloyd's algorithm).
 * Samples and centres are binary64 here; there is no blocking or reordering: samples are
 * visited in index order and sums are plain running sums.
 *
 * Pins (tests/test_oracle_pins.py): two hand-worked iterations; the inertia never increases;
 * a converged 1-D run on Gaussian samples reproduces the paper's NUQ-2 distortion (Table 5,
 * 0.11747) and the closed-form fixed point of Lloyd's iteration on the Gaussian density; a
 * converged 2-D run with 16 centres reproduces the paper's VQ-2 distortion (Table 5, 0.10857);
 * a converged result is a fixed point of assignment + update and no single reassignment of a
 * sample lowers the inertia (brute force on small inputs).
 */
#include <float.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* a[i] for all samples; returns the inertia sum_i |x_i - m_a[i]|^2.  x: [n][d], m: [k][d]. */
double qpo_kmeans_assign(const double *x, int64_t n, int d, const double *m, int k, int32_t *a)
{
    double inertia = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double best = DBL_MAX;
        int bc = 0;
        for (int c = 0; c < k; ++c) {
            double dist = 0.0;
            for (int j = 0; j < d; ++j) {
                double t = x[i * d + j] - m[c * d + j];
                dist += t * t;
            }
            if (dist < best) {
                best = dist;
                bc = c;
            }
        }
        a[i] = bc;
        inertia += best;
    }
    return inertia;
}

/* New centres from an assignment; m_out may not alias m_in.  count[c] = samples of cluster c.
 * Returns the total squared movement. */
double qpo_kmeans_update(const double *x, int64_t n, int d, const int32_t *a, const double *m_in, int k,
                         double *m_out, int64_t *count)
{
    memset(m_out, 0, sizeof(double) * (size_t)k * (size_t)d);
    memset(count, 0, sizeof(int64_t) * (size_t)k);
    for (int64_t i = 0; i < n; ++i) {
        int c = a[i];
        count[c] += 1;
        for (int j = 0; j < d; ++j) m_out[c * d + j] += x[i * d + j];
    }
    double moved = 0.0;
    for (int c = 0; c < k; ++c) {
        for (int j = 0; j < d; ++j) {
            if (count[c] > 0) m_out[c * d + j] /= (double)count[c];
            else m_out[c * d + j] = m_in[c * d + j];
            double t = m_out[c * d + j] - m_in[c * d + j];
            moved += t * t;
        }
    }
    return moved;
}

/* Lloyd's algorithm from the centres in m (in: start, out: result).  Returns the number of
 * updates made; *inertia (optional) receives the inertia of the last assignment, i.e. of the
 * centres before the last update. */
int qpo_kmeans(const double *x, int64_t n, int d, double *m, int k, int max_iter, double tol, double *inertia)
{
    int32_t *a = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    double *m2 = (double *)malloc(sizeof(double) * (size_t)k * (size_t)d);
    int64_t *count = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    int it = 0;
    double last = 0.0;
    while (it < max_iter) {
        last = qpo_kmeans_assign(x, n, d, m, k, a);
        double moved = qpo_kmeans_update(x, n, d, a, m, k, m2, count);
        memcpy(m, m2, sizeof(double) * (size_t)k * (size_t)d);
        ++it;
        if (moved <= tol) break;
    }
    if (inertia) *inertia = last;
    free(a);
    free(m2);
    free(count);
    return it;
}
