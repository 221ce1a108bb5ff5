/*
 * CPU oracle for the clustering stage of ClusComp (Section 3.1 of the paper): Lloyd k-means over the
 * length-d sub-vectors of a weight matrix, and the codebook-gather reconstruction.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. It is a plain, slow, by-the-definition implementation
 * that the tests, the smoke check and the benchmark's cpu_baseline leg compare the HIP library
 * against. It shares no code, header, table or helper with the HIP library and is never called by it.
 *
 * Arithmetic: inputs are fp32; every difference, square, sum and mean is taken in fp64; a centroid
 * component is rounded to fp32 exactly once (after the division by the cluster size).
 *
 * Readings of points the paper leaves open (each is also listed in the design notes):
 *   - E-step ties (the E-step set uses "<=", so a tied vector belongs to several clusters):
 *     the lowest centroid index wins.
 *   - Empty cluster in the M-step (division by |C_j| = 0): the centroid keeps its previous value.
 *   - The returned codes q_i are the argmin over the RETURNED codebook (the definition of q in
 *     Section 3.1), so a fit of T iterations performs T (assign, update) pairs and one last assign.
 *   - All N vectors take part in every iteration; exactly T iterations; no early stop.
 *
 * Pins (tests/test_oracle_*.py): exact rational brute force on tiny inputs, a kd-tree library
 * query, grouped means by an independent numpy route, monotone inertia, K=1 / K=N closed forms,
 * zero inertia when every distinct vector is a centroid, a library Lloyd run on tie-free data,
 * and the bits-per-parameter values printed in Table 1 / Eq. 1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Squared Euclidean distance ||x - c||^2, the quantity inside the k-means objective (Section 3.1). */
static double sqdist(const float *x, const float *c, int d)
{
    double s = 0.0;
    for (int j = 0; j < d; ++j) {
        double t = (double)x[j] - (double)c[j];
        s += t * t;
    }
    return s;
}

/*
 * E-step (Section 3.1): for every vector the nearest centroid k1 and its distance D1, plus the
 * runner-up (k2, D2) so that callers can tell how close to a tie the decision was.
 * Ties go to the lowest index. With K == 1 the runner-up is (UINT32_MAX, +inf).
 * k2, D1, D2 may be NULL.
 */
void oracle_assign_top2(const float *X, int64_t N, int d, const float *C, int64_t K,
                        uint32_t *k1, double *D1, uint32_t *k2, double *D2)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const float *x = X + i * d;
        double b1 = INFINITY, b2 = INFINITY;
        uint32_t a1 = UINT32_MAX, a2 = UINT32_MAX;
        for (int64_t k = 0; k < K; ++k) {
            double D = sqdist(x, C + k * d, d);
            if (D < b1) {
                b2 = b1; a2 = a1;
                b1 = D;  a1 = (uint32_t)k;
            } else if (D < b2) {
                b2 = D;  a2 = (uint32_t)k;
            }
        }
        k1[i] = a1;
        if (D1) D1[i] = b1;
        if (k2) k2[i] = a2;
        if (D2) D2[i] = b2;
    }
}

/*
 * M-step (Section 3.1): c_k <- mean of the vectors assigned to k. Sums run over i in increasing
 * order in fp64. A cluster with no member keeps prev[k]. counts may be NULL.
 * out may alias prev.
 */
void oracle_update(const float *X, int64_t N, int d, const uint32_t *idx, int64_t K,
                   const float *prev, float *out, uint32_t *counts)
{
    double *sum = (double *)calloc((size_t)K * d, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    for (int64_t i = 0; i < N; ++i) {
        int64_t k = idx[i];
        for (int j = 0; j < d; ++j) sum[k * d + j] += (double)X[i * d + j];
        cnt[k] += 1;
    }
    for (int64_t k = 0; k < K; ++k) {
        for (int j = 0; j < d; ++j) {
            if (cnt[k] > 0) out[k * d + j] = (float)(sum[k * d + j] / (double)cnt[k]);
            else            out[k * d + j] = prev[k * d + j];
        }
        if (counts) counts[k] = (uint32_t)cnt[k];
    }
    free(sum);
    free(cnt);
}

/* The k-means objective for a given (codebook, codes): sum_i ||x_i - c_{idx_i}||^2, in fp64, i ascending. */
double oracle_inertia(const float *X, int64_t N, int d, const float *C, const uint32_t *idx)
{
    double J = 0.0;
    for (int64_t i = 0; i < N; ++i) J += sqdist(X + i * d, C + (int64_t)idx[i] * d, d);
    return J;
}

/* Reconstruction (Section 3.1; the gather in the paper's layer listing): out_i = c_{idx_i}. */
void oracle_decode(const float *C, int d, const uint32_t *idx, int64_t N, float *out)
{
    for (int64_t i = 0; i < N; ++i)
        memcpy(out + i * d, C + (int64_t)idx[i] * d, (size_t)d * sizeof(float));
}

/*
 * Lloyd's algorithm as the paper states it: iters x (E-step, M-step) from init, then the codes and
 * the objective for the returned codebook. history (nullable, iters+1 doubles) receives the
 * objective seen by each E-step: history[t] is measured against the centroids entering iteration t,
 * history[iters] against the returned ones.
 */
void oracle_kmeans_fit(const float *X, int64_t N, int d, int64_t K, int iters, const float *init,
                       float *C, uint32_t *idx, double *inertia, double *history)
{
    double *D1 = (double *)malloc((size_t)N * sizeof(double));
    if (C != init) memcpy(C, init, (size_t)K * d * sizeof(float));
    for (int t = 0; t <= iters; ++t) {
        oracle_assign_top2(X, N, d, C, K, idx, D1, NULL, NULL);
        double J = 0.0;
        for (int64_t i = 0; i < N; ++i) J += D1[i];
        if (history) history[t] = J;
        if (t == iters) { *inertia = J; break; }
        oracle_update(X, N, d, idx, K, C, C, NULL);
    }
    free(D1);
}
