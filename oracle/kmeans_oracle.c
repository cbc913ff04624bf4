/*
 * Reference ("oracle") implementation of one K-Means (Lloyd) iteration, in plain C and fp64.
 *
 * THIS IS TEST INFRASTRUCTURE, like glm_oracle.c beside it: only the tests, the smoke check and
 * the benchmark's CPU baseline use it; it shares nothing with the GPU library.
 *
 * What it follows.  The paper names K-Means among the unsupervised jobs it schedules (Sec. 3,
 * "Setup") and Expectation Maximization among the iterative solvers whose per-iteration quality
 * it tracks (Sec. 1, "ML training is typically iterative with diminishing returns").  It prints
 * no formula and no value for it, so against paper-printed values this oracle is "parity
 * unpinned"; hand examples, library routines and invariants in the CPU tests pin it instead.
 * The textbook definition of the iteration, for points x_i (rows of X) and centroids c_k:
 *
 *   distance     d_ik = sum_j (x_ij - c_kj)^2
 *   assignment   a_i  = the smallest k that attains min_k d_ik
 *   loss         L    = (1/N) sum_i d_{i, a_i}              (at the centroids that enter)
 *   update       c_k <- mean of the x_i with a_i = k;  a centroid with no point keeps its value
 *
 * X holds the fp32 bit patterns the GPU reads, widened where used; everything else is double.
 * Points in index order, centroids in index order, coordinates in index order.
 */
#include <stdint.h>
#include <stdlib.h>

/*
 * For every point: its assignment, the squared distance to its centroid (best) and to the
 * nearest other centroid (second; +inf coded as -1 when K == 1).  Rows are independent, so the
 * loop may run in parallel without changing any value.
 */
int oracle_kmeans_assign(const float *X, int64_t N, int32_t D, const double *C, int32_t K,
                         int32_t *assign, double *best, double *second)
{
    if (N < 1 || D < 1 || K < 1) return -1;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < N; ++i) {
        const float *x = X + i * (int64_t)D;
        int32_t a = -1;
        double b = 0.0, s = -1.0;
        for (int32_t k = 0; k < K; ++k) {
            const double *c = C + (int64_t)k * D;
            double d = 0.0;
            for (int32_t j = 0; j < D; ++j) {
                double t = (double)x[j] - c[j];
                d += t * t;
            }
            if (a < 0) { a = k; b = d; }
            else if (d < b) { s = b; b = d; a = k; }
            else if (s < 0.0 || d < s) { s = d; }
        }
        assign[i] = a;
        best[i] = b;
        if (second) second[i] = s;
    }
    return 0;
}

/*
 * One iteration from C (updated in place).  loss_out receives L at the entering centroids,
 * assign [N] the assignments, counts [K] the cluster sizes.
 */
int oracle_kmeans_step(const float *X, int64_t N, int32_t D, double *C, int32_t K,
                       int32_t *assign, int64_t *counts, double *loss_out)
{
    if (N < 1 || D < 1 || K < 1) return -1;
    double *best = (double *)malloc(sizeof(double) * (size_t)N);
    double *sums = (double *)calloc((size_t)K * (size_t)D, sizeof(double));
    if (!best || !sums) { free(best); free(sums); return -1; }
    int rc = oracle_kmeans_assign(X, N, D, C, K, assign, best, NULL);
    if (rc != 0) { free(best); free(sums); return rc; }
    double S = 0.0;
    for (int32_t k = 0; k < K; ++k) counts[k] = 0;
    for (int64_t i = 0; i < N; ++i) {
        S += best[i];
        int32_t a = assign[i];
        counts[a] += 1;
        for (int32_t j = 0; j < D; ++j) sums[(int64_t)a * D + j] += (double)X[i * (int64_t)D + j];
    }
    *loss_out = S / (double)N;
    for (int32_t k = 0; k < K; ++k) {
        if (counts[k] == 0) continue;
        for (int32_t j = 0; j < D; ++j) C[(int64_t)k * D + j] = sums[(int64_t)k * D + j] / (double)counts[k];
    }
    free(best); free(sums);
    return 0;
}
