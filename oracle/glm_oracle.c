/*
 * Reference ("oracle") implementation of one full-batch gradient-descent
 * iteration of a generalized linear model, in plain C and fp64.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists only so that tests, the smoke check
 * and the benchmark's CPU baseline can compare the GPU library against an
 * independent, slow and obviously correct computation.  It shares no code,
 * headers, constants or helpers with the GPU library, and the GPU library
 * never calls it.
 *
 * What it follows.  The paper (Sec. 2, "Normalizing Quality Metrics") says
 * only that an iterative training job evaluates its loss function in every
 * iteration, names gradient descent as the first-order optimiser whose
 * convergence its predictor models (Sec. 2, class I), and lists logistic
 * regression, SVM and linear regression among the jobs it schedules (Sec. 3,
 * "Setup").  It prints no formula, no loss value and no worked iteration, so
 * against values printed by the paper this oracle is "parity unpinned"; what
 * pins it instead are closed forms, finite differences, the normal equations
 * and convexity invariants in the CPU test-suite.  The formulas below are the
 * textbook definitions of the three models:
 *
 *   margin      z_i = sum_j X[i][j] * w[j]
 *   logistic    l_i = softplus(z_i) - y_i z_i       r_i = sigmoid(z_i) - y_i     y in {0,1}
 *   hinge       l_i = max(0, 1 - y_i z_i)           r_i = -y_i if 1 - y_i z_i > 0 else 0   y in {-1,+1}
 *   squared     l_i = (z_i - y_i)^2 / 2             r_i = z_i - y_i              y real
 *   loss        L   = (1/N) sum_i l_i + (lambda/2) sum_j w[j]^2
 *   gradient    g_j = (1/N) sum_i X[i][j] r_i + lambda w[j]
 *   update      w_j <- w_j - eta g_j
 *
 * X and y are given as the very fp32 bit patterns the GPU reads; each element
 * is widened to double where it is used.  All arithmetic is double.  Rows are
 * visited in index order, columns in index order, nothing is blocked or
 * fused beyond what the definition states.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_LOGISTIC = 0, ORACLE_HINGE = 1, ORACLE_SQUARED = 2 };

/* Per-sample loss and residual d(l)/d(z) for one margin z and label y. */
static void sample_loss_residual(int loss, double z, double y, double *l, double *r)
{
    if (loss == ORACLE_LOGISTIC) {
        /* softplus(z) = log(1 + e^z), written so that neither branch overflows */
        double sp = (z > 0.0 ? z : 0.0) + log1p(exp(-fabs(z)));
        double sig;
        if (z >= 0.0) {
            sig = 1.0 / (1.0 + exp(-z));
        } else {
            double e = exp(z);
            sig = e / (1.0 + e);
        }
        *l = sp - y * z;
        *r = sig - y;
    } else if (loss == ORACLE_HINGE) {
        double m = 1.0 - y * z;
        if (m > 0.0) { *l = m;   *r = -y;  }
        else         { *l = 0.0; *r = 0.0; }
    } else {
        double d = z - y;
        *l = 0.5 * d * d;
        *r = d;
    }
}

/*
 * Data-term sums over rows [i0, i1):  S = sum_i l_i,  s[j] = sum_i X[i][j] r_i.
 * s must hold D doubles; it is overwritten.
 */
static void data_sums(int loss, const float *X, const float *y, int64_t i0, int64_t i1,
                      int32_t D, const double *w, double *S, double *s)
{
    double acc = 0.0;
    for (int32_t j = 0; j < D; ++j) s[j] = 0.0;
    for (int64_t i = i0; i < i1; ++i) {
        const float *row = X + i * (int64_t)D;
        double z = 0.0;
        for (int32_t j = 0; j < D; ++j) z += (double)row[j] * w[j];
        double l, r;
        sample_loss_residual(loss, z, (double)y[i], &l, &r);
        acc += l;
        for (int32_t j = 0; j < D; ++j) s[j] += (double)row[j] * r;
    }
    *S = acc;
}

/*
 * Loss and gradient at w.  g must hold D doubles.  Returns 0, or -1 on bad
 * arguments / allocation failure.
 */
int oracle_loss_grad(int loss, const float *X, const float *y, int64_t N, int32_t D,
                     const double *w, double lambda, double *L_out, double *g)
{
    if (loss < 0 || loss > 2 || N < 1 || D < 1) return -1;
    double S;
    data_sums(loss, X, y, 0, N, D, w, &S, g);
    double ww = 0.0;
    for (int32_t j = 0; j < D; ++j) ww += w[j] * w[j];
    *L_out = S / (double)N + 0.5 * lambda * ww;
    for (int32_t j = 0; j < D; ++j) g[j] = g[j] / (double)N + lambda * w[j];
    return 0;
}

/*
 * The same quantities with the row range cut into `chunks` equal contiguous
 * pieces that are evaluated by data_sums() independently (in parallel when
 * compiled with OpenMP) and then added in chunk order.  Mathematically
 * identical to oracle_loss_grad; only the association of the fp64 row sums
 * differs, and the result does not depend on the number of threads.
 */
int oracle_loss_grad_chunked(int loss, const float *X, const float *y, int64_t N, int32_t D,
                             const double *w, double lambda, int32_t chunks,
                             double *L_out, double *g)
{
    if (loss < 0 || loss > 2 || N < 1 || D < 1 || chunks < 1) return -1;
    if ((int64_t)chunks > N) chunks = (int32_t)N;
    double *S = (double *)malloc(sizeof(double) * (size_t)chunks);
    double *s = (double *)malloc(sizeof(double) * (size_t)chunks * (size_t)D);
    if (!S || !s) { free(S); free(s); return -1; }
#ifdef _OPENMP
#pragma omp parallel for schedule(static, 1)
#endif
    for (int32_t c = 0; c < chunks; ++c) {
        int64_t i0 = N * (int64_t)c / chunks;
        int64_t i1 = N * (int64_t)(c + 1) / chunks;
        data_sums(loss, X, y, i0, i1, D, w, &S[c], s + (size_t)c * D);
    }
    double Stot = 0.0;
    for (int32_t j = 0; j < D; ++j) g[j] = 0.0;
    for (int32_t c = 0; c < chunks; ++c) {
        Stot += S[c];
        for (int32_t j = 0; j < D; ++j) g[j] += s[(size_t)c * D + j];
    }
    free(S); free(s);
    double ww = 0.0;
    for (int32_t j = 0; j < D; ++j) ww += w[j] * w[j];
    *L_out = Stot / (double)N + 0.5 * lambda * ww;
    for (int32_t j = 0; j < D; ++j) g[j] = g[j] / (double)N + lambda * w[j];
    return 0;
}

/*
 * K gradient-descent iterations with a constant step from w (updated in
 * place).  loss_hist[k] and gnorm_hist[k] are the loss and the gradient L2
 * norm at the iterate that ENTERS iteration k (so loss_hist[0] is the loss at
 * the initial w).  g_last receives the gradient of the last iteration run.
 * chunks <= 1 selects the strictly sequential evaluation.
 */
int oracle_run(int loss, const float *X, const float *y, int64_t N, int32_t D,
               double *w, double lambda, double eta, int32_t K, int32_t chunks,
               double *loss_hist, double *gnorm_hist, double *g_last)
{
    if (K < 0) return -1;
    double *g = (double *)malloc(sizeof(double) * (size_t)(D > 0 ? D : 1));
    if (!g) return -1;
    for (int32_t k = 0; k < K; ++k) {
        double L;
        int rc = (chunks <= 1)
                     ? oracle_loss_grad(loss, X, y, N, D, w, lambda, &L, g)
                     : oracle_loss_grad_chunked(loss, X, y, N, D, w, lambda, chunks, &L, g);
        if (rc != 0) { free(g); return rc; }
        double gg = 0.0;
        for (int32_t j = 0; j < D; ++j) gg += g[j] * g[j];
        loss_hist[k] = L;
        gnorm_hist[k] = sqrt(gg);
        for (int32_t j = 0; j < D; ++j) w[j] -= eta * g[j];
        if (g_last) memcpy(g_last, g, sizeof(double) * (size_t)D);
    }
    free(g);
    return 0;
}

/* As oracle_run, with the step of every iteration given by a schedule.  k counts the iterations
 * of the job from its start: k = k0 + position in this call, so that a run split into several
 * calls takes the same steps as one call.
 *   schedule 0: eta_k = eta
 *   schedule 1: eta_k = eta / sqrt(k + 1)   (the decay of MLlib's gradient descent, the library
 *               the jobs of Sec. 3 "Setup" ran on; a first-order method of Sec. 2, class I) */
int oracle_run_schedule(int loss, const float *X, const float *y, int64_t N, int32_t D,
                        double *w, double lambda, double eta, int schedule, int64_t k0, int32_t K,
                        double *loss_hist, double *gnorm_hist, double *g_last)
{
    if (K < 0 || k0 < 0 || (schedule != 0 && schedule != 1)) return -1;
    double *g = (double *)malloc(sizeof(double) * (size_t)(D > 0 ? D : 1));
    if (!g) return -1;
    for (int32_t i = 0; i < K; ++i) {
        double L;
        int rc = oracle_loss_grad(loss, X, y, N, D, w, lambda, &L, g);
        if (rc != 0) { free(g); return rc; }
        double gg = 0.0;
        for (int32_t j = 0; j < D; ++j) gg += g[j] * g[j];
        loss_hist[i] = L;
        gnorm_hist[i] = sqrt(gg);
        const int64_t k = k0 + i;
        const double eta_k = (schedule == 1) ? eta / sqrt((double)(k + 1)) : eta;
        for (int32_t j = 0; j < D; ++j) w[j] = w[j] - eta_k * g[j];
        if (g_last) memcpy(g_last, g, sizeof(double) * (size_t)D);
    }
    free(g);
    return 0;
}

/*
 * The same loss and gradient for a sparse X given in CSR form (row_ptr [N+1], col_idx and val
 * [nnz]; entries of a row in stored order, duplicates add).  Plain loops over the stored entries:
 * absent entries are zeros of the dense definition above.  g must hold D doubles.
 */
int oracle_sparse_loss_grad(int loss, const int64_t *row_ptr, const int32_t *col_idx,
                            const float *val, const float *y, int64_t N, int64_t D,
                            const double *w, double lambda, double *L_out, double *g)
{
    if (loss < 0 || loss > 2 || N < 1 || D < 1) return -1;
    double S = 0.0;
    for (int64_t j = 0; j < D; ++j) g[j] = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        double z = 0.0;
        for (int64_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            if (col_idx[e] < 0 || col_idx[e] >= D) return -1;
            z += (double)val[e] * w[col_idx[e]];
        }
        double l, r;
        sample_loss_residual(loss, z, (double)y[i], &l, &r);
        S += l;
        for (int64_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) g[col_idx[e]] += (double)val[e] * r;
    }
    double ww = 0.0;
    for (int64_t j = 0; j < D; ++j) ww += w[j] * w[j];
    *L_out = S / (double)N + 0.5 * lambda * ww;
    for (int64_t j = 0; j < D; ++j) g[j] = g[j] / (double)N + lambda * w[j];
    return 0;
}

/* K constant-step iterations on a CSR matrix; histories as in oracle_run. */
int oracle_sparse_run(int loss, const int64_t *row_ptr, const int32_t *col_idx, const float *val,
                      const float *y, int64_t N, int64_t D, double *w, double lambda, double eta,
                      int32_t K, double *loss_hist, double *gnorm_hist, double *g_last)
{
    if (K < 0 || D < 1) return -1;
    double *g = (double *)malloc(sizeof(double) * (size_t)D);
    if (!g) return -1;
    for (int32_t k = 0; k < K; ++k) {
        double L;
        int rc = oracle_sparse_loss_grad(loss, row_ptr, col_idx, val, y, N, D, w, lambda, &L, g);
        if (rc != 0) { free(g); return rc; }
        double gg = 0.0;
        for (int64_t j = 0; j < D; ++j) gg += g[j] * g[j];
        loss_hist[k] = L;
        gnorm_hist[k] = sqrt(gg);
        for (int64_t j = 0; j < D; ++j) w[j] -= eta * g[j];
        if (g_last) memcpy(g_last, g, sizeof(double) * (size_t)D);
    }
    free(g);
    return 0;
}

/* As oracle_sparse_run, with the step schedule of oracle_run_schedule (k = k0 + position in
 * this call; schedule 0: eta, schedule 1: eta / sqrt(k + 1)). */
int oracle_sparse_run_schedule(int loss, const int64_t *row_ptr, const int32_t *col_idx, const float *val,
                               const float *y, int64_t N, int64_t D, double *w, double lambda, double eta,
                               int schedule, int64_t k0, int32_t K, double *loss_hist, double *gnorm_hist,
                               double *g_last)
{
    if (K < 0 || D < 1 || k0 < 0 || (schedule != 0 && schedule != 1)) return -1;
    double *g = (double *)malloc(sizeof(double) * (size_t)D);
    if (!g) return -1;
    for (int32_t i = 0; i < K; ++i) {
        double L;
        int rc = oracle_sparse_loss_grad(loss, row_ptr, col_idx, val, y, N, D, w, lambda, &L, g);
        if (rc != 0) { free(g); return rc; }
        double gg = 0.0;
        for (int64_t j = 0; j < D; ++j) gg += g[j] * g[j];
        loss_hist[i] = L;
        gnorm_hist[i] = sqrt(gg);
        const int64_t ks = k0 + i;
        const double eta_ks = (schedule == 1) ? eta / sqrt((double)(ks + 1)) : eta;
        for (int64_t j = 0; j < D; ++j) w[j] = w[j] - eta_ks * g[j];
        if (g_last) memcpy(g_last, g, sizeof(double) * (size_t)D);
    }
    free(g);
    return 0;
}

/* Number of threads the chunked evaluation can use (1 without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int oracle_max_threads(void) { return omp_get_max_threads(); }
#else
int oracle_max_threads(void) { return 1; }
#endif
