/*
 * fp64 CPU oracle for the convergence-curve fit (TEST INFRASTRUCTURE: called only by tests, the
 * smoke check and the benchmark's CPU leg; shares nothing with the GPU library).
 *
 * Sec. 2 of the paper, "Predicting Quality Improvement": a curve
 *     class I  (sublinear convergence)           f(k) = 1 / (a k^2 + b k + c) + d
 *     class II (linear or superlinear)           f(k) = mu^(k - b) + c
 * is fitted to the exponentially weighted loss history.  Written out, over the m losses L_i of
 * the window, at scaled times t_i = i / (m - 1) and with weights w_i = gamma^(m-1-i):
 *     minimise  E(theta) = sum_i w_i (f(t_i; theta) - L_i)^2   over all parameters of the curve.
 * The paper gives neither the weight decay nor a parameter domain; the readings taken here:
 *   - the asymptote (d, resp. c) lies below every loss of the window, between 1e-4 and 100 spans
 *     under the smallest one (span = max - min of the window):
 *         offset = min L - span * 10^e,   -4 <= e <= 2.
 *     Without such a box there is no minimiser on histories that fall along a straight line (E
 *     keeps decreasing as the asymptote goes to minus infinity);
 *   - class I needs a positive denominator at every fitted point; class II is written
 *     f = exp(p t + q) + c  (mu^(k-b) with mu > 0).
 *
 * The problem is not convex and its valleys are narrow, so the minimiser is found by elimination:
 * for a fixed exponent e the other parameters come from a damped Gauss-Newton iteration, which
 * defines the profile  phi(e) = min over the others of E;  phi is scanned on kScan values of e,
 * every local minimum of the scan is refined by golden-section search between its neighbours, and
 * the lowest refined minimum wins.
 *
 * Everything works on the window mapped to [0, 1]:  l = (L - min) / span;  there the offset is
 * -10^e and the other parameters are lin = (a, b, c), f = 1/(a t^2 + b t + c) - 10^e, resp.
 * lin = (p, q), f = exp(p t + q) - 10^e.
 *
 * The paper prints no numeric example: against paper values this is "parity unpinned"; the CPU
 * tests pin it against scipy.optimize.least_squares started from many points, on exact and noisy
 * curves of every length from 8 to 128.
 */
#include <math.h>
#include <stddef.h>

#define MAXM 128
enum { CLASS_SUBLINEAR = 1, CLASS_LINEAR = 2 };
static const double kExpLo = -4.0, kExpHi = 2.0;
enum { kScan = 1201 };                        /* scan step 0.005 in e */
static const double kGoldenTol = 1e-10;       /* width in e at which the golden-section search stops */

typedef struct {
    int cls, m;
    double t[MAXM], l[MAXM], w[MAXM];
} Window;

static int nparams(int cls) { return cls == CLASS_SUBLINEAR ? 3 : 2; }

/* E at (lin, e); +inf when the point is not admissible. */
static double sse_at(const Window *W, const double *lin, double e) {
    const double off = -pow(10.0, e);
    double s = 0.0;
    for (int i = 0; i < W->m; ++i) {
        const double t = W->t[i];
        double f;
        if (W->cls == CLASS_SUBLINEAR) {
            const double q = (lin[0] * t + lin[1]) * t + lin[2];
            if (!(q > 0.0) || !isfinite(q)) return INFINITY;
            f = 1.0 / q + off;
        } else {
            f = exp(lin[0] * t + lin[1]) + off;
        }
        const double r = f - W->l[i];
        s += W->w[i] * r * r;
    }
    return isfinite(s) ? s : INFINITY;
}

/* Gauss-Newton normal equations at an admissible point: A = J^T W J, g = J^T W r, where J holds
 * the derivatives of f with respect to lin. */
static void normal_equations(const Window *W, const double *lin, double e, double A[3][3], double g[3]) {
    const int n = nparams(W->cls);
    const double off = -pow(10.0, e);
    for (int a = 0; a < 3; ++a) { g[a] = 0.0; for (int b = 0; b < 3; ++b) A[a][b] = 0.0; }
    for (int i = 0; i < W->m; ++i) {
        const double t = W->t[i];
        double f, J[3];
        if (W->cls == CLASS_SUBLINEAR) {
            const double q = (lin[0] * t + lin[1]) * t + lin[2];
            const double dq = -1.0 / (q * q);
            f = 1.0 / q + off;
            J[0] = dq * t * t; J[1] = dq * t; J[2] = dq;
        } else {
            const double E = exp(lin[0] * t + lin[1]);
            f = E + off;
            J[0] = E * t; J[1] = E; J[2] = 0.0;
        }
        const double r = f - W->l[i];
        for (int a = 0; a < n; ++a) {
            g[a] += W->w[i] * J[a] * r;
            for (int b = 0; b < n; ++b) A[a][b] += W->w[i] * J[a] * J[b];
        }
    }
}

/* Solves the n x n system A x = b (n <= 3) by elimination with partial pivoting; 0 on a zero pivot. */
static int solve_small(int n, double A[3][3], const double b[3], double x[3]) {
    double M[3][4];
    for (int r = 0; r < n; ++r) { for (int c = 0; c < n; ++c) M[r][c] = A[r][c]; M[r][n] = b[r]; }
    for (int c = 0; c < n; ++c) {
        int piv = c;
        for (int r = c + 1; r < n; ++r) if (fabs(M[r][c]) > fabs(M[piv][c])) piv = r;
        if (!(fabs(M[piv][c]) > 0.0) || !isfinite(M[piv][c])) return 0;
        if (piv != c) for (int k = 0; k <= n; ++k) { const double tmp = M[c][k]; M[c][k] = M[piv][k]; M[piv][k] = tmp; }
        for (int r = c + 1; r < n; ++r) {
            const double f = M[r][c] / M[c][c];
            for (int k = c; k <= n; ++k) M[r][k] -= f * M[c][k];
        }
    }
    for (int r = n - 1; r >= 0; --r) {
        double s = M[r][n];
        for (int c = r + 1; c < n; ++c) s -= M[r][c] * x[c];
        x[r] = s / M[r][r];
    }
    for (int r = 0; r < n; ++r) if (!isfinite(x[r])) return 0;
    return 1;
}

/* A starting point for a fixed offset -10^e: weighted linear least squares on the transformed
 * losses 1/(l - off), resp. log(l - off), with first-order weights. */
static int transformed_start(const Window *W, double e, double *lin) {
    const int n = nparams(W->cls);
    const double gap = pow(10.0, e);
    double A[3][3] = {{0}}, b[3] = {0};
    for (int i = 0; i < W->m; ++i) {
        const double g = W->l[i] + gap;               /* l - offset > 0 */
        const double t = W->t[i];
        double u, wt, B[3];
        if (W->cls == CLASS_SUBLINEAR) { u = 1.0 / g; wt = W->w[i] * g * g * g * g; B[0] = t * t; B[1] = t; B[2] = 1.0; }
        else { u = log(g); wt = W->w[i] * g * g; B[0] = t; B[1] = 1.0; B[2] = 0.0; }
        for (int a = 0; a < n; ++a) {
            b[a] += wt * B[a] * u;
            for (int c = 0; c < n; ++c) A[a][c] += wt * B[a] * B[c];
        }
    }
    return solve_small(n, A, b, lin);
}

/* The constant curve through the weighted mean of the window: admissible for every offset. */
static void flat_start(const Window *W, double e, double *lin) {
    double sw = 0.0, sl = 0.0;
    for (int i = 0; i < W->m; ++i) { sw += W->w[i]; sl += W->w[i] * W->l[i]; }
    const double mean_gap = sl / sw + pow(10.0, e);   /* mean - offset > 0 */
    if (W->cls == CLASS_SUBLINEAR) { lin[0] = 0.0; lin[1] = 0.0; lin[2] = 1.0 / mean_gap; }
    else { lin[0] = 0.0; lin[1] = log(mean_gap); lin[2] = 0.0; }
}

/* phi(e) and its minimiser: damped Gauss-Newton (Levenberg-Marquardt with Marquardt's scaling) on
 * the parameters other than e, from `start` when that is admissible, else from the transformed
 * problem's solution, else (that solution can have a denominator that changes sign) from the
 * constant curve.  Returns phi and writes lin. */
static double profile(const Window *W, double e, const double *start, double *lin) {
    const int n = nparams(W->cls);
    double sse = INFINITY;
    if (start) { for (int a = 0; a < n; ++a) lin[a] = start[a]; sse = sse_at(W, lin, e); }
    if (!isfinite(sse)) {
        if (transformed_start(W, e, lin)) sse = sse_at(W, lin, e);
        if (!isfinite(sse)) {                         /* last resort: the constant curve at the weighted mean */
            flat_start(W, e, lin);
            sse = sse_at(W, lin, e);
            if (!isfinite(sse)) return INFINITY;
        }
    }
    double mu = 1e-4;
    for (int it = 0; it < 200; ++it) {
        double A[3][3], g[3];
        normal_equations(W, lin, e, A, g);
        int moved = 0;
        while (mu <= 1e10) {
            double D[3][3], rhs[3], step[3], cand[3];
            for (int a = 0; a < n; ++a) {
                rhs[a] = -g[a];
                for (int b = 0; b < n; ++b) D[a][b] = A[a][b];
                D[a][a] += mu * (A[a][a] > 0.0 ? A[a][a] : 1.0);
            }
            if (!solve_small(n, D, rhs, step)) { mu *= 10.0; continue; }
            for (int a = 0; a < n; ++a) cand[a] = lin[a] + step[a];
            const double s_new = sse_at(W, cand, e);
            if (s_new <= sse) {
                /* converged when the step no longer changes the parameters, or when the decrease the
                 * linearised model promises, -(g.step) - step.A.step/2, is below rounding in E */
                double rel = 0.0, gs = 0.0, sAs = 0.0;
                for (int a = 0; a < n; ++a) {
                    rel = fmax(rel, fabs(step[a]) / (fabs(cand[a]) + 1e-30));
                    gs += g[a] * step[a];
                    for (int b = 0; b < n; ++b) sAs += step[a] * A[a][b] * step[b];
                }
                const int done = rel <= 1e-13 || s_new == sse || -gs - 0.5 * sAs <= 1e-15 * s_new;
                for (int a = 0; a < n; ++a) lin[a] = cand[a];
                sse = s_new; moved = 1;
                mu = fmax(mu * 0.1, 1e-14);
                if (done) return sse;
                break;
            }
            mu *= 10.0;
        }
        if (!moved) break;                            /* no damping gives a decrease: a minimum to rounding */
    }
    return sse;
}

/* Golden-section search for the minimum of phi on [lo, hi]; every evaluation starts its
 * Gauss-Newton iteration from the minimiser of the previous one. */
static double golden(const Window *W, double lo, double hi, const double *start, double *e_out, double *lin_out) {
    const double inv = (sqrt(5.0) - 1.0) / 2.0;
    double a = lo, b = hi;
    double x1 = b - inv * (b - a), x2 = a + inv * (b - a);
    double p1[3] = {0}, p2[3] = {0};
    double f1 = profile(W, x1, start, p1), f2 = profile(W, x2, start, p2);
    while (b - a > kGoldenTol) {
        if (f1 <= f2) {
            b = x2; x2 = x1; f2 = f1; for (int k = 0; k < 3; ++k) p2[k] = p1[k];
            x1 = b - inv * (b - a);
            f1 = profile(W, x1, p2, p1);
        } else {
            a = x1; x1 = x2; f1 = f2; for (int k = 0; k < 3; ++k) p1[k] = p2[k];
            x2 = a + inv * (b - a);
            f2 = profile(W, x2, p1, p2);
        }
    }
    if (f1 <= f2) { *e_out = x1; for (int k = 0; k < 3; ++k) lin_out[k] = p1[k]; return f1; }
    *e_out = x2; for (int k = 0; k < 3; ++k) lin_out[k] = p2[k];
    return f2;
}

/* Fits the curve of class `cls` to the window L[0..m-1] (5 <= m <= 128, finite values, not all
 * equal; with as many points as class I has parameters the curve would interpolate them, every
 * interpolant has error 0 and they extrapolate differently: nothing to choose between).  out = {ok, offset, p0, p1, p2, E, e} in the units of L and in scaled time:
 *   class I:  f(t) = 1 / (p0 t^2 + p1 t + p2) + offset;   class II:  f(t) = exp(p0 t + p1) + offset.
 * Returns 0; ok = 0 when the arguments are out of range or nothing admissible was found. */
int oracle_fit_curve(int cls, const double *L, int m, double gamma, double *out) {
    for (int k = 0; k < 7; ++k) out[k] = 0.0;
    if ((cls != CLASS_SUBLINEAR && cls != CLASS_LINEAR) || m < 5 || m > MAXM) return 0;
    double lo = L[0], hi = L[0];
    for (int i = 0; i < m; ++i) {
        if (!isfinite(L[i])) return 0;
        lo = fmin(lo, L[i]); hi = fmax(hi, L[i]);
    }
    const double span = hi - lo;
    if (!(span > 0.0) || !isfinite(span)) return 0;
    Window W;
    W.cls = cls; W.m = m;
    for (int i = 0; i < m; ++i) {
        W.t[i] = (double)i / (double)(m - 1);
        W.l[i] = (L[i] - lo) / span;
        W.w[i] = pow(gamma, (double)(m - 1 - i));
    }

    /* The scan.  The Gauss-Newton iteration for a fixed e can end in different local minima from
     * different starts, so every scan point is solved from the transformed problem's solution, from
     * its left neighbour's minimiser and (in a second sweep) from its right neighbour's; the lowest
     * of the three is phi. */
    double phi[kScan], lins[kScan][3];
    for (int i = 0; i < kScan; ++i) {
        const double e = kExpLo + (kExpHi - kExpLo) * (double)i / (double)(kScan - 1);
        phi[i] = profile(&W, e, NULL, lins[i]);
        if (i > 0 && isfinite(phi[i - 1])) {
            double alt[3];
            const double v = profile(&W, e, lins[i - 1], alt);
            if (v < phi[i]) { phi[i] = v; for (int k = 0; k < 3; ++k) lins[i][k] = alt[k]; }
        }
    }
    for (int i = kScan - 2; i >= 0; --i) {
        if (!isfinite(phi[i + 1])) continue;
        const double e = kExpLo + (kExpHi - kExpLo) * (double)i / (double)(kScan - 1);
        double alt[3];
        const double v = profile(&W, e, lins[i + 1], alt);
        if (v < phi[i]) { phi[i] = v; for (int k = 0; k < 3; ++k) lins[i][k] = alt[k]; }
    }
    double best = INFINITY, best_e = 0.0, best_lin[3] = {0, 0, 0};
    for (int i = 0; i < kScan; ++i) {
        if (!isfinite(phi[i])) continue;
        const double left = i > 0 ? phi[i - 1] : INFINITY;
        const double right = i + 1 < kScan ? phi[i + 1] : INFINITY;
        if (phi[i] < left && phi[i] <= right) {        /* a local minimum of the scan (first of a plateau) */
            const int il = i > 0 ? i - 1 : 0, ih = i + 1 < kScan ? i + 1 : kScan - 1;
            const double e_lo = kExpLo + (kExpHi - kExpLo) * (double)il / (double)(kScan - 1);
            const double e_hi = kExpLo + (kExpHi - kExpLo) * (double)ih / (double)(kScan - 1);
            double e, lin[3];
            double v = golden(&W, e_lo, e_hi, lins[i], &e, lin);
            if (phi[i] < v) {                          /* the grid point itself, should the search end above it */
                v = phi[i]; e = kExpLo + (kExpHi - kExpLo) * (double)i / (double)(kScan - 1);
                for (int k = 0; k < 3; ++k) lin[k] = lins[i][k];
            }
            if (v < best) { best = v; best_e = e; for (int k = 0; k < 3; ++k) best_lin[k] = lin[k]; }
        }
    }
    if (!isfinite(best)) return 0;
    out[0] = 1.0;
    out[1] = lo - span * pow(10.0, best_e);
    if (cls == CLASS_SUBLINEAR) {                      /* 1 / (q / span) = span / q */
        out[2] = best_lin[0] / span; out[3] = best_lin[1] / span; out[4] = best_lin[2] / span;
    } else {
        out[2] = best_lin[0]; out[3] = best_lin[1] + log(span); out[4] = 0.0;
    }
    out[5] = best * span * span;
    out[6] = best_e;
    return 0;
}
