// Scheduler-side steps that consume the loss histories: the loss-change normaliser, the
// convergence-curve predictor (one wave per job, fp64) and the greedy allocator (host, binary heap).
//
// Predictor, per job, on the last m <= window losses L_0..L_{m-1}, mapped to l = (L - min)/span,
// at t_i = i / (m-1) with weights w_i = gamma^(m-1-i): the weighted least-squares fit of
//   class 1 (sublinear):  f(t) = 1 / (a t^2 + b t + c) - 10^e      class 2 (linear):  f(t) = exp(p t + q) - 10^e
// over all parameters, the offset confined to -10^e with -4 <= e <= 2 (the asymptote lies between
// 1e-4 and 100 spans under the smallest loss of the window).
//
// The error surface has narrow curved valleys along e, so the search eliminates the other
// parameters: phi(e) = min over (a, b, c), resp. (p, q), of the weighted squared error, found per
// lane by a damped Gauss-Newton iteration.  The wave scans phi on 256 values of e (4 consecutive
// ones per lane, each started from its left neighbour's solution), takes the lowest local minima of
// the scan and narrows each by 64-way subdivision of its bracket (every lane solves one e of the
// bracket; the bracket shrinks to the winner's neighbours): two rounds for every such minimum, four
// more for the best of them, then one tightly converged solve at the winning e.
#include <cmath>
#include <mutex>
#include <queue>
#include <vector>

#include "glm_internal.h"

namespace slaqglm {

constexpr double kExpLo = -4.0, kExpHi = 2.0;
constexpr int kScanPerLane = 4;              // 64 lanes x 4 = 256 scan points, 0.0235 apart
constexpr int kScanPoints = 64 * kScanPerLane;
constexpr int kBasins = 4;                   // local minima of the scan that are refined
constexpr int kRoundsAll = 2;                // subdivision rounds for every basin; each shrinks the bracket by 2/63
constexpr int kRoundsBest = 4;               // further rounds for the best basin: 0.094 -> 1e-10 in e

struct Lin { double a, b, c; };              // class 1: (a, b, c); class 2: (p, q, unused)

// Weighted squared error of the curve with parameters (p, off) on the window; +inf if not admissible.
__device__ double window_error(const int cls, const int m, const double *__restrict__ l,
                               const double *__restrict__ w, const double inv, const Lin p, const double off) {
    double s = 0.0;
    for (int i = 0; i < m; ++i) {
        const double t = (double)i * inv;
        double f;
        if (cls == GLM_CURVE_SUBLINEAR) {
            const double q = (p.a * t + p.b) * t + p.c;
            if (!(q > 0.0) || !isfinite(q)) return INFINITY;
            f = 1.0 / q + off;
        } else {
            f = exp(p.a * t + p.b) + off;
        }
        const double r = f - l[i];
        s += w[i] * (r * r);
    }
    return isfinite(s) ? s : INFINITY;
}

// Symmetric positive definite n x n system (n = 2 or 3), unit diagonal plus mu, by elimination
// without pivoting.  Upper triangle in (a01, a02, a12); false if a pivot is not positive.
__device__ __forceinline__ bool solve_scaled(const int n, const double mu, const double a01, const double a02,
                                             const double a12, const double b0, const double b1, const double b2,
                                             double &x0, double &x1, double &x2) {
    const double d = 1.0 + mu;
    if (n == 2) {
        const double l10 = a01 / d;
        const double p11 = d - l10 * a01;
        if (!(p11 > 0.0)) return false;
        x1 = (b1 - l10 * b0) / p11;
        x0 = (b0 - a01 * x1) / d;
        x2 = 0.0;
        return isfinite(x0) && isfinite(x1);
    }
    const double l10 = a01 / d, l20 = a02 / d;
    const double p11 = d - l10 * a01, p12 = a12 - l10 * a02, y1 = b1 - l10 * b0;
    if (!(p11 > 0.0)) return false;
    const double l21 = p12 / p11;
    const double p22 = (d - l20 * a02) - l21 * p12, y2 = (b2 - l20 * b0) - l21 * y1;
    if (!(p22 > 0.0)) return false;
    x2 = y2 / p22;
    x1 = (y1 - p12 * x2) / p11;
    x0 = (b0 - a01 * x1 - a02 * x2) / d;
    return isfinite(x0) && isfinite(x1) && isfinite(x2);
}

// Starting point for a fixed offset: weighted linear least squares on the transformed losses
// u = 1/(l - off), resp. log(l - off), with first-order weights w (l-off)^4, resp. w (l-off)^2.
__device__ bool transformed_start(const int cls, const int m, const double *__restrict__ l,
                                  const double *__restrict__ w, const double inv, const double gap, Lin &p) {
    double s4 = 0, s3 = 0, s2 = 0, s1 = 0, s0 = 0, r2 = 0, r1 = 0, r0 = 0;
    for (int i = 0; i < m; ++i) {
        const double g = l[i] + gap;
        const double t = (double)i * inv;
        double u, W;
        if (cls == GLM_CURVE_SUBLINEAR) { u = 1.0 / g; const double g2 = g * g; W = w[i] * (g2 * g2); }
        else { u = log(g); W = w[i] * (g * g); }
        const double t2 = t * t;
        s0 += W; s1 += W * t; s2 += W * t2; s3 += W * (t2 * t); s4 += W * (t2 * t2);
        r0 += W * u; r1 += W * (t * u); r2 += W * (t2 * u);
    }
    if (cls == GLM_CURVE_SUBLINEAR) {
        // [s4 s3 s2; s3 s2 s1; s2 s1 s0] (a b c)^T = (r2 r1 r0)^T, scaled to a unit diagonal
        if (!(s4 > 0.0) || !(s2 > 0.0) || !(s0 > 0.0)) return false;
        const double d0 = sqrt(s4), d1 = sqrt(s2), d2 = sqrt(s0);
        double x0, x1, x2;
        if (!solve_scaled(3, 0.0, s3 / (d0 * d1), s2 / (d0 * d2), s1 / (d1 * d2), r2 / d0, r1 / d1, r0 / d2, x0, x1, x2))
            return false;
        p.a = x0 / d0; p.b = x1 / d1; p.c = x2 / d2;
    } else {
        if (!(s2 > 0.0) || !(s0 > 0.0)) return false;
        const double d0 = sqrt(s2), d1 = sqrt(s0);
        double x0, x1, x2;
        if (!solve_scaled(2, 0.0, s1 / (d0 * d1), 0.0, 0.0, r1 / d0, r0 / d1, 0.0, x0, x1, x2)) return false;
        p.a = x0 / d0; p.b = x1 / d1; p.c = 0.0;
    }
    return true;
}

// Error of the curve (p, off) on the window, +inf if it is not admissible, together with the
// Gauss-Newton normal equations J^T W J, J^T W r there (J: derivatives of the curve by p).
struct NormalEq { double A00, A01, A02, A11, A12, A22, g0, g1, g2; };
__device__ double normal_equations(const int cls, const int m, const double *__restrict__ l,
                                   const double *__restrict__ w, const double inv, const Lin p, const double off,
                                   NormalEq &q) {
    double A00 = 0, A01 = 0, A02 = 0, A11 = 0, A12 = 0, A22 = 0, g0 = 0, g1 = 0, g2 = 0, s = 0;
    for (int i = 0; i < m; ++i) {
        const double t = (double)i * inv;
        double f, j0, j1, j2;
        if (cls == GLM_CURVE_SUBLINEAR) {
            const double den = (p.a * t + p.b) * t + p.c;
            if (!(den > 0.0) || !isfinite(den)) return INFINITY;
            const double iq = 1.0 / den;
            f = iq + off;
            j2 = -(iq * iq); j1 = j2 * t; j0 = j1 * t;
        } else {
            const double E = exp(p.a * t + p.b);
            f = E + off;
            j0 = E * t; j1 = E; j2 = 0.0;
        }
        const double wi = w[i];
        const double r = f - l[i];
        const double wr = wi * r;
        s += wr * r;
        g0 += j0 * wr; g1 += j1 * wr; g2 += j2 * wr;
        const double w0 = wi * j0, w1 = wi * j1;
        A00 += w0 * j0; A01 += w0 * j1; A02 += w0 * j2; A11 += w1 * j1; A12 += w1 * j2; A22 += wi * j2 * j2;
    }
    q.A00 = A00; q.A01 = A01; q.A02 = A02; q.A11 = A11; q.A12 = A12; q.A22 = A22; q.g0 = g0; q.g1 = g1; q.g2 = g2;
    return isfinite(s) ? s : INFINITY;
}

// phi(e): damped Gauss-Newton on the parameters other than e.  Starts from p when `warm` and p is
// admissible, else from the transformed problem's solution; with `both`, from whichever of the two
// has the lower error; if neither is admissible, from the constant curve.  Returns phi, p = minimiser.
// Stops after max_iter steps, or when a step no longer changes the parameters, or when the decrease
// promised by the linearised model falls below tol times the error, or at an error of 1e-28 (the
// window is scaled to [0, 1]: an exact fit to rounding).
__device__ double profile(const int cls, const int m, const double *__restrict__ l, const double *__restrict__ w,
                          const double inv, const double e, const bool warm, const bool both, const int max_iter,
                          const double tol, Lin &p) {
    const double gap = pow(10.0, e);
    const double off = -gap;
    const int n = cls == GLM_CURVE_SUBLINEAR ? 3 : 2;
    double sse = warm ? window_error(cls, m, l, w, inv, p, off) : INFINITY;
    if (both || !(sse < INFINITY)) {         // the transformed problem's solution, if that starts lower
        Lin q;
        if (transformed_start(cls, m, l, w, inv, gap, q)) {
            const double sq = window_error(cls, m, l, w, inv, q, off);
            if (sq < sse) { sse = sq; p = q; }
        }
        if (!(sse < INFINITY)) {             // last resort: the constant curve at the weighted mean
            double sw = 0.0, sl = 0.0;
            for (int i = 0; i < m; ++i) { sw += w[i]; sl += w[i] * l[i]; }
            const double mean_gap = sl / sw + gap;
            p.a = 0.0; p.b = 0.0; p.c = 0.0;
            if (cls == GLM_CURVE_SUBLINEAR) p.c = 1.0 / mean_gap; else p.b = log(mean_gap);
            sse = window_error(cls, m, l, w, inv, p, off);
            if (!(sse < INFINITY)) return INFINITY;
        }
    }
    // One pass over the window gives the error AND the Gauss-Newton normal equations at a point, so a
    // trial step costs one pass: if it is accepted its equations are already there for the next step.
    NormalEq cur;
    sse = normal_equations(cls, m, l, w, inv, p, off, cur);
    if (!(sse < INFINITY)) return INFINITY;
    double mu = 1e-4;
    for (int it = 0; it < max_iter; ++it) {
        const int nn = n;
        const double d0 = cur.A00 > 0.0 ? sqrt(cur.A00) : 1.0, d1 = cur.A11 > 0.0 ? sqrt(cur.A11) : 1.0,
                     d2 = (nn == 3 && cur.A22 > 0.0) ? sqrt(cur.A22) : 1.0;
        const double a01 = cur.A01 / (d0 * d1), a02 = cur.A02 / (d0 * d2), a12 = cur.A12 / (d1 * d2);
        const double b0 = -cur.g0 / d0, b1 = -cur.g1 / d1, b2 = -cur.g2 / d2;
        bool moved = false, done = false;
        while (mu <= 1e10) {
            double x0, x1, x2;
            if (solve_scaled(nn, mu, a01, a02, a12, b0, b1, b2, x0, x1, x2)) {
                Lin c;
                const double s0 = x0 / d0, s1 = x1 / d1, s2 = nn == 3 ? x2 / d2 : 0.0;
                c.a = p.a + s0; c.b = p.b + s1; c.c = p.c + s2;
                NormalEq nxt;
                const double s_new = normal_equations(cls, m, l, w, inv, c, off, nxt);
                if (s_new <= sse) {
                    double rel = fmax(fabs(s0) / (fabs(c.a) + 1e-30), fabs(s1) / (fabs(c.b) + 1e-30));
                    if (nn == 3) rel = fmax(rel, fabs(s2) / (fabs(c.c) + 1e-30));
                    // decrease promised by the linearised model: -(g.s) - s.A.s/2 = b.x - (x.x + 2 (a01 x0 x1 + ...))/2
                    const double promised = (b0 * x0 + b1 * x1 + b2 * x2) -
                        0.5 * (x0 * x0 + x1 * x1 + x2 * x2 + 2.0 * (a01 * x0 * x1 + a02 * x0 * x2 + a12 * x1 * x2));
                    done = rel <= 1e-13 || s_new == sse || promised <= tol * s_new || s_new <= 1e-28;
                    p = c; sse = s_new; cur = nxt; moved = true;
                    mu = fmax(mu * 0.1, 1e-14);
                    break;
                }
            }
            mu *= 10.0;
        }
        if (!moved || done) break;
    }
    return sse;
}

// Lane holding the smallest value (lowest lane on ties); every lane gets the same answer.
__device__ __forceinline__ int wave_argmin(double v, int lane) {
    int idx = lane;
    for (int o = 32; o >= 1; o >>= 1) {
        const double ov = __shfl_xor(v, o, 64);
        const int oi = __shfl_xor(idx, o, 64);
        if (ov < v || (ov == v && oi < idx)) { v = ov; idx = oi; }
    }
    return idx;
}

__device__ __forceinline__ Lin lin_from_lane(const Lin &p, int src) {
    Lin r;
    r.a = __shfl(p.a, src, 64); r.b = __shfl(p.b, src, 64); r.c = __shfl(p.c, src, 64);
    return r;
}

__device__ __forceinline__ double scan_exponent(int idx) {
    return kExpLo + (kExpHi - kExpLo) * (double)idx / (double)(kScanPoints - 1);
}

__global__ __launch_bounds__(64) void predict_kernel(const PredJob *__restrict__ jobs, double gamma,
                                                     int window, int horizon, double *__restrict__ pred,
                                                     double *__restrict__ gain, double *__restrict__ fit) {
    __shared__ double Ls[kPredWindowMax];
    __shared__ double Ws[kPredWindowMax];
    const int lane = threadIdx.x;
    const PredJob jb = jobs[blockIdx.x];
    const long long n = jb.n;
    const int m = (int)(n < window ? n : window);
    const float *__restrict__ h = jb.hist;
    const long long start = n - m;

    // largest single-iteration change over the whole history (a maximum: order-free)
    double norm = 0.0;
    for (long long i = 1 + lane; i < n; i += 64) norm = fmax(norm, fabs((double)h[i - 1] - (double)h[i]));
    for (int o = 32; o >= 1; o >>= 1) norm = fmax(norm, __shfl_xor(norm, o, 64));

    double lo = INFINITY, hi = -INFINITY;
    bool finite = true;
    for (int i = lane; i < m; i += 64) {
        const double v = (double)h[start + i];
        Ls[i] = v;
        Ws[i] = pow(gamma, (double)(m - 1 - i));
        finite = finite && isfinite(v);
        lo = fmin(lo, v); hi = fmax(hi, v);
    }
    for (int o = 32; o >= 1; o >>= 1) { lo = fmin(lo, __shfl_xor(lo, o, 64)); hi = fmax(hi, __shfl_xor(hi, o, 64)); }
    finite = __all(finite);
    __syncthreads();
    const double last = m > 0 ? Ls[m - 1] : 0.0;
    const double span = hi - lo;
    double *fo = fit + (size_t)blockIdx.x * 8;
    double *po = pred + (size_t)blockIdx.x * horizon;
    double *go = gain + (size_t)blockIdx.x * horizon;

    const int cls = jb.cls;
    double best_phi = INFINITY, best_e = 0.0;
    Lin best_p; best_p.a = best_p.b = best_p.c = 0.0;
    if (m >= kPredMinPoints && finite && span > 0.0 && isfinite(span)) {
        __syncthreads();
        for (int i = lane; i < m; i += 64) Ls[i] = (Ls[i] - lo) / span;      // the window mapped to [0, 1]
        __syncthreads();
        const double inv = 1.0 / (double)(m - 1);

        // scan: lane g solves the points 4 g .. 4 g + 3, each from its left neighbour's solution, and
        // remembers the lowest of them that is a local minimum of the whole 256-point sequence
        double phi[kScanPerLane];
        Lin sol[kScanPerLane];
        Lin p; p.a = p.b = p.c = 0.0;
        bool warm = false;
#pragma unroll
        for (int k = 0; k < kScanPerLane; ++k) {
            phi[k] = profile(cls, m, Ls, Ws, inv, scan_exponent(lane * kScanPerLane + k), warm, true, 20, 1e-8, p);
            sol[k] = p;
            warm = phi[k] < INFINITY;
        }
        double left = __shfl_up(phi[kScanPerLane - 1], 1, 64);
        double right = __shfl_down(phi[0], 1, 64);
        if (lane == 0) left = INFINITY;
        if (lane == 63) right = INFINITY;
        double my_phi = INFINITY; int my_idx = 0; Lin my_p = p;
#pragma unroll
        for (int k = 0; k < kScanPerLane; ++k) {
            const double lf = k == 0 ? left : phi[k - 1];
            const double rt = k == kScanPerLane - 1 ? right : phi[k + 1];
            if (phi[k] < INFINITY && phi[k] < lf && phi[k] <= rt && phi[k] < my_phi) {
                my_phi = phi[k]; my_idx = lane * kScanPerLane + k; my_p = sol[k];
            }
        }

        // One subdivision round of the bracket [e_lo, e_hi] around (cur_e, cur): every lane solves one e.
        auto subdivide = [&](double &e_lo, double &e_hi, double &cur_phi, double &cur_e, Lin &cur) {
            const double step = (e_hi - e_lo) / 63.0;
            const double e = lane == 63 ? e_hi : e_lo + step * (double)lane;
            Lin q = cur;
            const double v = profile(cls, m, Ls, Ws, inv, e, true, false, 40, 1e-12, q);
            const int win = wave_argmin(v, lane);
            const double wv = __shfl(v, win, 64);
            if (wv < cur_phi) { cur_phi = wv; cur_e = __shfl(e, win, 64); cur = lin_from_lane(q, win); }
            const double n_lo = __shfl(e, win > 0 ? win - 1 : 0, 64);
            const double n_hi = __shfl(e, win < 63 ? win + 1 : 63, 64);
            e_lo = n_lo; e_hi = n_hi;
        };

        double b_lo = 0.0, b_hi = 0.0;                                       // bracket of the best basin so far
        for (int basin = 0; basin < kBasins; ++basin) {
            const int src = wave_argmin(my_phi, lane);
            const double seed_phi = __shfl(my_phi, src, 64);
            if (!(seed_phi < INFINITY)) break;
            const int seed_idx = __shfl(my_idx, src, 64);
            Lin cur = lin_from_lane(my_p, src);
            if (lane == src) my_phi = INFINITY;                              // taken
            double cur_phi = seed_phi;
            double cur_e = scan_exponent(seed_idx);
            double e_lo = scan_exponent(seed_idx > 1 ? seed_idx - 2 : 0);    // two scan steps to either side
            double e_hi = scan_exponent(seed_idx < kScanPoints - 2 ? seed_idx + 2 : kScanPoints - 1);
            for (int round = 0; round < kRoundsAll; ++round) subdivide(e_lo, e_hi, cur_phi, cur_e, cur);
            if (cur_phi < best_phi) { best_phi = cur_phi; best_e = cur_e; best_p = cur; b_lo = e_lo; b_hi = e_hi; }
        }
        if (best_phi < INFINITY) {
            for (int round = 0; round < kRoundsBest; ++round) subdivide(b_lo, b_hi, best_phi, best_e, best_p);
            Lin q = best_p;                                                  // the same solve in every lane
            const double v = profile(cls, m, Ls, Ws, inv, best_e, true, false, 100, 1e-15, q);
            if (v <= best_phi) { best_phi = v; best_p = q; }
        }
    }

    if (!(best_phi < INFINITY)) {           // too short, flat, not finite or nothing admissible: repeat the last loss
        for (int hh = lane; hh < horizon; hh += 64) { po[hh] = last; go[hh] = 0.0; }
        if (lane == 0) { fo[0] = 0.0; fo[1] = 0.0; fo[2] = 0.0; fo[3] = 0.0; fo[4] = 0.0; fo[5] = 0.0; fo[6] = norm; fo[7] = (double)m; }
        return;
    }

    // back to the units of the losses: f = span (curve - 10^e) + lo
    const double gap = pow(10.0, best_e);
    const double inv = 1.0 / (double)(m - 1);
    for (int hh = lane; hh < horizon; hh += 64) {
        double f[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {       // s = 0: the iteration before (t = 1 for hh = 0), s = 1: this one
            const double t = (double)(m - 1 + hh + s) * inv;
            double c;
            bool ok = true;
            if (cls == GLM_CURVE_SUBLINEAR) {
                const double q = (best_p.a * t + best_p.b) * t + best_p.c;
                ok = q > 0.0;
                c = 1.0 / q;
            } else {
                c = exp(best_p.a * t + best_p.b);
            }
            f[s] = ok ? lo + span * (c - gap) : last;
        }
        po[hh] = f[1];
        go[hh] = norm > 0.0 ? (f[0] - f[1]) / norm : 0.0;
    }
    if (lane == 0) {
        fo[0] = 1.0; fo[1] = lo - span * gap;
        if (cls == GLM_CURVE_SUBLINEAR) { fo[2] = best_p.a / span; fo[3] = best_p.b / span; fo[4] = best_p.c / span; }
        else { fo[2] = best_p.a; fo[3] = best_p.b + log(span); fo[4] = 0.0; }
        fo[5] = best_phi * span * span; fo[6] = norm; fo[7] = (double)m;
    }
}

hipError_t launch_predict(const PredJob *jobs, int J, double gamma, int window, int horizon,
                          double *pred, double *gain, double *fit, hipStream_t st) {
    hipLaunchKernelGGL(predict_kernel, dim3((unsigned)J), dim3(64), 0, st, jobs, gamma, window, horizon,
                       pred, gain, fit);
    return hipGetLastError();
}

// Greedy allocation with a heap: the next unit goes to the job whose next unit has the largest
// predicted reduction (lowest job index on ties).  Same decisions as scanning all jobs per unit.
int allocate_greedy(const double *gain, int J, int H, long long capacity, int *alloc) {
    struct Item { double g; int j; };
    struct Less {   // priority_queue keeps the "largest": larger gain first, then lower index
        bool operator()(const Item &a, const Item &b) const { return a.g < b.g || (a.g == b.g && a.j > b.j); }
    };
    std::priority_queue<Item, std::vector<Item>, Less> heap;
    for (int j = 0; j < J; ++j) {
        alloc[j] = 1;
        if (H > 1) heap.push(Item{gain[(size_t)j * H + 1], j});
    }
    long long left = capacity - J;
    while (left > 0 && !heap.empty()) {
        const Item it = heap.top();
        heap.pop();
        const int a = ++alloc[it.j];
        --left;
        if (a < H) heap.push(Item{gain[(size_t)it.j * H + a], it.j});
    }
    return GLM_OK;
}

}  // namespace slaqglm
