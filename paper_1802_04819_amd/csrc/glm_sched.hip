// Scheduler-side steps that consume the loss histories: the loss-change normaliser, the
// convergence-curve predictor (one wave per job, one lane per offset candidate, fp64) and the
// greedy allocator (host, binary heap).
//
// Predictor, per job, on the last m <= window losses L_0..L_{m-1} (t_i = i / (m-1), weights
// w_i = gamma^(m-1-i)):
//   class 1 (sublinear):  f(t) = 1 / (a t^2 + b t + c) + d        class 2 (linear):  f(t) = exp(p t + q) + c
// For a candidate offset the other parameters enter linearly after u = 1/(L - d), resp.
// u = log(L - c); they come from weighted linear least squares with first-order weights
// w (L-d)^4, resp. w (L-c)^2.  Candidates: offset = min L - span * 10^e, 64 exponents e in
// [-4, 2], then 64 exponents within one grid step of the best; the candidate with the smallest
// weighted squared error of the untransformed curve wins, ties go to the lower index.
#include <cmath>
#include <mutex>
#include <queue>
#include <vector>

#include "glm_internal.h"

namespace slaqglm {

constexpr int kCand = 64;
constexpr double kExpLo = -4.0, kExpHi = 2.0;

struct Fit { double p0, p1, p2, off, sse; };

// Weighted fit for one offset; sse = +inf when the candidate is not admissible.
__device__ Fit fit_for_offset(const int cls, const double *__restrict__ L, const double *__restrict__ w,
                              const int m, const double off) {
    Fit r; r.p0 = r.p1 = r.p2 = 0.0; r.off = off; r.sse = INFINITY;
    const double inv = 1.0 / (double)(m - 1);
    double s4 = 0, s3 = 0, s2 = 0, s1 = 0, s0 = 0, r2 = 0, r1 = 0, r0 = 0;
    for (int i = 0; i < m; ++i) {
        const double g = L[i] - off;
        if (!(g > 0.0)) return r;
        const double t = (double)i * inv;
        double u, W;
        if (cls == GLM_CURVE_SUBLINEAR) { u = 1.0 / g; const double g2 = g * g; W = w[i] * (g2 * g2); }
        else { u = log(g); W = w[i] * (g * g); }
        const double t2 = t * t;
        s0 += W; s1 += W * t; s2 += W * t2; s3 += W * (t2 * t); s4 += W * (t2 * t2);
        r0 += W * u; r1 += W * (t * u); r2 += W * (t2 * u);
    }
    double a = 0.0, b, c;
    if (cls == GLM_CURVE_SUBLINEAR) {
        // normal equations [s4 s3 s2; s3 s2 s1; s2 s1 s0] [a b c]^T = [r2 r1 r0]^T, symmetric
        // positive definite: elimination without pivoting
        if (!(s4 > 0.0)) return r;
        const double l10 = s3 / s4, l20 = s2 / s4;
        const double a11 = s2 - l10 * s3, a12 = s1 - l10 * s2, y1 = r1 - l10 * r2;
        const double a22 = s0 - l20 * s2, y2 = r0 - l20 * r2;
        if (!(a11 > 0.0)) return r;
        const double l21 = a12 / a11;
        const double b22 = a22 - l21 * a12, z2 = y2 - l21 * y1;
        if (!(b22 > 0.0)) return r;
        c = z2 / b22;
        b = (y1 - a12 * c) / a11;
        a = (r2 - s3 * b - s2 * c) / s4;
    } else {
        // [s2 s1; s1 s0] [p q]^T = [r1 r0]^T
        if (!(s2 > 0.0)) return r;
        const double l = s1 / s2;
        const double d = s0 - l * s1;
        if (!(d > 0.0)) return r;
        c = (r0 - l * r1) / d;
        b = (r1 - s1 * c) / s2;
    }
    double sse = 0.0;
    for (int i = 0; i < m; ++i) {
        const double t = (double)i * inv;
        double f;
        if (cls == GLM_CURVE_SUBLINEAR) {
            const double lin = (a * t + b) * t + c;
            if (!(lin > 0.0) || !isfinite(lin)) return r;
            f = 1.0 / lin + off;
        } else {
            const double lin = b * t + c;
            if (!isfinite(lin)) return r;
            f = exp(lin) + off;
        }
        const double e = f - L[i];
        sse += w[i] * (e * e);
    }
    if (!isfinite(sse)) return r;
    r.p0 = a; r.p1 = b; r.p2 = c; r.sse = sse;
    return r;
}

// Lane holding the smallest sse (lowest lane on ties); every lane gets the same answer.
__device__ __forceinline__ int wave_argmin(double sse, int lane) {
    int idx = lane;
    for (int o = 32; o >= 1; o >>= 1) {
        const double os = __shfl_xor(sse, o, 64);
        const int oi = __shfl_xor(idx, o, 64);
        if (os < sse || (os == sse && oi < idx)) { sse = os; idx = oi; }
    }
    return idx;
}

__device__ __forceinline__ double curve_at(int cls, const Fit &f, double t, double fallback) {
    if (cls == GLM_CURVE_SUBLINEAR) {
        const double lin = (f.p0 * t + f.p1) * t + f.p2;
        return lin > 0.0 ? 1.0 / lin + f.off : fallback;
    }
    return exp(f.p1 * t + f.p2) + f.off;
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
    for (int i = lane; i < m; i += 64) {
        const double v = (double)h[start + i];
        Ls[i] = v;
        Ws[i] = pow(gamma, (double)(m - 1 - i));
        lo = fmin(lo, v); hi = fmax(hi, v);
    }
    for (int o = 32; o >= 1; o >>= 1) { lo = fmin(lo, __shfl_xor(lo, o, 64)); hi = fmax(hi, __shfl_xor(hi, o, 64)); }
    __syncthreads();
    const double last = m > 0 ? Ls[m - 1] : 0.0;
    const double span = hi - lo;
    double *fo = fit + (size_t)blockIdx.x * 8;
    double *po = pred + (size_t)blockIdx.x * horizon;
    double *go = gain + (size_t)blockIdx.x * horizon;

    if (m < 4 || !(span > 0.0)) {           // too short or flat: repeat the last loss, no reduction
        for (int hh = lane; hh < horizon; hh += 64) { po[hh] = last; go[hh] = 0.0; }
        if (lane == 0) { fo[0] = 0.0; fo[1] = 0.0; fo[2] = 0.0; fo[3] = 0.0; fo[4] = 0.0; fo[5] = 0.0; fo[6] = norm; fo[7] = (double)m; }
        return;
    }

    const int cls = jb.cls;
    const double step = (kExpHi - kExpLo) / (double)(kCand - 1);
    // level 1
    const double e1 = kExpLo + step * (double)lane;
    Fit mine = fit_for_offset(cls, Ls, Ws, m, lo - span * pow(10.0, e1));
    int gb = wave_argmin(mine.sse, lane);
    const double best1 = __shfl(mine.sse, gb, 64);
    const double e0 = kExpLo + step * (double)gb;
    Fit best;
    best.p0 = __shfl(mine.p0, gb, 64); best.p1 = __shfl(mine.p1, gb, 64); best.p2 = __shfl(mine.p2, gb, 64);
    best.off = __shfl(mine.off, gb, 64); best.sse = best1;
    if (!(best1 < INFINITY)) {              // no admissible candidate
        for (int hh = lane; hh < horizon; hh += 64) { po[hh] = last; go[hh] = 0.0; }
        if (lane == 0) { fo[0] = 0.0; fo[1] = 0.0; fo[2] = 0.0; fo[3] = 0.0; fo[4] = 0.0; fo[5] = 0.0; fo[6] = norm; fo[7] = (double)m; }
        return;
    }
    // level 2: 64 exponents in [e0 - step, e0 + step]
    const double step2 = 2.0 * step / (double)(kCand - 1);
    const double e2 = (e0 - step) + step2 * (double)lane;
    Fit mine2 = fit_for_offset(cls, Ls, Ws, m, lo - span * pow(10.0, e2));
    const int gb2 = wave_argmin(mine2.sse, lane);
    const double best2 = __shfl(mine2.sse, gb2, 64);
    if (best2 < best1) {
        best.p0 = __shfl(mine2.p0, gb2, 64); best.p1 = __shfl(mine2.p1, gb2, 64); best.p2 = __shfl(mine2.p2, gb2, 64);
        best.off = __shfl(mine2.off, gb2, 64); best.sse = best2;
    }

    const double inv = 1.0 / (double)(m - 1);
    for (int hh = lane; hh < horizon; hh += 64) {
        const double t = (double)(m - 1 + hh + 1) * inv;
        const double tp = (double)(m - 1 + hh) * inv;          // previous iteration (t = 1 for hh = 0)
        const double f = curve_at(cls, best, t, last);
        const double fp = curve_at(cls, best, tp, last);
        po[hh] = f;
        go[hh] = norm > 0.0 ? (fp - f) / norm : 0.0;
    }
    if (lane == 0) {
        fo[0] = 1.0; fo[1] = best.off; fo[2] = best.p0; fo[3] = best.p1; fo[4] = best.p2; fo[5] = best.sse;
        fo[6] = norm; fo[7] = (double)m;
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
