// Vector work of L-BFGS between two evaluations of the objective (the evaluations themselves are
// the row pass and finalize kernels with step = 0).  D <= 4096, so one block of 1024 threads holds
// a vector with at most four elements per thread; dot products are fp64 block sums in a fixed
// order.  The ring of curvature pairs and its counters stay on the device.
//
//   direction : two-loop recursion over the stored pairs (newest to oldest, scale by s.y / y.y of
//               the newest pair, oldest to newest), p = -H g; also g.p, |g| and the first trial step
//               (1 once a pair exists, else min(1, 1/|g|)); writes the history entry.
//   trial     : wt = w + alpha p, alpha = first trial step / 2^halvings.
//   accept    : s = wt - w, y = gt - g; the pair is stored if s.y > 1e-10 y.y; w <- wt, g <- gt.
#include "lbfgs_internal.h"

namespace slaqglm {

constexpr int kLbThreads = 1024;
constexpr int kLbPer = 4;               // elements per thread (D <= 4096)

// Sum over the block, same value in every thread; red holds 16 doubles.
__device__ __forceinline__ double lb_block_sum(double v, double *red) {
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    const int wave = threadIdx.x >> 6;
    __syncthreads();                               // red may still be read from the previous call
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < kLbThreads / 64; ++w) s += red[w];
    return s;
}

__global__ __launch_bounds__(kLbThreads) void lbfgs_direction_kernel(LbArgs a, const float *__restrict__ g, int reset,
                                                                     float f_cur, float *__restrict__ hist_slot) {
    __shared__ double red[kLbThreads / 64];
    __shared__ double alpha[kLbMaxMemory];
    const int tid = threadIdx.x, D = a.D, m = a.memory;
    // The counters live in the caller's workspace: clamp them, so that a state that claims
    // "started" over memory that never held a ring cannot index outside S and Y.
    int pairs = reset ? 0 : a.ring[0];
    int head = reset ? 0 : a.ring[1];
    pairs = m == 0 ? 0 : min(max(pairs, 0), m);
    head = m == 0 ? 0 : min(max(head, 0), m - 1);
    double q[kLbPer], gv[kLbPer];
    double gg = 0.0;
#pragma unroll
    for (int e = 0; e < kLbPer; ++e) {
        const int i = tid + kLbThreads * e;
        gv[e] = i < D ? (double)g[i] : 0.0;
        q[e] = gv[e];
        gg += gv[e] * gv[e];
    }
    gg = lb_block_sum(gg, red);
    for (int t = 0; t < pairs; ++t) {                  // newest pair first
        const int i = (head - 1 - t + 2 * m) % m;
        double d = 0.0;
#pragma unroll
        for (int e = 0; e < kLbPer; ++e) {
            const int j = tid + kLbThreads * e;
            if (j < D) d += (double)a.S[(size_t)i * D + j] * q[e];
        }
        const double al = a.rho[i] * lb_block_sum(d, red);
        if (tid == 0) alpha[t] = al;
#pragma unroll
        for (int e = 0; e < kLbPer; ++e) {
            const int j = tid + kLbThreads * e;
            if (j < D) q[e] -= al * (double)a.Y[(size_t)i * D + j];
        }
    }
    if (pairs > 0) {
        const int nw = (head - 1 + m) % m;
        const double scale = (1.0 / a.rho[nw]) / a.yy[nw];
#pragma unroll
        for (int e = 0; e < kLbPer; ++e) q[e] *= scale;
    }
    __syncthreads();                                   // alpha[] complete
    for (int t = pairs - 1; t >= 0; --t) {             // oldest pair first
        const int i = (head - 1 - t + 2 * m) % m;
        double d = 0.0;
#pragma unroll
        for (int e = 0; e < kLbPer; ++e) {
            const int j = tid + kLbThreads * e;
            if (j < D) d += (double)a.Y[(size_t)i * D + j] * q[e];
        }
        const double beta = a.rho[i] * lb_block_sum(d, red);
        const double c = alpha[t] - beta;
#pragma unroll
        for (int e = 0; e < kLbPer; ++e) {
            const int j = tid + kLbThreads * e;
            if (j < D) q[e] += c * (double)a.S[(size_t)i * D + j];
        }
    }
    double gp = 0.0;
#pragma unroll
    for (int e = 0; e < kLbPer; ++e) {
        const int j = tid + kLbThreads * e;
        if (j < D) a.p[j] = (float)(-q[e]);
        gp -= gv[e] * q[e];
    }
    gp = lb_block_sum(gp, red);
    if (tid == 0) {
        const double gn = sqrt(gg);
        a.scal[0] = gp;
        a.scal[1] = gn;
        a.scal[2] = pairs > 0 ? 1.0 : (gn > 1.0 ? 1.0 / gn : 1.0);
        a.scal[3] = (double)pairs;
        if (reset) { a.ring[0] = 0; a.ring[1] = 0; }
        if (hist_slot) *hist_slot = f_cur;
    }
}

__global__ __launch_bounds__(kLbThreads) void lbfgs_trial_kernel(LbArgs a, const float *__restrict__ w, int halvings) {
    const double alpha = ldexp(a.scal[2], -halvings);
    for (int j = threadIdx.x; j < a.D; j += kLbThreads) a.wt[j] = (float)((double)w[j] + alpha * (double)a.p[j]);
}

__global__ __launch_bounds__(kLbThreads) void lbfgs_accept_kernel(LbArgs a, float *__restrict__ w, float *__restrict__ g) {
    __shared__ double red[kLbThreads / 64];
    const int tid = threadIdx.x, D = a.D, m = a.memory;
    float s[kLbPer], y[kLbPer], wn[kLbPer], gn[kLbPer];
    double sy = 0.0, yy = 0.0;
#pragma unroll
    for (int e = 0; e < kLbPer; ++e) {
        const int j = tid + kLbThreads * e;
        s[e] = y[e] = wn[e] = gn[e] = 0.0f;
        if (j < D) {
            wn[e] = a.wt[j]; gn[e] = a.gt[j];
            s[e] = (float)((double)wn[e] - (double)w[j]);
            y[e] = (float)((double)gn[e] - (double)g[j]);
            sy += (double)s[e] * (double)y[e];
            yy += (double)y[e] * (double)y[e];
        }
    }
    sy = lb_block_sum(sy, red);
    yy = lb_block_sum(yy, red);
    const int pairs = m > 0 ? min(max(a.ring[0], 0), m) : 0;
    const int head = m > 0 ? min(max(a.ring[1], 0), m - 1) : 0;
    const bool keep = m > 0 && sy > 1e-10 * yy;
    __syncthreads();                                   // every thread has read the counters
#pragma unroll
    for (int e = 0; e < kLbPer; ++e) {
        const int j = tid + kLbThreads * e;
        if (j < D) {
            if (keep) { a.S[(size_t)head * D + j] = s[e]; a.Y[(size_t)head * D + j] = y[e]; }
            w[j] = wn[e]; g[j] = gn[e];
        }
    }
    if (tid == 0 && keep) {
        a.rho[head] = 1.0 / sy;
        a.yy[head] = yy;
        a.ring[0] = pairs < m ? pairs + 1 : m;
        a.ring[1] = (head + 1) % m;
    }
}

hipError_t launch_lbfgs_direction(const LbArgs &a, const float *g, int reset, float f_cur, float *hist_slot,
                                  hipStream_t st) {
    hipLaunchKernelGGL(lbfgs_direction_kernel, dim3(1), dim3(kLbThreads), 0, st, a, g, reset, f_cur, hist_slot);
    return hipGetLastError();
}

hipError_t launch_lbfgs_trial(const LbArgs &a, const float *w, int halvings, hipStream_t st) {
    hipLaunchKernelGGL(lbfgs_trial_kernel, dim3(1), dim3(kLbThreads), 0, st, a, w, halvings);
    return hipGetLastError();
}

hipError_t launch_lbfgs_accept(const LbArgs &a, float *w, float *g, hipStream_t st) {
    hipLaunchKernelGGL(lbfgs_accept_kernel, dim3(1), dim3(kLbThreads), 0, st, a, w, g);
    return hipGetLastError();
}

}  // namespace slaqglm
