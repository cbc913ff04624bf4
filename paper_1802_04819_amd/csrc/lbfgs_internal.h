// Internal declarations of the L-BFGS driver (glm_lbfgs.hip, driven from glm_api.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace slaqglm {

constexpr int kLbMaxMemory = 32;        // curvature pairs kept at most
constexpr int kLbScalars = 8;           // doubles written by the direction kernel

// Device-side part of the state of a run; lives in the caller's workspace between calls.
struct LbArgs {
    float *S, *Y;        // [memory, D] ring of curvature pairs s = w' - w, y = g' - g
    double *rho, *yy;    // [memory]    1 / s.y and y.y of each stored pair
    int *ring;           // [2]         pairs stored, ring position of the next pair
    float *p;            // [D] search direction
    float *wt, *gt;      // [D] trial point and its gradient
    double *scal;        // [kLbScalars] g.p, |g|, first trial step, pairs
    float *fslot;        // [1] loss at the trial point
    int memory, D;
};
hipError_t launch_lbfgs_direction(const LbArgs &a, const float *g, int reset, float f_cur, float *hist_slot,
                                  hipStream_t st);
hipError_t launch_lbfgs_trial(const LbArgs &a, const float *w, int halvings, hipStream_t st);
hipError_t launch_lbfgs_accept(const LbArgs &a, float *w, float *g, hipStream_t st);

}  // namespace slaqglm
