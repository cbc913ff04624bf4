// Per-sample loss l(z, y) and residual r = dl/dz in fp32, shared by the row-pass and the
// sweep kernels so that both evaluate exactly the same sequence of operations.
#pragma once

#include <hip/hip_runtime.h>

#include "slaqglm.h"

namespace slaqglm {

__device__ __forceinline__ void logistic_lr(float z, float y, float &l, float &r) {
    const float az = __builtin_fabsf(z);
    const float e = __builtin_amdgcn_exp2f(az * -1.44269504088896341f);   // e^-|z| in [0, 1]
    const float inv = __builtin_amdgcn_rcpf(1.0f + e);
    const float sig = (z >= 0.0f) ? inv : e * inv;
    // log(1 + e): series for small e, where 1 + e would round e away
    const float series = e * __builtin_fmaf(e, __builtin_fmaf(e, 0.333333333f, -0.5f), 1.0f);
    const float viaLog = __builtin_amdgcn_logf(1.0f + e) * 0.693147180559945309f;
    const float l1p = (e < 0.015625f) ? series : viaLog;
    l = __builtin_fmaf(-y, z, __builtin_fmaxf(z, 0.0f) + l1p);
    r = sig - y;
}

__device__ __forceinline__ void hinge_lr(float z, float y, float &l, float &r) {
    const float m = __builtin_fmaf(-y, z, 1.0f);
    const bool act = m > 0.0f;
    l = act ? m : 0.0f;
    r = act ? -y : 0.0f;
}

__device__ __forceinline__ void squared_lr(float z, float y, float &l, float &r) {
    const float d = z - y;
    l = 0.5f * d * d;
    r = d;
}

__device__ __forceinline__ void loss_residual(int loss, float z, float y, float &l, float &r) {
    if (loss == GLM_LOGISTIC) logistic_lr(z, y, l, r);
    else if (loss == GLM_HINGE) hinge_lr(z, y, l, r);
    else squared_lr(z, y, l, r);
}

}  // namespace slaqglm
