/* A plain C consumer of the library: no Python, no torch.  Builds a small logistic-regression
 * job with a fixed linear congruential generator, runs ten gradient-descent iterations through
 * glm_step and prints the losses, one per line.  The GPU test runs this program and checks what
 * the definition fixes: ln 2 at w = 0 and a decreasing loss. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "slaqglm.h"

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)

static uint32_t lcg_state = 12345u;
static float lcg_uniform(void) {           /* in (-1, 1) */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)((lcg_state >> 8) & 0xFFFFFF) / 8388608.0f - 1.0f;
}

int main(void) {
    const int64_t N = 20000; const int32_t D = 64; const int32_t iters = 10;
    float *hX = (float *)malloc(sizeof(float) * N * D), *hy = (float *)malloc(sizeof(float) * N);
    float wstar[64];
    if (!hX || !hy) return 2;
    for (int j = 0; j < D; ++j) wstar[j] = lcg_uniform();
    for (int64_t i = 0; i < N; ++i) {
        float m = 0.0f;
        for (int j = 0; j < D; ++j) { hX[i * D + j] = lcg_uniform(); m += hX[i * D + j] * wstar[j]; }
        hy[i] = m > 0.0f ? 1.0f : 0.0f;
    }
    glm_job_t job;
    float *dX, *dy, *dw, *dg, *dh;
    CHECK(hipMalloc((void **)&dX, sizeof(float) * N * D));
    CHECK(hipMalloc((void **)&dy, sizeof(float) * N));
    CHECK(hipMalloc((void **)&dw, sizeof(float) * D));
    CHECK(hipMalloc((void **)&dg, sizeof(float) * D));
    CHECK(hipMalloc((void **)&dh, sizeof(float) * iters));
    CHECK(hipMemcpy(dX, hX, sizeof(float) * N * D, hipMemcpyHostToDevice));
    CHECK(hipMemcpy(dy, hy, sizeof(float) * N, hipMemcpyHostToDevice));
    CHECK(hipMemset(dw, 0, sizeof(float) * D));
    job.X = dX; job.y = dy; job.w = dw; job.grad = dg; job.loss_hist = dh;
    job.N = N; job.D = D; job.loss = GLM_LOGISTIC; job.lambda = 1e-4f; job.step = 1.0f;
    job.hist_len = 0; job.hist_cap = iters; job.schedule = GLM_STEP_CONSTANT;
    size_t ws_bytes = 0;
    int rc = glm_workspace_bytes(&job, 1, 0, &ws_bytes);
    if (rc != GLM_OK) { fprintf(stderr, "glm_workspace_bytes: %s\n", glm_strerror(rc)); return 3; }
    void *ws;
    CHECK(hipMalloc(&ws, ws_bytes ? ws_bytes : 256));
    rc = glm_step(&job, iters, ws, ws_bytes, NULL);
    if (rc != GLM_OK) { fprintf(stderr, "glm_step: %s\n", glm_strerror(rc)); return 3; }
    CHECK(hipDeviceSynchronize());
    float hh[10];
    CHECK(hipMemcpy(hh, dh, sizeof(float) * iters, hipMemcpyDeviceToHost));
    if (job.hist_len != iters) return 4;
    for (int k = 0; k < iters; ++k) printf("%.9g\n", hh[k]);
    return 0;
}
