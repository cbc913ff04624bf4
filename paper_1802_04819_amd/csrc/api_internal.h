// Shared between the translation units that hold the C-ABI entry points (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

#include "slaqglm.h"

namespace slaqglm {

size_t api_align_up(size_t v);                         // workspace offsets are multiples of 256 bytes
int api_validate_shape(long long N, int D);            // GLM_OK or GLM_EINVAL
int api_validate_job(const glm_job_t &j);              // pointers, alignment, hyper-parameters, history
size_t api_dense_workspace_bytes(const glm_job_t &job);
// `iters[j]` iterations of each job (row pass + finalize per round), enqueued on st.
hipError_t api_run_rounds(const glm_job_t *jobs, int J, const int *iters, void *ws, hipStream_t st);
// One evaluation of loss and gradient at job.w (step 0: w is left alone); the loss goes to
// job.loss_hist[job.hist_len] in fp32 and, unrounded, to *loss64 (device).
hipError_t api_evaluate(const glm_job_t &job, void *ws, double *loss64, hipStream_t st);
// While a profile is being recorded: 2 * launches events to bracket `launches` kernel launches, else nullptr.
hipEvent_t *api_profile_take(int launches);

}  // namespace slaqglm
