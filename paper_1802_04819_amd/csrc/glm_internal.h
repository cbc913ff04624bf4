// Internal declarations shared by the translation units of libslaqglm (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "slaqglm.h"

namespace slaqglm {

// Device-side view of one job for the duration of one call.  Built on the host,
// copied into the workspace, read by the kernels through scalar loads.
struct DevJob {
    const float *X;
    const float *y;
    float       *w;
    float       *grad;
    float       *loss_out;   // loss_hist + hist_len: round r of the call writes loss_out[r]
    float       *gpart;      // [P, D]  per-row-block partial sums of X^T r
    float       *lpart;      // [P]     per-row-block partial sums of the per-sample loss
    double      *wn2;        // [1]     |w|^2 of the iterate that entered the round
    double      *loss64;     // if not null: receives the loss of the call's last round before it is rounded to fp32
    float       *gpart2;     // resident kernel only: second buffers for the partials (odd rounds)
    float       *lpart2;
    void        *ctl;        // resident kernel only: barrier counter and failure flag
    long long    N;
    double       invN;
    int          D;
    int          loss;
    float        lambda;
    float        step;
    int          sched;      // glm_step_schedule_t
    long long    k0;         // iterations the job had done when the call started
    int          P;          // row blocks; a function of (N, D) only
    int          cls;        // lane-layout class; a function of D only
    int          iters;      // rounds this job takes part in during this call
    int          blk0;       // first row block of this job in the packed grid of the call
};

// Lane-layout classes of the row pass.  A row of D floats is D/4 float4 slots; a wave of 64
// lanes covers it with LPR lanes per row (64/LPR rows side by side) and C slots per lane.
constexpr int kNumClasses = 9;
struct ClassInfo { int lpr; int c; int b; int pmax; };
// b = wave-loads in flight per loop trip; pmax = cap on row blocks per job (two blocks per
// compute unit: measured best both for one large job and for many jobs packed in one launch).
__host__ __device__ constexpr ClassInfo class_info(int cls) {
    constexpr ClassInfo t[kNumClasses] = {
        {4, 1, 8, 512},     // D <= 16
        {8, 1, 8, 512},     // D <= 32
        {16, 1, 8, 512},    // D <= 64
        {32, 1, 8, 512},    // D <= 128
        {64, 1, 8, 512},    // D <= 256
        {64, 2, 8, 512},    // D <= 512
        {64, 4, 8, 1024},   // D <= 1024
        {64, 8, 2, 512},    // D <= 2048
        {64, 16, 1, 512},   // D <= 4096
    };
    return t[cls];
}
int class_of_D(int D);
int row_blocks(long long N, int cls);

constexpr int kRowBlockThreads = 256;   // 4 waves
constexpr int kFinCols = 16;            // columns per finalize block
constexpr int kFinSegs = 64;            // row-block segments summed side by side per column

// Launchers (glm_rows.hip).  `tab_*` are device pointers into the workspace.
hipError_t launch_row_pass(const DevJob *jobs, const int *blk_job, int total_blocks,
                           int max_cls, hipStream_t st);
hipError_t launch_finalize(const DevJob *jobs, const int *cblk0, int nact, int total_blocks,
                           int round, hipStream_t st);
// One job passed by value (its blk0 is 0): grid = jb.P row blocks, resp. ceil(D / kFinCols) blocks.
hipError_t launch_row_pass_one(const DevJob &jb, hipStream_t st);
hipError_t launch_finalize_one(const DevJob &jb, int round, hipStream_t st);
// Whole call of one tiny job in one launch (iters = jb.iters); needs gpart2, lpart2, ctl and
// jb.P <= resident_capacity(jb.cls).
hipError_t launch_resident(const DevJob &jb, hipStream_t st);
int resident_capacity(int cls);
// A job is run by the resident kernel when its partials are small enough for every block to add all
// of them (P * D floats) and all its row blocks fit on the chip at once.
constexpr long long kResidentMaxPartials = 16384;
hipError_t launch_read_probe(const float *src, size_t n, float *sink, hipStream_t st);
constexpr int kProbeBlocks = 512;   // two per compute unit, as the row pass: measured best for 1 GB and 16 GB

// Sweep (glm_sweep.hip).  Models run in groups of kSweepM; a group is padded to kSweepM columns of R
// and rows of Gpart.
constexpr int kSweepM = 64;
constexpr int kSweepFwdRows = 128;      // rows per forward tile
constexpr int kSweepBwdRows = 32;       // rows per backward chunk
constexpr int kSweepBwdCols = 256;      // columns per backward slab
constexpr int kSweepSplitMax = 128;     // row splits of the backward contraction
constexpr int kSweepFusedM = 16;        // a group of at most this many models runs the one-pass kernel (row lengths it takes)
constexpr int kSweepFusedBlocksMax = 1024;  // most blocks of the one-pass kernel = partial gradients per model
bool sweep_uses_fused(int D, int M);        // whether a group of M models on rows of D runs the one-pass kernel
int sweep_fused_blocks(long long N, int D); // its blocks for that shape
struct SweepArgs {            // one group of at most kSweepM models
    const float *X; const float *y; float *W; float *G;
    float *loss_row;                                // [M] the group's entries of this iteration's history row
    const float *lambdas; const float *steps;       // device copies, [M]
    float *R;        // [N, kSweepM] residuals
    float *lossP;    // [M, T] per-tile loss sums
    float *Gpart;    // [S, kSweepM, D] partial gradients
    long long N; int D, M, loss, T, S;
};
// Enqueues forward, backward and finalize of iteration k.  `ev`, if not null, points at
// four events recorded around the forward and around the backward kernel.
hipError_t launch_sweep_iteration(const SweepArgs &a, int k, hipEvent_t *ev, hipStream_t st);


// Scheduler-side steps (glm_sched.hip).
constexpr int kPredWindowMax = 128;     // most recent losses a fit may use
constexpr int kPredMinPoints = 5;       // one more than the curve with the most parameters has: fewer points are interpolated, not fitted
constexpr int kPredHorizonMax = 4096;   // future iterations a call may predict
struct PredJob {
    const float *hist;      // device: the job's loss history
    long long    n;         // entries in it
    int          cls;       // glm_curve_t
    int          pad;
};
hipError_t launch_predict(const PredJob *jobs, int J, double gamma, int window, int horizon,
                          double *pred, double *gain, double *fit, hipStream_t st);
int allocate_greedy(const double *gain, int J, int H, long long capacity, int *alloc);

// Sparse iteration (glm_sparse.hip).  All pointers are device pointers; the second block lives
// in the caller's workspace.
constexpr int kSparseChunk = 512;       // entries per wave of the segmented sums
struct SparseArgs {
    const long long *row_ptr; const int *col_idx; const float *row_val;
    const long long *col_ptr; const int *row_idx; const float *col_val;
    const float *y; float *w; float *grad; float *loss_out;
    long long N, D, nnz, nch;           // nch = ceil(nnz / kSparseChunk)
    int loss; float lambda, step;
    int sched; long long k0;            // step schedule; iterations done when the call started
    int *seg0R, *seg0C;                 // [nch + 1] segment holding each chunk's first entry
    int *closes, *headless, *slast;     // [nch] per-chunk leftovers of the pass in flight
    float *H, *T;                       // [nch]
    float *z;                           // [N] margins, immediately followed by
    float *gs;                          // [D] column sums X^T r  (gs == z + N)
    float *r;                           // [N] residuals
    float *lossP;                       // [ceil(N / 256)]
    double *wwP;                        // [ceil(D / 256)]
};
hipError_t launch_sparse_setup(const SparseArgs &a, hipStream_t st);
hipError_t launch_sparse_iteration(const SparseArgs &a, int k, hipEvent_t *ev, hipStream_t st);

}  // namespace slaqglm
