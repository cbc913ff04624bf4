/*
 * slaqglm -- full-batch training iteration of generalized-linear-model jobs on
 * one AMD Instinct MI355X (gfx950), as a plain C ABI.
 *
 * Background.  A quality-driven cluster scheduler for ML training (SLAQ,
 * arXiv:1802.04819) runs a set J of iterative training jobs; every scheduling
 * epoch it hands each job j an allocation a_j (Sec. 2, "Scheduling Based on
 * Quality Improvements") and consumes the loss value each job produces in
 * every iteration (Sec. 2, "Normalizing Quality Metrics").  The jobs include
 * logistic regression, SVM and linear regression trained by gradient descent
 * (Sec. 2, class I; Sec. 3, "Setup").  This library is the execution layer
 * under such a scheduler for those three models: it runs iterations and
 * appends one loss value per iteration to each job's loss history.
 *
 * One iteration k of a job with data X [N, D], labels y [N], weights w_k [D]:
 *     z_i   = sum_j X[i][j] w_k[j]
 *     l_i,r_i = per-sample loss and residual dl/dz (see glm_loss_t)
 *     L_k   = (1/N) sum_i l_i + (lambda/2) |w_k|^2          -> loss_hist[hist_len + k]
 *     g_k   = (1/N) X^T r + lambda w_k                       -> grad
 *     w_k+1 = w_k - step_k * g_k                             -> w   (step_k: glm_step_schedule_t)
 * X is streamed from device memory exactly once per iteration.
 *
 * Conventions for every entry point
 *   - Returns a glm_status_t; never throws, aborts or prints.
 *   - All arguments are validated before anything is enqueued: a call that
 *     returns an error has had no effect on device memory or on the structs.
 *   - Pointers marked DEVICE are device addresses owned by the caller; the
 *     library does not allocate, free or keep them.  Pointers marked HOST are
 *     ordinary host memory, read during the call only.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns without waiting for it.
 *     Results are valid once the stream has been synchronised.  Calls that
 *     share a workspace must be ordered on one stream.
 *   - Host threads may call the entry points concurrently (on different jobs,
 *     workspaces and streams); the small host-side staging areas the library keeps
 *     are guarded by locks.  The measurement hooks at the end are the exception.
 *   - Results are deterministic: the same library, device and arguments give
 *     bit-identical loss_hist, grad and w on every run (no floating-point
 *     atomics; every reduction has a fixed order that depends only on N and D
 *     of the job, never on what else is packed into the launch).
 */
#ifndef SLAQGLM_H
#define SLAQGLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per-sample loss l(z, y) and residual r = dl/dz for margin z and label y.
 *   GLM_LOGISTIC  y in {0,1}    l = log(1 + e^z) - y z       r = 1/(1+e^-z) - y
 *   GLM_HINGE     y in {-1,+1}  l = max(0, 1 - y z)          r = -y if 1 - y z > 0, else 0
 *   GLM_SQUARED   y real        l = (z - y)^2 / 2            r = z - y
 * (logistic regression, linear SVM and linear regression of Sec. 3 "Setup"). */
typedef enum { GLM_LOGISTIC = 0, GLM_HINGE = 1, GLM_SQUARED = 2 } glm_loss_t;

/* Step of iteration k, k counted from the start of the job (= its index in loss_hist).  The paper
 * states no step schedule; both are options of this library, constant being the default:
 *   GLM_STEP_CONSTANT  step
 *   GLM_STEP_INV_SQRT  step / sqrt(k + 1), the usual decay for subgradient methods.  With it
 *                      subgradient descent on the hinge loss shows the diminishing returns that a
 *                      quality-driven scheduler relies on (Sec. 1); with a constant step its loss
 *                      falls almost linearly for hundreds of iterations. */
typedef enum { GLM_STEP_CONSTANT = 0, GLM_STEP_INV_SQRT = 1 } glm_step_schedule_t;

typedef enum {
    GLM_OK       =  0,
    GLM_EINVAL   = -1,  /* null/misaligned pointer, size or hyper-parameter out of range */
    GLM_ENOSPC   = -2,  /* loss history or workspace too small for the request */
    GLM_EHIP     = -3,  /* the HIP runtime reported an error (launch, copy, no device) */
    GLM_ENOTIMPL = -4
} glm_status_t;

/* One training job (Sec. 3 "Setup": an algorithm, a dataset, hyper-parameters
 * and the current model) together with its loss history (Sec. 2: the sequence
 * of per-iteration loss values the scheduler's predictor fits). HOST struct. */
typedef struct {
    const float *X;        /* DEVICE [N, D] fp32, row-major, leading dimension D, 16-byte aligned */
    const float *y;        /* DEVICE [N] fp32 labels / targets, encoding per glm_loss_t            */
    float       *w;        /* DEVICE [D] fp32, 16-byte aligned; in: w_k, out: w_{k+iters}          */
    float       *grad;     /* DEVICE [D] fp32; out: gradient at the iterate that entered the last
                              iteration run (untouched if no iteration ran)                        */
    float       *loss_hist;/* DEVICE [hist_cap] fp32; the call writes entries
                              hist_len .. hist_len+iters-1; entry k is L at the iterate ENTERING
                              iteration k, so entry 0 is the loss of the initial model            */
    int64_t      N;        /* rows, >= 1                                                           */
    int32_t      D;        /* columns, multiple of 4, 4 <= D <= 4096                               */
    int32_t      loss;     /* glm_loss_t                                                           */
    float        lambda;   /* L2 coefficient, finite, >= 0                                         */
    float        step;     /* gradient-descent step, finite, >= 0; 0 evaluates loss and gradient
                              and leaves w unchanged                                               */
    int64_t      hist_len; /* entries already in loss_hist (= iterations done so far); advanced by
                              the number of iterations enqueued when a call succeeds               */
    int64_t      hist_cap; /* capacity of loss_hist                                                */
    int32_t      schedule; /* glm_step_schedule_t; read by glm_step and glm_step_batched only; a run
                              split into several calls takes the same steps as one call            */
} glm_job_t;

/* Bytes of DEVICE workspace that glm_step (J = 1), glm_step_batched (J jobs) or
 * glm_sweep (M_sweep > 0: jobs[0] gives N and D, only those two fields are read)
 * need for these shapes.  The workspace holds per-block partial sums and launch
 * tables; it carries no state between calls and must be 256-byte aligned.
 * A job of a few MB (every wave holds at most one tile of rows and the partial sums
 * number at most 16384) runs a whole glm_step call in one launch whose blocks stay on
 * the chip and exchange their partial sums through the workspace; its results are
 * bit-identical to the general path.  Such a launch takes at most a quarter of the chip; its
 * blocks wait for one another with a bound (seconds), and if other work keeps part of them off
 * the chip beyond that bound the remaining history entries of the call are NaN.
 * Errors: GLM_EINVAL for a null pointer, J < 1, or a shape outside the limits. */
int glm_workspace_bytes(const glm_job_t *jobs /*HOST [J]*/, int32_t J, int32_t M_sweep,
                        size_t *out_bytes /*HOST*/);

/* Run `iters` >= 0 gradient-descent iterations of one job (Sec. 2, class I).
 * Appends `iters` values to the job's loss history and advances job->hist_len.
 * Errors: GLM_EINVAL (bad field, iters < 0), GLM_ENOSPC (hist_len + iters >
 * hist_cap, or ws_bytes below glm_workspace_bytes(job, 1, 0)), GLM_EHIP. */
int glm_step(glm_job_t *job /*HOST*/, int32_t iters, void *ws /*DEVICE*/, size_t ws_bytes,
             void *hip_stream);

/* glm_step for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results; the per-row-block partial sums live in a device array that is
 * part of the library's image (glm_step_noalloc_scratch_bytes() bytes, 8.06 MiB, held by every GPU
 * the library runs on until the process ends), which covers every shape glm_step accepts; a shape
 * whose partial sums would not fit returns GLM_ENOSPC and enqueues nothing.  The call allocates
 * and frees nothing, copies nothing and never waits for the device (the first call on a device
 * looks the array's address up once).  All calls on one GPU share the array: they must be ordered
 * on one stream, or otherwise not overlap; two calls in flight at once on one GPU race.  Nothing in
 * the array has to start at zero (every slot a round reads is written earlier in that round), so
 * whatever an earlier call left there is harmless.  Errors otherwise as glm_step. */
int glm_step_noalloc(glm_job_t *job /*HOST*/, int32_t iters, void *hip_stream);
size_t glm_step_noalloc_scratch_bytes(void);

/* One scheduling epoch for J concurrent jobs (Sec. 2 "Scheduling Based on
 * Quality Improvements": jobs j in J, allocation a_j): job j runs alloc[j] >= 0
 * iterations (0 = idle this epoch).  The jobs may differ in every field.  All
 * jobs still active in round r = 1..max_j alloc[j] are packed into one launch.
 * The result for each job is bit-identical to glm_step(&jobs[j], alloc[j]).
 * Jobs must not share w, grad or loss_hist; they may share X and y.
 * Errors as glm_step, checked for every job before anything is enqueued;
 * ws_bytes is checked against glm_workspace_bytes(jobs, J, 0). */
int glm_step_batched(glm_job_t *jobs /*HOST [J]*/, int32_t J, const int32_t *alloc /*HOST [J]*/,
                     void *ws /*DEVICE*/, size_t ws_bytes, void *hip_stream);

/* Hyper-parameter sweep (Sec. 1, "Training ML is an exploratory process"):
 * M models with their own lambda and step train on one shared X for `iters`
 * iterations; model m is exactly the job (X, y, W[m], lambdas[m], steps[m]).
 * X.W and X^T.R are computed as dense fp32 matrix products.
 *   W         DEVICE [M, D] model-major, in/out          G  DEVICE [M, D] out, last gradients
 *   loss_hist DEVICE [iters, M], entry [k, m] = L_m at the iterate entering iteration k
 *   lambdas, steps  HOST [M]
 * Models run in groups of 64 that take turns on the workspace (the time grows with ceil(M / 64); a
 * group of at most 32 models costs about two thirds of a full one; a group of at most 16 models on
 * rows of a multiple of 16 up to 1024 floats reads X once per iteration instead of twice and costs
 * about two fifths).  A model's results do not depend on which other models share its group, but a
 * model in a group of at most 16 is summed in another order than the same model in a larger group
 * (both within the tolerance of the job it equals).
 * Limits: 1 <= M <= 65536, D a multiple of 4, 4 <= D <= 4096 (else GLM_EINVAL). */
int glm_sweep(const float *X /*DEVICE*/, const float *y /*DEVICE*/, int64_t N, int32_t D, int32_t M,
              int32_t loss, float *W /*DEVICE*/, float *G /*DEVICE*/,
              const float *lambdas /*HOST*/, const float *steps /*HOST*/, int32_t iters,
              float *loss_hist /*DEVICE*/, void *ws /*DEVICE*/, size_t ws_bytes, void *hip_stream);

/* ---- L-BFGS ----------------------------------------------------------------------------- */

/* State of an L-BFGS run between calls (L-BFGS is the paper's example of a solver with linear or
 * superlinear convergence, Sec. 2 "Predicting Quality Improvement").  HOST struct owned by the
 * caller: zero it to start a run from job->w; keep it, the workspace and the job unchanged
 * between calls to continue the run. */
typedef struct {
    int32_t started;  /* set by the library once the objective has been evaluated at job->w       */
    int32_t memory;   /* curvature pairs kept, fixed by the first call                            */
    int64_t evals;    /* evaluations of the objective so far; each is one pass over X             */
    double  f;        /* loss at job->w                                                           */
} glm_lbfgs_state_t;

/* Workspace bytes for glm_lbfgs on this job with this memory (reads N, D only). */
int glm_lbfgs_workspace_bytes(const glm_job_t *job /*HOST*/, int32_t memory, size_t *out_bytes /*HOST*/);

/* `iters` L-BFGS iterations on the objective of glm_step (job->step is ignored): two-loop recursion
 * over the last `memory` (0 .. 32) curvature pairs scaled by s.y / y.y of the newest, then a
 * backtracking line search: the first trial step is 1 (min(1, 1/|g|) while no pair is stored) and is
 * halved, at most 30 times, until f(w + a p) <= f(w) + 1e-4 a g.p (the losses compared here are the
 * fp64 sums of the evaluation, before they are rounded to the fp32 history entries); a pair with
 * s.y <= 1e-10 y.y is not stored.  Every evaluation is one row pass with step = 0.
 * loss_hist[hist_len + k] receives the loss at the iterate that enters iteration k; job->w and
 * job->grad are the current iterate and its gradient when the call returns.  The call synchronises
 * with hip_stream once per evaluation (it reads the loss back to decide the line search).
 * Errors as glm_step; GLM_EINVAL also for memory outside 0 .. 32 or a memory that differs from the
 * one the run was started with. */
int glm_lbfgs(glm_job_t *job /*HOST*/, glm_lbfgs_state_t *state /*HOST*/, int32_t iters, int32_t memory,
              void *ws /*DEVICE*/, size_t ws_bytes, void *hip_stream);

/* ---- K-Means ---------------------------------------------------------------------------- */

/* A clustering job (K-Means is one of the unsupervised jobs of Sec. 3, "Setup"; it is an
 * Expectation-Maximization iteration in the sense of Sec. 1, "ML training is typically
 * iterative with diminishing returns").  One iteration, from centroids c_k:
 *   a_i = the lowest k that minimises |x_i - c_k|^2,   L = (1/N) sum_i |x_i - c_{a_i}|^2,
 *   c_k <- mean of the x_i with a_i = k (a centroid without points keeps its value).
 * loss_hist[hist_len + k] receives L at the centroids that ENTER iteration k.  HOST struct; the
 * arrays are DEVICE and owned by the caller. */
typedef struct {
    const float *X;         /* [N, D] row-major fp32, 16-byte aligned                           */
    float       *C;         /* [K, D] centroids, in/out, 16-byte aligned                        */
    int32_t     *assign;    /* [N] out: a_i of the last iteration run                           */
    int32_t     *counts;    /* [K] out: cluster sizes of the last iteration run                 */
    float       *loss_hist; /* [hist_cap]                                                       */
    int64_t      N;         /* 1 <= N < 2^31                                                    */
    int32_t      D;         /* multiple of 4, 4 <= D <= 1024                                    */
    int32_t      K;         /* 1 <= K <= 1024                                                   */
    int64_t      hist_len, hist_cap;
} glm_kmeans_job_t;

/* Workspace bytes for glm_kmeans_step on this shape (reads N, D, K only). */
int glm_kmeans_workspace_bytes(const glm_kmeans_job_t *job /*HOST*/, size_t *out_bytes /*HOST*/);

/* `iters` K-Means iterations, enqueued on hip_stream; returns without synchronising.  The
 * products x_i . c_k have fp32 accuracy on every path: on the vector units for few centroids
 * (K <= 32, or K <= 64 with K D <= 4096), else on the matrix cores (for D <= 128 as six bfloat16
 * products of three-way split operands, else in fp32).  They are taken on points and centroids
 * minus a common shift (the column means of a sample of the rows), so the distance of the data
 * from the origin does not matter; the nearest centroid is decided on |c_k|^2 - 2 x_i . c_k in
 * fp32, so where two centroids are equally near to within fp32 rounding either may be chosen; the
 * squared distance that enters L is recomputed from the definition.
 * Sums use a fixed order (no floating-point atomics in global memory): reruns are bit-identical.
 * Errors: GLM_EINVAL for bad pointers, alignment or shapes, GLM_ENOSPC if ws_bytes or the
 * history capacity is too small, GLM_EHIP if a launch fails; nothing is enqueued on
 * GLM_EINVAL / GLM_ENOSPC. */
int glm_kmeans_step(glm_kmeans_job_t *job /*HOST*/, int32_t iters, void *ws /*DEVICE*/, size_t ws_bytes,
                    void *hip_stream);

/* ---- Sparse data ------------------------------------------------------------------------ */

/* A job whose X is sparse (the paper's text and LIBSVM-style data sets, Sec. 3 "Setup").  The
 * matrix is needed twice: by rows (CSR) for the margins and by columns (CSC) for X^T r, so that
 * both are gathers with a fixed summation order.  The caller gives the row layout and either the
 * column layout as well, or col_ptr = row_idx = col_val = NULL: then the first call on the matrix
 * builds the column layout in the workspace (a stable sort of the entries by column, about 0.1 s
 * for 2e8 entries, 32 more bytes of workspace per entry).  Entries of a row / column may come in
 * any order and may repeat (repeats add).  HOST struct; the arrays are DEVICE. */
typedef struct {
    const int64_t *row_ptr;  /* [N+1] non-decreasing, row_ptr[0] = 0, row_ptr[N] = nnz            */
    const int32_t *col_idx;  /* [nnz] column of each entry, 0 <= col < D                            */
    const float   *row_val;  /* [nnz] value of each entry, in row order                             */
    const int64_t *col_ptr;  /* [D+1] the same entries grouped by column; NULL (with the next two): built by the library */
    const int32_t *row_idx;  /* [nnz] row of each entry, 0 <= row < N                               */
    const float   *col_val;  /* [nnz] value of each entry, in column order                          */
    const float   *y;        /* [N]                                                                 */
    float         *w;        /* [D] in/out                                                          */
    float         *grad;     /* [D] out                                                             */
    float         *loss_hist;/* [hist_cap], written at hist_len .. hist_len + iters - 1             */
    int64_t        N, D, nnz;/* 1 <= N, D < 2^31; 0 <= nnz                                          */
    int32_t        loss;     /* glm_loss_t                                                          */
    float          lambda, step;
    int64_t        hist_len, hist_cap;
    int32_t        prepared; /* 0 at first: the call then builds its auxiliary column layout in the
                                workspace (once) and sets this to 1 (built) or 2 (not needed or not
                                possible).  Set it back to 0 whenever the CONTENTS of the matrix or of
                                the workspace have changed.  A value of 1 is believed only for the
                                workspace address and column (CSR alone: row) arrays it was set on (the library keeps
                                a host-side record); otherwise the layout is built again.  Other
                                values: GLM_EINVAL                                                   */
    int32_t        schedule; /* glm_step_schedule_t, as in glm_job_t                                */
} glm_sparse_job_t;

/* Workspace bytes for glm_step_sparse on this shape (reads N, D, nnz and whether col_ptr is NULL).  From 4,194,304 stored
 * entries on this includes room for the library's own copies of the matrix (16 bytes per entry, a
 * few percent of padding and some tens of MB of partial sums); with more than 786,432 rows, below
 * that, for a second copy of the column layout (8 bytes per entry). */
int glm_sparse_workspace_bytes(const glm_sparse_job_t *job /*HOST*/, size_t *out_bytes /*HOST*/);

/* `iters` gradient-descent iterations of one sparse job: the same iteration as glm_step, with
 * absent entries counting as zeros.  Reads each stored entry twice per iteration (once per
 * layout).  The first call on a matrix (job->prepared == 0) may build auxiliary layouts in the
 * workspace: from 4,194,304 stored entries on (for a product whose two vectors have at most 16,777,216
 * elements each, with at least 16384
 * entries for every pair of an output panel of 16384 and a window of 262,144 gathered elements),
 * one copy per product ordered by panels of 16384
 * outputs, whose sums are then formed in LDS as 64-bit fixed-point integers (order-free, hence
 * bit-identical from run to run, and finer than the fp32 products they add); below that, with more
 * than 786,432 rows, a copy of the column layout ordered by panels of 524,288 rows, which needs the
 * rows of every column in ascending order (checked on the device; otherwise the caller's layout is
 * used as it is) and synchronises with hip_stream once.  The contents of the index arrays are
 * trusted (they live on the device); sizes, pointers and hyper-parameters are validated as in
 * glm_step, with the same error codes. */
int glm_step_sparse(glm_sparse_job_t *job /*HOST*/, int32_t iters, void *ws /*DEVICE*/, size_t ws_bytes,
                    void *hip_stream);

/* ---- Scheduler-side steps that consume the loss histories (Sec. 2) ---------------------- */

/* Convergence classes of Sec. 2 "Predicting Quality Improvement": class I, sublinear
 * (first-order methods such as gradient descent), f(k) = 1/(a k^2 + b k + c) + d; class II,
 * linear or superlinear, f(k) = mu^(k-b) + c. */
typedef enum { GLM_CURVE_SUBLINEAR = 1, GLM_CURVE_LINEAR = 2 } glm_curve_t;

/* For each of J jobs: normalise the loss changes by the largest change seen so far (Sec. 2,
 * "Normalizing Quality Metrics"), fit the job's convergence curve to its exponentially weighted
 * loss history and evaluate it at the next `horizon` iterations (Sec. 2, "Predicting Quality
 * Improvement").  Of each job only loss_hist (DEVICE) and hist_len are read.
 * The fit is the weighted least-squares problem over all parameters of the curve: with the last
 * m <= window losses L_i at scaled times t_i = i/(m-1) and weights gamma^(m-1-i),
 *     minimise sum_i w_i (f(t_i) - L_i)^2,
 *     class I  f(t) = 1/(p0 t^2 + p1 t + p2) + offset  (positive denominator on the window),
 *     class II f(t) = exp(p0 t + p1) + offset,
 * the offset (the asymptote d, resp. c) confined to min L - span 10^e with -4 <= e <= 2, span the
 * range of the window (the paper gives no domain; without one a history that falls along a
 * straight line has no minimiser).  The problem is not convex; the library scans e, refines the
 * deepest valleys and returns the best local minimum it finds.
 *   curve   HOST [J] glm_curve_t per job
 *   gamma   weight decay per iteration, 0 < gamma <= 1: history point i of n weighs gamma^(n-1-i)
 *   window  most recent losses used for the fit, 5 <= window <= 128
 *   pred    DEVICE [J, horizon] fp64: predicted loss after h = 1..horizon further iterations
 *   gain    DEVICE [J, horizon] fp64: predicted reduction contributed by the h-th further
 *           iteration, divided by the largest single-iteration change in the job's history
 *   fit     DEVICE [J, 8] fp64: {fitted (1/0), offset, p0, p1, p2 (0 for class II), weighted squared
 *           error, largest change, points used}.  A job with fewer than 5 losses (class I has four
 *           parameters: fewer points would be interpolated, not fitted), a flat or non-finite
 *           history or no admissible fit gets fitted = 0, pred = its last loss, gain = 0.
 *   ws      DEVICE workspace of glm_predict_workspace_bytes(J) bytes, 256-byte aligned
 * Every job needs hist_len >= 1.  Errors: GLM_EINVAL, GLM_ENOSPC (workspace), GLM_EHIP. */
int glm_predict_batched(const glm_job_t *jobs /*HOST [J]*/, int32_t J, const int32_t *curve /*HOST*/,
                        double gamma, int32_t window, int32_t horizon, double *pred /*DEVICE*/,
                        double *gain /*DEVICE*/, double *fit /*DEVICE*/, void *ws /*DEVICE*/,
                        size_t ws_bytes, void *hip_stream);
int glm_predict_workspace_bytes(int32_t J, size_t *out_bytes /*HOST*/);

/* The greedy allocation of Sec. 2 "Scheduling Based on Quality Improvements": every job starts
 * with one unit; one unit at a time goes to the job whose next unit has the largest predicted
 * reduction (lowest job index on ties) until `capacity` units are handed out or every job holds
 * H units.  gain is HOST [J, H] (entry [j, h-1] = reduction of job j's h-th unit, as written by
 * glm_predict_batched and copied to the host), alloc HOST [J] out.  Runs on the host.
 * Errors: GLM_EINVAL (null pointer, J < 1, H < 1, capacity < J, a gain that is not finite). */
int glm_allocate_greedy(const double *gain /*HOST*/, int32_t J, int32_t H, int64_t capacity,
                        int32_t *alloc /*HOST*/);

/* Measurement aid: reads n floats of DEVICE memory once with the same 128-bit
 * access pattern as the training kernels and writes one float per block to
 * `sink` (DEVICE, at least glm_read_probe_sink_floats() floats), so a caller
 * can time the attainable streaming-read rate of the device.  n % 4 == 0. */
int glm_read_probe(const float *src /*DEVICE*/, size_t n, float *sink /*DEVICE*/, void *hip_stream);
int32_t glm_read_probe_sink_floats(void);

/* Per-launch timing of the row-pass kernel (the one that streams X), for
 * roofline reporting.  After glm_profile_begin(cap) every row-pass launch is
 * bracketed by HIP events on its own stream, up to cap launches.
 * glm_profile_end waits for those events, writes the durations in milliseconds
 * to ms[0..*count-1] (HOST, room for cap values) and turns recording off.
 * Not thread-safe; meant for a benchmark's single thread. */
int glm_profile_begin(int32_t cap);
int glm_profile_end(float *ms /*HOST*/, int32_t *count /*HOST*/);

/* Static text for a status code. */
const char *glm_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SLAQGLM_H */
