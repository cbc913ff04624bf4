// C-ABI entry points of libslaqglm: validation, workspace layout, launch tables, launch loops.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <numeric>
#include <vector>

#include "api_internal.h"
#include "glm_internal.h"

// Device-resident scratch of glm_step_noalloc (one copy per GPU, held until the process ends).
// In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[(8u << 20) + (64u << 10)];

namespace slaqglm {

int class_of_D(int D) {
    for (int k = 0; k < kNumClasses; ++k) {
        const ClassInfo ci = class_info(k);
        if (D <= 4 * ci.lpr * ci.c) return k;
    }
    return -1;
}

// Row blocks of a job: enough that every wave gets at least one loop trip, capped per class.
// Depends on (N, D) only, so a job is reduced in the same order whatever it is packed with.
int row_blocks(long long N, int cls) {
    const ClassInfo ci = class_info(cls);
    const long long rows_per_block_trip = 4LL * ci.b * (64 / ci.lpr);
    const long long want = (N + rows_per_block_trip - 1) / rows_per_block_trip;
    return (int)std::max<long long>(1, std::min<long long>(want, ci.pmax));
}

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_shape(long long N, int D) {
    if (N < 1 || D < 4 || D > 4096 || (D & 3) != 0) return GLM_EINVAL;
    return GLM_OK;
}

int validate_job(const glm_job_t &j) {
    if (validate_shape(j.N, j.D) != GLM_OK) return GLM_EINVAL;
    if (!j.X || !j.y || !j.w || !j.grad || !j.loss_hist) return GLM_EINVAL;
    if (!aligned16(j.X) || !aligned16(j.w)) return GLM_EINVAL;
    if ((reinterpret_cast<uintptr_t>(j.y) & 3u) || (reinterpret_cast<uintptr_t>(j.grad) & 3u) ||
        (reinterpret_cast<uintptr_t>(j.loss_hist) & 3u))
        return GLM_EINVAL;
    if (j.loss < GLM_LOGISTIC || j.loss > GLM_SQUARED) return GLM_EINVAL;
    if (!std::isfinite(j.lambda) || j.lambda < 0.0f) return GLM_EINVAL;
    if (!std::isfinite(j.step) || j.step < 0.0f) return GLM_EINVAL;
    if (j.schedule != GLM_STEP_CONSTANT && j.schedule != GLM_STEP_INV_SQRT) return GLM_EINVAL;
    if (j.hist_len < 0 || j.hist_cap < 0 || j.hist_len > j.hist_cap) return GLM_EINVAL;
    return GLM_OK;
}

// Workspace slots of one job (offsets from `off0`): partial gradients [P, D], partial losses [P],
// |w|^2; for a job small enough for the resident kernel also the second pair of partial buffers and
// the barrier words.  A function of (N, D) only.
struct JobSlots { size_t gpart, lpart, wn2, gpart2, lpart2, ctl, end; int P, cls; bool tiny; };

// Tiny: every wave of the job has at most one tile of rows (the row blocks are not capped) and
// the partials are few enough for every block to add all of them.
bool job_is_tiny(long long N, int D, int P, int cls) {
    const ClassInfo ci = class_info(cls);
    const long long rows_per_block_trip = 4LL * ci.b * (64 / ci.lpr);
    return (long long)P * D <= kResidentMaxPartials && P <= 1024 && N <= rows_per_block_trip * P;
}

JobSlots job_slots(long long N, int D, size_t off0) {
    JobSlots s;
    s.cls = class_of_D(D);
    s.P = row_blocks(N, s.cls);
    s.tiny = job_is_tiny(N, D, s.P, s.cls);
    size_t off = off0;
    // a tiny job keeps its partial losses right behind its partial gradients, and the resident kernel
    // stores every partial as a 64-bit word (tag, value)
    const size_t gbytes = s.tiny ? sizeof(unsigned long long) * ((size_t)s.P * D + (size_t)s.P)
                                 : sizeof(float) * (size_t)s.P * D;
    s.gpart = off; off = align_up(off + gbytes);
    if (s.tiny) s.lpart = s.gpart + sizeof(float) * (size_t)s.P * D;
    else { s.lpart = off; off = align_up(off + sizeof(float) * (size_t)s.P); }
    s.wn2 = off;   off = align_up(off + sizeof(double));
    s.gpart2 = s.lpart2 = s.ctl = 0;
    if (s.tiny) {
        s.gpart2 = off; off = align_up(off + gbytes);
        s.lpart2 = s.gpart2 + sizeof(float) * (size_t)s.P * D;
        s.ctl = off;    off = align_up(off + 2 * sizeof(unsigned));
    }
    s.end = off;
    return s;
}

// Workspace layout for a set of jobs: [launch tables][job 0 partials][job 1 partials]...
struct Layout {
    size_t tab_jobs = 0, tab_map = 0, tab_cblk0 = 0;    // byte offsets
    size_t tab_end = 0;                                 // tables occupy [0, tab_end)
    std::vector<JobSlots> slots;
    size_t total = 0;
};

Layout make_layout(const glm_job_t *jobs, int J) {
    Layout L;
    size_t off = 0;
    L.tab_jobs = off;  off = align_up(off + sizeof(DevJob) * (size_t)J);
    L.tab_cblk0 = off; off = align_up(off + sizeof(int) * (size_t)(J + 1));
    L.slots.resize(J);
    size_t blocks = 0;
    for (int j = 0; j < J; ++j) blocks += (size_t)row_blocks(jobs[j].N, class_of_D(jobs[j].D));
    L.tab_map = off;   off = align_up(off + sizeof(int) * blocks);   // block -> job, one int per row block
    L.tab_end = off;
    for (int j = 0; j < J; ++j) {
        L.slots[j] = job_slots(jobs[j].N, jobs[j].D, off);
        off = L.slots[j].end;
    }
    L.total = off;
    return L;
}

// Pinned host staging for the launch tables: a ring of slots, each with an event that marks the
// copy that last read it.  A call takes the next slot and waits only if the copy issued
// kStageSlots calls ago has not finished, so the host can run that many calls ahead of the device.
constexpr int kStageSlots = 8;
struct Staging {
    std::mutex mu;
    struct Slot { void *host = nullptr; size_t cap = 0; hipEvent_t ev = nullptr; bool pending = false; };
    Slot slot[kStageSlots];
    int next = 0, cur = 0;
};
Staging g_stage;

// Profiling of row-pass launches (bench only).
struct Profile {
    bool on = false;
    int cap = 0;
    std::vector<hipEvent_t> ev;   // 2 per launch
    int used = 0;
};
Profile g_prof;

// Takes the next slot of the ring, waits until the copy that last used it is done, makes it at
// least `bytes` large and returns it.  Caller holds g_stage.mu, fills the buffer, enqueues the copy
// and calls stage_mark().
hipError_t stage_acquire(size_t bytes, char **out) {
    hipError_t e;
    g_stage.cur = g_stage.next;
    g_stage.next = (g_stage.next + 1) % kStageSlots;
    Staging::Slot &sl = g_stage.slot[g_stage.cur];
    if (sl.pending) {
        if ((e = hipEventSynchronize(sl.ev)) != hipSuccess) return e;
        sl.pending = false;
    }
    if (sl.cap < bytes) {
        if (sl.host) { (void)hipHostFree(sl.host); sl.host = nullptr; sl.cap = 0; }
        const size_t want = std::max<size_t>(bytes, 1 << 16);
        if ((e = hipHostMalloc(&sl.host, want, hipHostMallocDefault)) != hipSuccess) return e;
        sl.cap = want;
    }
    if (!sl.ev) {
        if ((e = hipEventCreateWithFlags(&sl.ev, hipEventDisableTiming)) != hipSuccess) return e;
    }
    *out = static_cast<char *>(sl.host);
    return hipSuccess;
}

hipError_t stage_mark(hipStream_t st) {
    Staging::Slot &sl = g_stage.slot[g_stage.cur];
    const hipError_t e = hipEventRecord(sl.ev, st);
    if (e == hipSuccess) sl.pending = true;
    return e;
}

hipError_t run_rounds(const glm_job_t *jobs, int J, const int *iters, void *ws, hipStream_t st) {
    // Active jobs sorted by iteration count, descending (stable): the jobs still active in
    // round r are then a prefix of the table, and one table serves every round.
    std::vector<int> order;
    order.reserve(J);
    for (int j = 0; j < J; ++j) if (iters[j] > 0) order.push_back(j);
    if (order.empty()) return hipSuccess;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return iters[a] > iters[b]; });
    const int A = (int)order.size();
    const int R = iters[order[0]];

    const Layout L = make_layout(jobs, J);
    char *base = static_cast<char *>(ws);
    const size_t tab_bytes = L.tab_end;

    std::lock_guard<std::mutex> lock(g_stage.mu);
    hipError_t e;
    char *h = nullptr;
    if ((e = stage_acquire(tab_bytes, &h)) != hipSuccess) return e;
    std::memset(h, 0, tab_bytes);
    DevJob *dj = reinterpret_cast<DevJob *>(h + L.tab_jobs);
    int *blk_job = reinterpret_cast<int *>(h + L.tab_map);
    std::vector<int> blk0(A + 1, 0);
    int *cblk0 = reinterpret_cast<int *>(h + L.tab_cblk0);
    int max_cls = 0;
    cblk0[0] = 0;
    for (int a = 0; a < A; ++a) {
        const int j = order[a];
        const glm_job_t &src = jobs[j];
        const JobSlots &s = L.slots[j];
        DevJob &d = dj[a];
        d.X = src.X; d.y = src.y; d.w = src.w; d.grad = src.grad;
        d.loss_out = src.loss_hist + src.hist_len;
        d.gpart = reinterpret_cast<float *>(base + s.gpart);
        d.lpart = reinterpret_cast<float *>(base + s.lpart);
        d.wn2 = reinterpret_cast<double *>(base + s.wn2);
        d.N = src.N; d.invN = 1.0 / (double)src.N; d.D = src.D; d.loss = src.loss;
        d.lambda = src.lambda; d.step = src.step; d.sched = src.schedule; d.k0 = src.hist_len; d.P = s.P; d.cls = s.cls; d.iters = iters[j];
        max_cls = std::max(max_cls, s.cls);
        d.blk0 = blk0[a];
        for (int b = 0; b < s.P; ++b) blk_job[blk0[a] + b] = a;
        blk0[a + 1] = blk0[a] + s.P;
        cblk0[a + 1] = cblk0[a] + (src.D + kFinCols - 1) / kFinCols;
    }
    if ((e = hipMemcpyAsync(base, h, tab_bytes, hipMemcpyHostToDevice, st)) != hipSuccess) return e;
    if ((e = stage_mark(st)) != hipSuccess) return e;

    const DevJob *d_jobs = reinterpret_cast<const DevJob *>(base + L.tab_jobs);
    const int *d_map = reinterpret_cast<const int *>(base + L.tab_map);
    const int *d_cblk0 = reinterpret_cast<const int *>(base + L.tab_cblk0);
    int nact = A;
    for (int r = 0; r < R; ++r) {
        while (nact > 0 && iters[order[nact - 1]] <= r) --nact;
        const bool prof = g_prof.on && g_prof.used < g_prof.cap;
        if (prof && (e = hipEventRecord(g_prof.ev[2 * g_prof.used], st)) != hipSuccess) return e;
        if ((e = launch_row_pass(d_jobs, d_map, blk0[nact], max_cls, st)) != hipSuccess) return e;
        if (prof) {
            if ((e = hipEventRecord(g_prof.ev[2 * g_prof.used + 1], st)) != hipSuccess) return e;
            ++g_prof.used;
        }
        if ((e = launch_finalize(d_jobs, d_cblk0, nact, cblk0[nact], r, st)) != hipSuccess) return e;
    }
    return hipSuccess;
}

// One job: the descriptor travels in the kernel arguments, so nothing is staged or copied and
// the host never waits; block b of the row pass is row block b.  Same kernel bodies and the same
// workspace slots as run_rounds, hence the same bits.
// Device-side descriptor of one job whose slots start at `base`.
DevJob device_job(const glm_job_t &src, const JobSlots &s, char *base, int iters) {
    DevJob d;
    std::memset(&d, 0, sizeof(d));
    d.X = src.X; d.y = src.y; d.w = src.w; d.grad = src.grad;
    d.loss_out = src.loss_hist + src.hist_len;
    d.gpart = reinterpret_cast<float *>(base + s.gpart);
    d.lpart = reinterpret_cast<float *>(base + s.lpart);
    d.wn2 = reinterpret_cast<double *>(base + s.wn2);
    if (s.tiny) {
        d.gpart2 = reinterpret_cast<float *>(base + s.gpart2);
        d.lpart2 = reinterpret_cast<float *>(base + s.lpart2);
        d.ctl = base + s.ctl;
    }
    d.N = src.N; d.invN = 1.0 / (double)src.N; d.D = src.D; d.loss = src.loss;
    d.lambda = src.lambda; d.step = src.step; d.sched = src.schedule; d.k0 = src.hist_len;
    d.P = s.P; d.cls = s.cls; d.iters = iters; d.blk0 = 0;
    return d;
}

// A tiny job runs its whole call in one resident launch when its row blocks take at most a quarter
// of the places the chip has for them (and the iteration tags cannot overflow); everything else
// takes two launches per iteration.  The blocks of a resident launch wait for one another, so all
// of them must be on the chip together; the quarter leaves room for other work of the process (up
// to four such launches on different streams still all fit).  Should blocks be kept off the chip
// all the same, the waits are bounded and the call ends with NaN in its remaining history entries.
bool use_resident(const JobSlots &s, int iters) {
    return s.tiny && (long long)iters * s.P < (1LL << 31) && s.P <= resident_capacity(s.cls) / 4;
}

hipError_t run_single(const glm_job_t &src, int iters, void *ws, hipStream_t st, double *loss64 = nullptr) {
    if (iters <= 0) return hipSuccess;
    const JobSlots s = job_slots(src.N, src.D, make_layout(&src, 1).tab_end);
    DevJob d = device_job(src, s, static_cast<char *>(ws), iters);
    d.loss64 = loss64;
    hipError_t e;
    if (use_resident(s, iters)) {
        const bool prof = g_prof.on && g_prof.used < g_prof.cap;
        if (prof && (e = hipEventRecord(g_prof.ev[2 * g_prof.used], st)) != hipSuccess) return e;
        if ((e = launch_resident(d, st)) != hipSuccess) return e;
        if (prof) {
            if ((e = hipEventRecord(g_prof.ev[2 * g_prof.used + 1], st)) != hipSuccess) return e;
            ++g_prof.used;
        }
        return hipSuccess;
    }
    for (int r = 0; r < iters; ++r) {
        const bool prof = g_prof.on && g_prof.used < g_prof.cap;
        if (prof && (e = hipEventRecord(g_prof.ev[2 * g_prof.used], st)) != hipSuccess) return e;
        if ((e = launch_row_pass_one(d, st)) != hipSuccess) return e;
        if (prof) {
            if ((e = hipEventRecord(g_prof.ev[2 * g_prof.used + 1], st)) != hipSuccess) return e;
            ++g_prof.used;
        }
        if ((e = launch_finalize_one(d, r, st)) != hipSuccess) return e;
    }
    return hipSuccess;
}

// Scratch of glm_step_noalloc: the dense step's workspace (per-row-block partial sums) held in the
// library's own device image instead of a caller's buffer.  The largest layout of any supported
// shape is D = 4096 with 512 row blocks: 8 MiB of partial gradients plus a few KiB.
constexpr size_t kScratchBytes = (8u << 20) + (64u << 10);
constexpr int kScratchDevices = 64;
struct ScratchPtrs {
    std::mutex mu;
    void *ptr[kScratchDevices] = {};       // device address of `scratch` on each device, once known
};
ScratchPtrs g_scratch;

// Workspace layout of the sweep: [lambdas | steps][R][lossP][Gpart].
struct SweepLayout { size_t hyper, R, lossP, Gpart, total; int T, S; };

constexpr int kSweepModelsMax = 1 << 16;

SweepLayout make_sweep_layout(long long N, int D, int M) {
    SweepLayout L;
    L.T = (int)((N + kSweepFwdRows - 1) / kSweepFwdRows);
    const long long chunks = (N + kSweepBwdRows - 1) / kSweepBwdRows;
    L.S = (int)std::min<long long>(chunks, kSweepSplitMax);
    size_t off = 0;
    const size_t Mpad = (size_t)(M + kSweepM - 1) / kSweepM * kSweepM;
    L.hyper = off; off = align_up(off + sizeof(float) * 2 * Mpad);
    // residuals of the two-pass kernels; a sweep whose only group runs the one-pass kernel keeps none
    const bool needs_R = !sweep_uses_fused(D, M);
    L.R = off;     off = align_up(off + (needs_R ? sizeof(float) * (size_t)N * kSweepM : 0));
    // the one-pass kernel of a small last group keeps kSweepFusedM rows per block in the same two areas
    const size_t Gf = sweep_uses_fused(D, 1) ? (size_t)sweep_fused_blocks(N, D) : 0;
    L.lossP = off; off = align_up(off + sizeof(float) * std::max((size_t)kSweepM * L.T, Gf * kSweepFusedM));
    L.Gpart = off; off = align_up(off + sizeof(float) * std::max((size_t)L.S * kSweepM, Gf * kSweepFusedM) * D);
    L.total = off;
    return L;
}

int validate_sweep_shape(long long N, int D, int M) {
    if (N < 1 || N > (1LL << 31) * kSweepFwdRows - 1) return GLM_EINVAL;
    if (D < 4 || D > 4096 || (D % 4) != 0 || M < 1 || M > kSweepModelsMax) return GLM_EINVAL;
    return GLM_OK;
}

}  // namespace

// What the entry points of the other job kinds (glm_api_jobs.hip) use from this file.
size_t api_align_up(size_t v) { return align_up(v); }
int api_validate_shape(long long N, int D) { return validate_shape(N, D); }
int api_validate_job(const glm_job_t &j) { return validate_job(j); }
size_t api_dense_workspace_bytes(const glm_job_t &job) { return make_layout(&job, 1).total; }
hipError_t api_run_rounds(const glm_job_t *jobs, int J, const int *iters, void *ws, hipStream_t st) {
    if (J == 1) return run_single(jobs[0], iters[0], ws, st);
    return run_rounds(jobs, J, iters, ws, st);
}
hipError_t api_evaluate(const glm_job_t &job, void *ws, double *loss64, hipStream_t st) {
    glm_job_t tmp = job;
    tmp.step = 0.0f;
    return run_single(tmp, 1, ws, st, loss64);
}
hipEvent_t *api_profile_take(int launches) {
    if (!g_prof.on || g_prof.used + launches > g_prof.cap) return nullptr;
    hipEvent_t *ev = &g_prof.ev[2 * g_prof.used];
    g_prof.used += launches;
    return ev;
}
}  // namespace slaqglm

using namespace slaqglm;

extern "C" {

int glm_workspace_bytes(const glm_job_t *jobs, int32_t J, int32_t M_sweep, size_t *out_bytes) {
    if (!jobs || !out_bytes || J < 1 || M_sweep < 0) return GLM_EINVAL;
    if (M_sweep > 0) {
        if (validate_sweep_shape(jobs[0].N, jobs[0].D, M_sweep) != GLM_OK) return GLM_EINVAL;
        *out_bytes = make_sweep_layout(jobs[0].N, jobs[0].D, M_sweep).total;
        return GLM_OK;
    }
    for (int j = 0; j < J; ++j)
        if (validate_shape(jobs[j].N, jobs[j].D) != GLM_OK) return GLM_EINVAL;
    *out_bytes = make_layout(jobs, J).total;
    return GLM_OK;
}

int glm_step_batched(glm_job_t *jobs, int32_t J, const int32_t *alloc, void *ws, size_t ws_bytes,
                     void *hip_stream) {
    if (!jobs || !alloc || J < 1) return GLM_EINVAL;
    for (int j = 0; j < J; ++j) {
        const int rc = validate_job(jobs[j]);
        if (rc != GLM_OK) return rc;
        if (alloc[j] < 0) return GLM_EINVAL;
    }
    for (int j = 0; j < J; ++j)
        if (jobs[j].hist_len + (int64_t)alloc[j] > jobs[j].hist_cap) return GLM_ENOSPC;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % 256) != 0) return GLM_EINVAL;
    if (ws_bytes < make_layout(jobs, J).total) return GLM_ENOSPC;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = J == 1 ? run_single(jobs[0], alloc[0], ws, st) : run_rounds(jobs, J, alloc, ws, st);
    if (e != hipSuccess) return GLM_EHIP;
    for (int j = 0; j < J; ++j) jobs[j].hist_len += alloc[j];
    return GLM_OK;
}

int glm_step(glm_job_t *job, int32_t iters, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!job) return GLM_EINVAL;
    return glm_step_batched(job, 1, &iters, ws, ws_bytes, hip_stream);
}

size_t glm_step_noalloc_scratch_bytes(void) { return kScratchBytes; }

int glm_step_noalloc(glm_job_t *job, int32_t iters, void *hip_stream) {
    if (!job || iters < 0) return GLM_EINVAL;
    const int rc = validate_job(*job);
    if (rc != GLM_OK) return rc;
    if (job->hist_len + (int64_t)iters > job->hist_cap) return GLM_ENOSPC;
    // the slots of one job from offset 0, computed without touching the heap
    const JobSlots sl = job_slots(job->N, job->D, 0);
    if (sl.end > kScratchBytes) return GLM_ENOSPC;   // shape needs more scratch than the library holds

    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kScratchDevices) return GLM_EHIP;
    char *base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch.mu);
        if (!g_scratch.ptr[dev]) {
            // each device holds its own copy of the array at its own address; the symbol itself is
            // only a host-side handle
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GLM_EHIP;
            g_scratch.ptr[dev] = p;
        }
        base = static_cast<char *>(g_scratch.ptr[dev]);
    }
    if (iters == 0) return GLM_OK;

    const DevJob d = device_job(*job, sl, base, iters);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // Every slot of the scratch that a round reads has been written earlier in the same round
    // (each row block writes its partial row and loss, row block 0 writes |w|^2), and the barrier
    // words of the resident kernel are cleared by a kernel of their own before it starts, so
    // nothing else has to be cleared although the array keeps the previous call's contents.
    if (use_resident(sl, iters)) {
        if (launch_resident(d, st) != hipSuccess) return GLM_EHIP;
    } else {
        for (int r = 0; r < iters; ++r) {
            if (launch_row_pass_one(d, st) != hipSuccess) return GLM_EHIP;
            if (launch_finalize_one(d, r, st) != hipSuccess) return GLM_EHIP;
        }
    }
    job->hist_len += iters;
    return GLM_OK;
}

int glm_sweep(const float *X, const float *y, int64_t N, int32_t D, int32_t M, int32_t loss, float *W,
              float *G, const float *lambdas, const float *steps, int32_t iters, float *loss_hist,
              void *ws, size_t ws_bytes, void *hip_stream) {
    if (!X || !y || !W || !G || !lambdas || !steps || !loss_hist || iters < 0) return GLM_EINVAL;
    if (validate_sweep_shape(N, D, M) != GLM_OK) return GLM_EINVAL;
    if (!aligned16(X) || !aligned16(W)) return GLM_EINVAL;
    if ((reinterpret_cast<uintptr_t>(y) & 3u) || (reinterpret_cast<uintptr_t>(G) & 3u) ||
        (reinterpret_cast<uintptr_t>(loss_hist) & 3u))
        return GLM_EINVAL;
    if (loss < GLM_LOGISTIC || loss > GLM_SQUARED) return GLM_EINVAL;
    for (int m = 0; m < M; ++m) {
        if (!std::isfinite(lambdas[m]) || lambdas[m] < 0.0f) return GLM_EINVAL;
        if (!std::isfinite(steps[m]) || steps[m] < 0.0f) return GLM_EINVAL;
    }
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % 256) != 0) return GLM_EINVAL;
    const SweepLayout L = make_sweep_layout(N, D, M);
    if (ws_bytes < L.total) return GLM_ENOSPC;
    if (iters == 0) return GLM_OK;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(ws);
    const int Mpad = (M + kSweepM - 1) / kSweepM * kSweepM;
    {
        std::lock_guard<std::mutex> lock(g_stage.mu);
        char *h = nullptr;
        if (stage_acquire(sizeof(float) * 2 * (size_t)Mpad, &h) != hipSuccess) return GLM_EHIP;
        float *hf = reinterpret_cast<float *>(h);
        for (int m = 0; m < Mpad; ++m) {
            hf[m] = m < M ? lambdas[m] : 0.0f;
            hf[Mpad + m] = m < M ? steps[m] : 0.0f;
        }
        if (hipMemcpyAsync(base + L.hyper, h, sizeof(float) * 2 * (size_t)Mpad, hipMemcpyHostToDevice, st) !=
            hipSuccess)
            return GLM_EHIP;
        if (stage_mark(st) != hipSuccess) return GLM_EHIP;
    }
    // groups of kSweepM models take turns on the same R, lossP and Gpart (stream order keeps them apart)
    for (int k = 0; k < iters; ++k) {
        for (int g0 = 0; g0 < M; g0 += kSweepM) {
            SweepArgs a;
            a.X = X; a.y = y; a.W = W + (size_t)g0 * D; a.G = G + (size_t)g0 * D;
            a.loss_row = loss_hist + (size_t)k * M + g0;
            a.lambdas = reinterpret_cast<const float *>(base + L.hyper) + g0;
            a.steps = reinterpret_cast<const float *>(base + L.hyper) + Mpad + g0;
            a.R = reinterpret_cast<float *>(base + L.R);
            a.lossP = reinterpret_cast<float *>(base + L.lossP);
            a.Gpart = reinterpret_cast<float *>(base + L.Gpart);
            a.N = N; a.D = D; a.M = std::min(kSweepM, M - g0); a.loss = loss; a.T = L.T; a.S = L.S;
            hipEvent_t *ev = nullptr;
            if (g_prof.on && g_prof.used + 2 <= g_prof.cap) {
                ev = &g_prof.ev[2 * g_prof.used];
                g_prof.used += 2;
            }
            if (launch_sweep_iteration(a, k, ev, st) != hipSuccess) return GLM_EHIP;
        }
    }
    return GLM_OK;
}

int glm_predict_workspace_bytes(int32_t J, size_t *out_bytes) {
    if (J < 1 || !out_bytes) return GLM_EINVAL;
    *out_bytes = align_up(sizeof(PredJob) * (size_t)J);
    return GLM_OK;
}

int glm_predict_batched(const glm_job_t *jobs, int32_t J, const int32_t *curve, double gamma,
                        int32_t window, int32_t horizon, double *pred, double *gain, double *fit,
                        void *ws, size_t ws_bytes, void *hip_stream) {
    if (!jobs || !curve || !pred || !gain || !fit || J < 1) return GLM_EINVAL;
    if (!(gamma > 0.0) || !(gamma <= 1.0)) return GLM_EINVAL;
    if (window < kPredMinPoints || window > kPredWindowMax || horizon < 1 || horizon > kPredHorizonMax) return GLM_EINVAL;
    if ((reinterpret_cast<uintptr_t>(pred) & 7u) || (reinterpret_cast<uintptr_t>(gain) & 7u) ||
        (reinterpret_cast<uintptr_t>(fit) & 7u))
        return GLM_EINVAL;
    for (int j = 0; j < J; ++j) {
        if (!jobs[j].loss_hist || (reinterpret_cast<uintptr_t>(jobs[j].loss_hist) & 3u)) return GLM_EINVAL;
        if (jobs[j].hist_len < 1) return GLM_EINVAL;
        if (curve[j] != GLM_CURVE_SUBLINEAR && curve[j] != GLM_CURVE_LINEAR) return GLM_EINVAL;
    }
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % 256) != 0) return GLM_EINVAL;
    const size_t need = align_up(sizeof(PredJob) * (size_t)J);
    if (ws_bytes < need) return GLM_ENOSPC;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    {
        std::lock_guard<std::mutex> lock(g_stage.mu);
        char *h = nullptr;
        if (stage_acquire(need, &h) != hipSuccess) return GLM_EHIP;
        PredJob *pj = reinterpret_cast<PredJob *>(h);
        for (int j = 0; j < J; ++j) {
            pj[j].hist = jobs[j].loss_hist; pj[j].n = jobs[j].hist_len; pj[j].cls = curve[j]; pj[j].pad = 0;
        }
        if (hipMemcpyAsync(ws, h, sizeof(PredJob) * (size_t)J, hipMemcpyHostToDevice, st) != hipSuccess)
            return GLM_EHIP;
        if (stage_mark(st) != hipSuccess) return GLM_EHIP;
    }
    if (launch_predict(static_cast<const PredJob *>(ws), J, gamma, window, horizon, pred, gain, fit, st) !=
        hipSuccess)
        return GLM_EHIP;
    return GLM_OK;
}

int glm_allocate_greedy(const double *gain, int32_t J, int32_t H, int64_t capacity, int32_t *alloc) {
    if (!gain || !alloc || J < 1 || H < 1 || capacity < J) return GLM_EINVAL;
    for (size_t i = 0; i < (size_t)J * H; ++i)
        if (!std::isfinite(gain[i])) return GLM_EINVAL;
    return allocate_greedy(gain, J, H, capacity, alloc);
}

int glm_read_probe(const float *src, size_t n, float *sink, void *hip_stream) {
    if (!src || !sink || n == 0 || (n & 3) != 0 || !aligned16(src)) return GLM_EINVAL;
    return launch_read_probe(src, n, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? GLM_OK : GLM_EHIP;
}

int32_t glm_read_probe_sink_floats(void) { return kProbeBlocks; }

int glm_profile_begin(int32_t cap) {
    if (cap < 1 || cap > (1 << 20) || g_prof.on) return GLM_EINVAL;
    g_prof.ev.resize(2 * (size_t)cap);
    for (size_t i = 0; i < g_prof.ev.size(); ++i) {
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
            for (size_t k = 0; k < i; ++k) (void)hipEventDestroy(g_prof.ev[k]);
            g_prof.ev.clear();
            return GLM_EHIP;
        }
    }
    g_prof.cap = cap; g_prof.used = 0; g_prof.on = true;
    return GLM_OK;
}

int glm_profile_end(float *ms, int32_t *count) {
    if (!ms || !count || !g_prof.on) return GLM_EINVAL;
    int rc = GLM_OK;
    for (int i = 0; i < g_prof.used; ++i) {
        if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms[i], g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess)
            rc = GLM_EHIP;
    }
    *count = g_prof.used;
    for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
    g_prof.ev.clear();
    g_prof.on = false; g_prof.cap = 0; g_prof.used = 0;
    return rc;
}

const char *glm_strerror(int status) {
    switch (status) {
        case GLM_OK: return "ok";
        case GLM_EINVAL: return "invalid argument";
        case GLM_ENOSPC: return "loss history or workspace too small";
        case GLM_EHIP: return "HIP runtime error";
        case GLM_ENOTIMPL: return "not implemented";
        default: return "unknown status";
    }
}

}  // extern "C"
