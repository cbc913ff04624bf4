// C-ABI entry points of the job kinds other than the dense GLM step: sparse GLM step, K-Means,
// L-BFGS.  Validation happens before anything is enqueued; see include/slaqglm.h.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "api_internal.h"
#include "glm_internal.h"
#include "kmeans_internal.h"
#include "lbfgs_internal.h"
#include "sparse_internal.h"

using namespace slaqglm;

extern "C" {

namespace {
struct SparseLayout {
    size_t seg0R, seg0C, closes, headless, slast, H, T, z, r, lossP, wwP, total;
    size_t pp, ptr2, bsum, idx2, val2, seg0P, gs2, flag;     // row-panelled column layout (P > 1)
    size_t fx_slots, fx_cnt, fx_bsum;                        // fixed-point scatter path
    size_t fx_ent[2], fx_val[2], fx_tbase[2], fx_pstart[2], fx_shift[2], fx_rstart[2], fx_rlen[2], fx_wsrc[2], fx_tfirst[2],
        fx_part[2];                                          // [0] row pass, [1] column pass
    FxPass fx_row, fx_col;
    long long nch;
    int P;
    size_t csc_ptr, csc_idx, csc_val, csc_keys[2], csc_vals[2], csc_temp, csc_temp_bytes;   // CSR-only callers
};
SparseLayout make_sparse_layout(long long N, long long D, long long nnz, bool csr_only) {
    SparseLayout L{};
    L.nch = (nnz + kSparseChunk - 1) / kSparseChunk;
    const size_t nc = (size_t)L.nch;
    size_t off = 0;
    L.seg0R = off;    off = api_align_up(off + sizeof(int) * (nc + 1));
    L.seg0C = off;    off = api_align_up(off + sizeof(int) * (nc + 1));
    L.closes = off;   off = api_align_up(off + sizeof(int) * nc);
    L.headless = off; off = api_align_up(off + sizeof(int) * nc);
    L.slast = off;    off = api_align_up(off + sizeof(int) * nc);
    L.H = off;        off = api_align_up(off + sizeof(float) * nc);
    L.T = off;        off = api_align_up(off + sizeof(float) * nc);
    L.z = off;        off = api_align_up(off + sizeof(float) * (size_t)(N + D));      // z [N] then gs [D]
    L.r = off;        off = api_align_up(off + sizeof(float) * (size_t)N);
    L.lossP = off;    off = api_align_up(off + sizeof(float) * (size_t)((N + 255) / 256));
    L.wwP = off;      off = api_align_up(off + sizeof(double) * (size_t)((D + 255) / 256));
    sparse_fx_plan(N, D, nnz, &L.fx_row, &L.fx_col);
    const bool any_fx = L.fx_row.on || L.fx_col.on;
    // the row-panelled column layout is the older remedy for the column pass; with the scatter
    // path in use it is not built
    L.P = any_fx ? 1 : sparse_panel_count(N, D);
    L.pp = L.ptr2 = L.bsum = L.idx2 = L.val2 = L.seg0P = L.gs2 = L.flag = off;
    if (L.P > 1) {
        const size_t S2 = (size_t)L.P * (size_t)D;
        L.flag = off;  off = api_align_up(off + sizeof(int));
        L.pp = off;    off = api_align_up(off + sizeof(long long) * (S2 + (size_t)D));
        L.ptr2 = off;  off = api_align_up(off + sizeof(long long) * (S2 + 1));
        L.bsum = off;  off = api_align_up(off + sizeof(long long) * ((S2 + kScanBlock - 1) / kScanBlock + 1));
        L.idx2 = off;  off = api_align_up(off + sizeof(int) * (size_t)nnz);
        L.val2 = off;  off = api_align_up(off + sizeof(float) * (size_t)nnz);
        L.seg0P = off; off = api_align_up(off + sizeof(int) * (nc + 1));
        L.gs2 = off;   off = api_align_up(off + sizeof(float) * S2);
    }
    L.fx_slots = L.fx_cnt = L.fx_bsum = off;
    for (int i = 0; i < 2; ++i)
        L.fx_ent[i] = L.fx_val[i] = L.fx_tbase[i] = L.fx_pstart[i] = L.fx_shift[i] = L.fx_rstart[i] = L.fx_rlen[i] =
            L.fx_wsrc[i] = L.fx_tfirst[i] = L.fx_part[i] = off;
    if (any_fx) {
        const FxPass *ps[2] = {&L.fx_row, &L.fx_col};
        size_t ncnt = 1;
        for (int i = 0; i < 2; ++i)
            if (ps[i]->on) ncnt = std::max(ncnt, (size_t)ps[i]->P * (size_t)ps[i]->ntiles);
        L.fx_slots = off; off = api_align_up(off + sizeof(unsigned) * kFxSlots);
        L.fx_cnt = off;   off = api_align_up(off + sizeof(long long) * (ncnt + 1));
        L.fx_bsum = off;  off = api_align_up(off + sizeof(long long) * ((ncnt + kScanBlock - 1) / kScanBlock + 2));
        for (int i = 0; i < 2; ++i) {
            if (!ps[i]->on) continue;
            const size_t cap = (size_t)ps[i]->cap, runs = (size_t)ps[i]->P * (size_t)ps[i]->W;
            L.fx_ent[i] = off;    off = api_align_up(off + sizeof(unsigned) * cap);
            L.fx_val[i] = off;    off = api_align_up(off + sizeof(float) * cap);
            L.fx_tbase[i] = off;  off = api_align_up(off + sizeof(int) * (cap / kFxRun));
            L.fx_shift[i] = off;  off = api_align_up(off + sizeof(long long) * runs);
            L.fx_rstart[i] = off; off = api_align_up(off + sizeof(long long) * runs);
            L.fx_rlen[i] = off;   off = api_align_up(off + sizeof(long long) * runs);
            L.fx_wsrc[i] = off;   off = api_align_up(off + sizeof(long long) * ((size_t)ps[i]->W + 1));
            L.fx_tfirst[i] = off; off = api_align_up(off + sizeof(long long) * ((size_t)ps[i]->W + 1));
            L.fx_pstart[i] = off; off = api_align_up(off + sizeof(long long) * ((size_t)ps[i]->P + 1));
            L.fx_part[i] = off;   off = api_align_up(off + sizeof(long long) * (size_t)ps[i]->slices * kFxPanel);
        }
    }
    L.csc_ptr = L.csc_idx = L.csc_val = L.csc_keys[0] = L.csc_keys[1] = L.csc_vals[0] = L.csc_vals[1] = L.csc_temp = off;
    L.csc_temp_bytes = 0;
    if (csr_only) {                 // the library's own column layout and the buffers of the sort that makes it
        const size_t n = (size_t)nnz;
        L.csc_ptr = off; off = api_align_up(off + sizeof(long long) * (size_t)(D + 1));
        L.csc_idx = off; off = api_align_up(off + sizeof(int) * n);
        L.csc_val = off; off = api_align_up(off + sizeof(float) * n);
        for (int i = 0; i < 2; ++i) { L.csc_keys[i] = off; off = api_align_up(off + sizeof(int) * n); }
        for (int i = 0; i < 2; ++i) { L.csc_vals[i] = off; off = api_align_up(off + sizeof(unsigned long long) * n); }
        L.csc_temp_bytes = sparse_csc_temp_bytes(nnz);
        L.csc_temp = off; off = api_align_up(off + L.csc_temp_bytes);
    }
    L.total = off;
    return L;
}
// Which workspaces hold a panelled layout, and of which matrix.  job->prepared == 1 is only
// believed when the workspace and the column arrays are the ones the layout was built from;
// anything else (a struct copied to another job, a reallocated workspace) rebuilds it.
struct PanelKey {
    const void *ws, *col_ptr, *row_idx, *col_val;
    long long N, D, nnz;
    bool operator==(const PanelKey &o) const {
        return ws == o.ws && col_ptr == o.col_ptr && row_idx == o.row_idx && col_val == o.col_val &&
               N == o.N && D == o.D && nnz == o.nnz;
    }
};
std::mutex g_panel_mu;
std::vector<PanelKey> g_panel_built;
constexpr size_t kPanelRegistryMax = 1024;

bool panel_registry_has(const PanelKey &k) {
    std::lock_guard<std::mutex> lock(g_panel_mu);
    for (const PanelKey &e : g_panel_built) if (e == k) return true;
    return false;
}
void panel_registry_put(const PanelKey &k) {
    std::lock_guard<std::mutex> lock(g_panel_mu);
    // one entry per workspace: a new layout in the same memory replaces the old one
    for (PanelKey &e : g_panel_built) if (e.ws == k.ws) { e = k; return; }
    if (g_panel_built.size() >= kPanelRegistryMax) g_panel_built.clear();   // forgotten layouts are rebuilt
    g_panel_built.push_back(k);
}

int validate_sparse_shape(const glm_sparse_job_t &j) {
    if (j.N < 1 || j.D < 1 || j.N >= (1LL << 31) || j.D >= (1LL << 31) || j.nnz < 0) return GLM_EINVAL;
    if (j.nnz / kSparseChunk >= (1LL << 31) - 8) return GLM_EINVAL;
    return GLM_OK;
}
}  // namespace

int glm_sparse_workspace_bytes(const glm_sparse_job_t *job, size_t *out_bytes) {
    if (!job || !out_bytes) return GLM_EINVAL;
    if (validate_sparse_shape(*job) != GLM_OK) return GLM_EINVAL;
    *out_bytes = make_sparse_layout(job->N, job->D, job->nnz, job->col_ptr == nullptr).total;
    return GLM_OK;
}

int glm_step_sparse(glm_sparse_job_t *job, int32_t iters, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!job || iters < 0) return GLM_EINVAL;
    const glm_sparse_job_t &j = *job;
    if (validate_sparse_shape(j) != GLM_OK) return GLM_EINVAL;
    if (!j.row_ptr || !j.y || !j.w || !j.grad || !j.loss_hist) return GLM_EINVAL;
    const bool csr_only = j.col_ptr == nullptr;         // then the library builds the column layout itself
    if (csr_only && (j.row_idx || j.col_val)) return GLM_EINVAL;
    if (j.nnz > 0 && (!j.col_idx || !j.row_val)) return GLM_EINVAL;
    if (j.nnz > 0 && !csr_only && (!j.row_idx || !j.col_val)) return GLM_EINVAL;
    const void *p4[] = {j.col_idx, j.row_val, j.row_idx, j.col_val, j.y, j.w, j.grad, j.loss_hist};
    for (const void *p : p4) if (reinterpret_cast<uintptr_t>(p) & 3u) return GLM_EINVAL;
    if ((reinterpret_cast<uintptr_t>(j.row_ptr) & 7u) || (reinterpret_cast<uintptr_t>(j.col_ptr) & 7u)) return GLM_EINVAL;
    if (j.loss < GLM_LOGISTIC || j.loss > GLM_SQUARED) return GLM_EINVAL;
    if (!std::isfinite(j.lambda) || j.lambda < 0.0f || !std::isfinite(j.step) || j.step < 0.0f) return GLM_EINVAL;
    if (j.hist_len < 0 || j.hist_cap < 0 || j.hist_len > j.hist_cap) return GLM_EINVAL;
    if (j.hist_len + (int64_t)iters > j.hist_cap) return GLM_ENOSPC;
    if (j.prepared < 0 || j.prepared > 2) return GLM_EINVAL;
    if (j.schedule != GLM_STEP_CONSTANT && j.schedule != GLM_STEP_INV_SQRT) return GLM_EINVAL;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % 256) != 0) return GLM_EINVAL;
    const SparseLayout L = make_sparse_layout(j.N, j.D, j.nnz, csr_only);
    if (ws_bytes < L.total) return GLM_ENOSPC;
    if (iters == 0) return GLM_OK;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(ws);
    SparseArgs a;
    a.row_ptr = reinterpret_cast<const long long *>(j.row_ptr); a.col_idx = j.col_idx; a.row_val = j.row_val;
    a.col_ptr = reinterpret_cast<const long long *>(j.col_ptr); a.row_idx = j.row_idx; a.col_val = j.col_val;
    SparseCsc csc{};
    if (csr_only) {
        csc.col_ptr = reinterpret_cast<long long *>(base + L.csc_ptr);
        csc.row_idx = reinterpret_cast<int *>(base + L.csc_idx);
        csc.col_val = reinterpret_cast<float *>(base + L.csc_val);
        for (int i = 0; i < 2; ++i) {
            csc.keys[i] = reinterpret_cast<int *>(base + L.csc_keys[i]);
            csc.vals[i] = reinterpret_cast<unsigned long long *>(base + L.csc_vals[i]);
        }
        csc.temp = base + L.csc_temp; csc.temp_bytes = L.csc_temp_bytes;
        a.col_ptr = csc.col_ptr; a.row_idx = csc.row_idx; a.col_val = csc.col_val;
    }
    a.y = j.y; a.w = j.w; a.grad = j.grad; a.loss_out = j.loss_hist + j.hist_len;
    a.N = j.N; a.D = j.D; a.nnz = j.nnz; a.nch = L.nch;
    a.loss = j.loss; a.lambda = j.lambda; a.step = j.step; a.sched = j.schedule; a.k0 = j.hist_len;
    a.seg0R = reinterpret_cast<int *>(base + L.seg0R); a.seg0C = reinterpret_cast<int *>(base + L.seg0C);
    a.closes = reinterpret_cast<int *>(base + L.closes); a.headless = reinterpret_cast<int *>(base + L.headless);
    a.slast = reinterpret_cast<int *>(base + L.slast);
    a.H = reinterpret_cast<float *>(base + L.H); a.T = reinterpret_cast<float *>(base + L.T);
    a.z = reinterpret_cast<float *>(base + L.z); a.gs = a.z + j.N;
    a.r = reinterpret_cast<float *>(base + L.r);
    a.lossP = reinterpret_cast<float *>(base + L.lossP); a.wwP = reinterpret_cast<double *>(base + L.wwP);
    // (for a CSR-only job the record is keyed by the row arrays: the column layout is the library's own
    // and lives in the workspace as well, so "2" cannot occur)
    const PanelKey key = csr_only ? PanelKey{ws, j.row_ptr, j.col_idx, j.row_val, j.N, j.D, j.nnz}
                                  : PanelKey{ws, j.col_ptr, j.row_idx, j.col_val, j.N, j.D, j.nnz};
    if (csr_only) {
        if (job->prepared != 1 || !panel_registry_has(key)) job->prepared = 0;
        if (job->prepared == 0 && launch_sparse_csc_build(a, csc, st) != hipSuccess) return GLM_EHIP;
    }
    if (launch_sparse_setup(a, st) != hipSuccess) return GLM_EHIP;
    SparsePanels pn;
    pn.P = L.P; pn.R = kSparsePanelRows;
    pn.pp = reinterpret_cast<long long *>(base + L.pp); pn.ptr2 = reinterpret_cast<long long *>(base + L.ptr2);
    pn.bsum = reinterpret_cast<long long *>(base + L.bsum);
    pn.idx2 = reinterpret_cast<int *>(base + L.idx2); pn.val2 = reinterpret_cast<float *>(base + L.val2);
    pn.seg0 = reinterpret_cast<int *>(base + L.seg0P); pn.gs2 = reinterpret_cast<float *>(base + L.gs2);
    pn.flag = reinterpret_cast<int *>(base + L.flag);
    SparseFx fx;
    fx.row = L.fx_row; fx.col = L.fx_col;
    fx.slots = reinterpret_cast<unsigned *>(base + L.fx_slots);
    fx.cnt = reinterpret_cast<long long *>(base + L.fx_cnt); fx.bsum = reinterpret_cast<long long *>(base + L.fx_bsum);
    {
        FxPass *ps[2] = {&fx.row, &fx.col};
        for (int i = 0; i < 2; ++i) {
            ps[i]->ent = reinterpret_cast<unsigned *>(base + L.fx_ent[i]);
            ps[i]->val = reinterpret_cast<float *>(base + L.fx_val[i]);
            ps[i]->tbase = reinterpret_cast<int *>(base + L.fx_tbase[i]);
            ps[i]->pstart = reinterpret_cast<long long *>(base + L.fx_pstart[i]);
            ps[i]->shift = reinterpret_cast<long long *>(base + L.fx_shift[i]);
            ps[i]->rstart = reinterpret_cast<long long *>(base + L.fx_rstart[i]);
            ps[i]->rlen = reinterpret_cast<long long *>(base + L.fx_rlen[i]);
            ps[i]->wsrc = reinterpret_cast<long long *>(base + L.fx_wsrc[i]);
            ps[i]->tfirst = reinterpret_cast<long long *>(base + L.fx_tfirst[i]);
            ps[i]->part = reinterpret_cast<long long *>(base + L.fx_part[i]);
        }
    }
    const bool any_fx = (fx.row.on || fx.col.on) && j.nnz > 0;
    // job->prepared: 0 = nothing built yet, 1 = auxiliary layouts in the workspace, 2 = caller's layout is used
    if (csr_only) {
        // (the layout itself was enqueued above, before anything that reads it)
    } else if (job->prepared == 1 && !((pn.P > 1 || any_fx) && j.nnz > 0 && panel_registry_has(key))) {
        job->prepared = 0;
    }
    if (any_fx && job->prepared == 0) {
        if (launch_sparse_fx_build(a, fx, st) != hipSuccess) return GLM_EHIP;
        panel_registry_put(key);
        job->prepared = 1;
    } else if (pn.P > 1 && j.nnz > 0 && job->prepared == 0) {
        if (launch_sparse_sorted_check(a, pn, st) != hipSuccess) return GLM_EHIP;
        int unsorted = 0;
        if (hipStreamSynchronize(st) != hipSuccess ||
            hipMemcpy(&unsorted, pn.flag, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess)
            return GLM_EHIP;
        if (unsorted) {
            job->prepared = 2;
        } else {
            if (launch_sparse_panel_build(a, pn, st) != hipSuccess) return GLM_EHIP;
            panel_registry_put(key);
            job->prepared = 1;
        }
    } else if (job->prepared == 0) {
        job->prepared = 2;
    }
    const bool aux_built = job->prepared == 1;          // panels or scatter layouts are in the workspace
    if (csr_only) {                                     // the column layout is: remember it either way
        if (job->prepared == 2) panel_registry_put(key);
        job->prepared = 1;
    }
    if (!aux_built) { pn.P = 1; fx.row.on = fx.col.on = 0; }
    if (!any_fx) fx.row.on = fx.col.on = 0;
    if ((fx.row.on || fx.col.on) && launch_sparse_fx_begin(a, fx, st) != hipSuccess) return GLM_EHIP;
    for (int k = 0; k < iters; ++k) {
        hipEvent_t *ev = api_profile_take(1);
        if (launch_sparse_iteration_any(a, pn, fx, k, ev, st) != hipSuccess) return GLM_EHIP;
    }
    job->hist_len += iters;
    return GLM_OK;
}

namespace {
struct KmLayout { size_t mean, Cc, cn, Cs, lossP, bestv, part, cntP, total; KmShape s; };
KmLayout make_kmeans_layout(long long N, int D, int K) {
    KmLayout L;
    L.s = km_shape(N, D, K);
    size_t off = 0;
    L.mean = off;  off = api_align_up(off + sizeof(float) * (size_t)D);
    L.Cc = off;    off = api_align_up(off + sizeof(float) * (size_t)K * D);
    L.cn = off;    off = api_align_up(off + sizeof(float) * (size_t)L.s.Kp);
    L.Cs = off;    off = api_align_up(off + sizeof(unsigned short) * 3 * (size_t)L.s.Kp * L.s.Dp);
    L.lossP = off; off = api_align_up(off + sizeof(float) * (size_t)L.s.lossN);
    L.bestv = off; off = api_align_up(off + (L.s.split && L.s.Kp > 256 ? sizeof(float) * (size_t)N : 0));
    L.part = off;  off = api_align_up(off + sizeof(float) * (size_t)L.s.P * K * D);
    L.cntP = off;  off = api_align_up(off + sizeof(int) * (size_t)L.s.P * K);
    L.total = off;
    return L;
}
int validate_kmeans_shape(const glm_kmeans_job_t &j) {
    if (j.N < 1 || j.N >= (1LL << 31)) return GLM_EINVAL;
    if (j.D < 4 || j.D > kKmMaxD || (j.D & 3)) return GLM_EINVAL;
    if (j.K < 1 || j.K > kKmMaxK) return GLM_EINVAL;
    return GLM_OK;
}
}  // namespace

int glm_kmeans_workspace_bytes(const glm_kmeans_job_t *job, size_t *out_bytes) {
    if (!job || !out_bytes) return GLM_EINVAL;
    if (validate_kmeans_shape(*job) != GLM_OK) return GLM_EINVAL;
    *out_bytes = make_kmeans_layout(job->N, job->D, job->K).total;
    return GLM_OK;
}

int glm_kmeans_step(glm_kmeans_job_t *job, int32_t iters, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!job || iters < 0) return GLM_EINVAL;
    const glm_kmeans_job_t &j = *job;
    if (validate_kmeans_shape(j) != GLM_OK) return GLM_EINVAL;
    if (!j.X || !j.C || !j.assign || !j.counts || !j.loss_hist) return GLM_EINVAL;
    if ((reinterpret_cast<uintptr_t>(j.X) & 15u) || (reinterpret_cast<uintptr_t>(j.C) & 15u)) return GLM_EINVAL;
    if ((reinterpret_cast<uintptr_t>(j.assign) & 3u) || (reinterpret_cast<uintptr_t>(j.counts) & 3u) ||
        (reinterpret_cast<uintptr_t>(j.loss_hist) & 3u))
        return GLM_EINVAL;
    if (j.hist_len < 0 || j.hist_cap < 0 || j.hist_len > j.hist_cap) return GLM_EINVAL;
    if (j.hist_len + (int64_t)iters > j.hist_cap) return GLM_ENOSPC;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % 256) != 0) return GLM_EINVAL;
    const KmLayout L = make_kmeans_layout(j.N, j.D, j.K);
    if (ws_bytes < L.total) return GLM_ENOSPC;
    if (iters == 0) return GLM_OK;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(ws);
    KmArgs a;
    a.X = j.X; a.C = j.C; a.assign = j.assign; a.counts = j.counts; a.loss_out = j.loss_hist + j.hist_len;
    a.N = j.N; a.D = j.D; a.K = j.K;
    a.mean = reinterpret_cast<float *>(base + L.mean); a.Cc = reinterpret_cast<float *>(base + L.Cc);
    a.Cs = reinterpret_cast<unsigned short *>(base + L.Cs);
    a.bestv = reinterpret_cast<float *>(base + L.bestv);
    a.cn = reinterpret_cast<float *>(base + L.cn); a.lossP = reinterpret_cast<float *>(base + L.lossP);
    a.part = reinterpret_cast<float *>(base + L.part); a.cntP = reinterpret_cast<int *>(base + L.cntP);
    a.s = L.s;
    for (int k = 0; k < iters; ++k) {
        hipEvent_t *ev = api_profile_take(2);
        if (launch_kmeans_iteration(a, k, ev, st) != hipSuccess) return GLM_EHIP;
    }
    job->hist_len += iters;
    return GLM_OK;
}

namespace {
struct LbLayout { size_t dense, S, Y, rho, yy, ring, p, wt, gt, scal, fslot, total; };
LbLayout make_lbfgs_layout(const glm_job_t &job, int memory) {
    LbLayout L;
    const size_t D = (size_t)job.D, m = (size_t)memory;
    size_t off = 0;
    L.dense = off; off = api_align_up(off + api_dense_workspace_bytes(job));
    L.S = off;     off = api_align_up(off + sizeof(float) * m * D);
    L.Y = off;     off = api_align_up(off + sizeof(float) * m * D);
    L.rho = off;   off = api_align_up(off + sizeof(double) * (m ? m : 1));
    L.yy = off;    off = api_align_up(off + sizeof(double) * (m ? m : 1));
    L.ring = off;  off = api_align_up(off + sizeof(int) * 2);
    L.p = off;     off = api_align_up(off + sizeof(float) * D);
    L.wt = off;    off = api_align_up(off + sizeof(float) * D);
    L.gt = off;    off = api_align_up(off + sizeof(float) * D);
    L.scal = off;  off = api_align_up(off + sizeof(double) * kLbScalars);
    L.fslot = off; off = api_align_up(off + 16);      // fp32 loss at +0, the same loss before rounding (fp64) at +8
    L.total = off;
    return L;
}

// Pinned landing area for the scalars read back after every evaluation.
struct LbHost { std::mutex mu; void *buf = nullptr; };
LbHost g_lb;
}  // namespace

int glm_lbfgs_workspace_bytes(const glm_job_t *job, int32_t memory, size_t *out_bytes) {
    if (!job || !out_bytes || memory < 0 || memory > kLbMaxMemory) return GLM_EINVAL;
    if (api_validate_shape(job->N, job->D) != GLM_OK) return GLM_EINVAL;
    *out_bytes = make_lbfgs_layout(*job, memory).total;
    return GLM_OK;
}

int glm_lbfgs(glm_job_t *job, glm_lbfgs_state_t *state, int32_t iters, int32_t memory, void *ws, size_t ws_bytes,
              void *hip_stream) {
    if (!job || !state || iters < 0 || memory < 0 || memory > kLbMaxMemory) return GLM_EINVAL;
    const int rc = api_validate_job(*job);
    if (rc != GLM_OK) return rc;
    if (state->started && state->memory != memory) return GLM_EINVAL;
    if (job->hist_len + (int64_t)iters > job->hist_cap) return GLM_ENOSPC;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % 256) != 0) return GLM_EINVAL;
    const LbLayout L = make_lbfgs_layout(*job, memory);
    if (ws_bytes < L.total) return GLM_ENOSPC;
    if (iters == 0) return GLM_OK;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(ws);
    LbArgs a;
    a.S = reinterpret_cast<float *>(base + L.S); a.Y = reinterpret_cast<float *>(base + L.Y);
    a.rho = reinterpret_cast<double *>(base + L.rho); a.yy = reinterpret_cast<double *>(base + L.yy);
    a.ring = reinterpret_cast<int *>(base + L.ring);
    a.p = reinterpret_cast<float *>(base + L.p); a.wt = reinterpret_cast<float *>(base + L.wt);
    a.gt = reinterpret_cast<float *>(base + L.gt);
    a.scal = reinterpret_cast<double *>(base + L.scal); a.fslot = reinterpret_cast<float *>(base + L.fslot);
    a.memory = memory; a.D = job->D;

    std::lock_guard<std::mutex> lock(g_lb.mu);
    if (!g_lb.buf && hipHostMalloc(&g_lb.buf, 256, hipHostMallocDefault) != hipSuccess) return GLM_EHIP;
    double *h_f = reinterpret_cast<double *>(static_cast<char *>(g_lb.buf) + 8);
    double *d_f = reinterpret_cast<double *>(base + L.fslot + 8);
    double *h_scal = reinterpret_cast<double *>(static_cast<char *>(g_lb.buf) + 64);

    // one evaluation: loss and gradient at w_at (step = 0 leaves w_at untouched); the loss is read back as
    // the fp64 value the finalize kernel forms before it rounds the history entry to fp32
    auto evaluate = [&](float *w_at, float *g_out, bool with_scalars) -> int {
        glm_job_t tmp = *job;
        tmp.w = w_at; tmp.grad = g_out; tmp.loss_hist = a.fslot; tmp.hist_len = 0; tmp.hist_cap = 1; tmp.step = 0.0f;
        if (api_evaluate(tmp, base + L.dense, d_f, st) != hipSuccess) return GLM_EHIP;
        if (hipMemcpyAsync(h_f, d_f, sizeof(double), hipMemcpyDeviceToHost, st) != hipSuccess) return GLM_EHIP;
        if (with_scalars &&
            hipMemcpyAsync(h_scal, a.scal, sizeof(double) * kLbScalars, hipMemcpyDeviceToHost, st) != hipSuccess)
            return GLM_EHIP;
        if (hipStreamSynchronize(st) != hipSuccess) return GLM_EHIP;
        state->evals += 1;
        return GLM_OK;
    };

    const bool fresh = !state->started;
    if (fresh) {
        const int e = evaluate(job->w, job->grad, false);
        if (e != GLM_OK) return e;
        state->f = *h_f;
        state->memory = memory;
        state->started = 1;
    }
    for (int k = 0; k < iters; ++k) {
        if (launch_lbfgs_direction(a, job->grad, fresh && k == 0, (float)state->f,
                                   job->loss_hist + job->hist_len + k, st) != hipSuccess)
            return GLM_EHIP;
        double ft = state->f;
        for (int h = 0; h <= 30; ++h) {
            if (launch_lbfgs_trial(a, job->w, h, st) != hipSuccess) return GLM_EHIP;
            const int e = evaluate(a.wt, a.gt, true);
            if (e != GLM_OK) return e;
            ft = *h_f;
            const double alpha = std::ldexp(h_scal[2], -h);
            if (ft <= state->f + 1e-4 * alpha * h_scal[0] || h == 30) break;
        }
        if (launch_lbfgs_accept(a, job->w, job->grad, st) != hipSuccess) return GLM_EHIP;
        state->f = ft;
    }
    job->hist_len += iters;
    return GLM_OK;
}

}  // extern "C"
