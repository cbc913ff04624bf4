"""The scheduling loop of Sec. 2 over jobs of different kinds on one GPU: dense GLM jobs, a sparse
GLM job and K-Means jobs train for a few epochs; after every epoch the predictor reads all loss
histories (losses of very different ranges, made comparable by the normaliser) and the greedy
allocator hands out the next epoch's iterations.  Checked: the loop runs end to end through the
C ABI, every job keeps at least one unit, the predictions handed to the allocator are those of the
oracle, and for the same total number of iterations the quality-driven run ends with a lower mean
normalised loss than equal shares.
"""
import numpy as np
import pytest
import torch

from oracle import sched_oracle as so
from paper_1802_04819_amd import glm, synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


class _Dense:
    def __init__(self, p, cap):
        self.job = glm.Job(p.X, p.y, p.w0.clone(), p.loss, p.lam, p.eta, cap)
        self.ws = glm.alloc_workspace([self.job])
        self.curve = glm.GLM_CURVE_LINEAR if p.loss == synth.SQUARED else glm.GLM_CURVE_SUBLINEAR

    def step(self, n):
        glm.glm_step(self.job, n, self.ws)


class _Sparse:
    def __init__(self, p, cap):
        self.job = glm.SparseJob(p.row_ptr, p.col_idx, p.row_val, p.col_ptr, p.row_idx, p.col_val, p.y,
                                 p.w0.clone(), p.loss, p.lam, p.eta, cap)
        self.ws = glm.alloc_sparse_workspace(self.job)
        self.curve = glm.GLM_CURVE_SUBLINEAR

    def step(self, n):
        glm.glm_step_sparse(self.job, n, self.ws)


class _KMeans:
    def __init__(self, p, cap):
        self.job = glm.KMeansJob(p.X, p.C0.clone(), cap)
        self.ws = glm.alloc_kmeans_workspace(self.job)
        self.curve = glm.GLM_CURVE_LINEAR          # Lloyd iterations converge fast (class II of Sec. 2)

    def step(self, n):
        glm.glm_kmeans_step(self.job, n, self.ws)


def _make_jobs(cap):
    d = "cuda"
    return [
        _Dense(synth.make_glm(synth.LOGISTIC, 20000, 64, 1, lam=1e-4, eta=0.5, K=1, device=d), cap),
        _Dense(synth.make_glm(synth.SQUARED, 30000, 32, 2, lam=1e-3, eta=0.05, K=1, device=d), cap),
        _Dense(synth.make_glm(synth.LOGISTIC, 8000, 256, 3, lam=1e-4, eta=1.0, K=1, device=d), cap),
        _Sparse(synth.make_sparse_glm(synth.LOGISTIC, 30000, 5000, 20.0, 4, lam=1e-5, eta=2.0, K=1, device=d), cap),
        _KMeans(synth.make_kmeans(40000, 32, 24, 5, blobs=12, device=d), cap),
        _KMeans(synth.make_kmeans(20000, 64, 10, 6, device=d), cap),
    ]


def _run(policy, E, H, C, warm):
    jobs = _make_jobs(max(warm) + E * H)
    J = len(jobs)
    for j, w in zip(jobs, warm):                   # jobs arrive with different amounts of progress
        j.step(w)
    pred = torch.zeros(J, H, dtype=torch.float64, device="cuda"); gain = torch.zeros_like(pred)
    fit = torch.zeros(J, 8, dtype=torch.float64, device="cuda")
    allocs = []
    for e in range(E):
        if policy == "greedy":
            views = [glm.HistoryView(j.job) for j in jobs]
            glm.glm_predict_batched(views, [j.curve for j in jobs], 0.9, 128, H, pred, gain, fit)
            torch.cuda.synchronize()
            g = gain.cpu().numpy()
            if e == 0:                              # what the allocator consumes is what the oracle predicts
                for i, j in enumerate(jobs):
                    h = j.job.history().cpu().numpy().astype(np.float64)
                    _, g_o, f_o = so.predict_job(h, j.curve, 0.9, 128, H)
                    scale = max(np.max(np.abs(g_o)), 1e-12)
                    assert np.max(np.abs(g[i] - g_o)) <= 1e-4 * scale + 1e-9, (i, g[i], g_o)
            alloc = glm.glm_allocate_greedy(g, C)
            assert alloc.sum() == C and alloc.min() >= 1 and alloc.max() <= H
        else:
            alloc = np.full(J, C // J, np.int32)
        allocs.append(alloc)
        for j, a in zip(jobs, alloc):
            j.step(int(a))
    torch.cuda.synchronize()
    return [j.job.history().cpu().numpy() for j in jobs], allocs


def test_mixed_jobs_closed_loop():
    _say("[case] closed loop over dense, sparse and K-Means jobs")
    E, H = 5, 12
    warm = [6, 30, 10, 8, 5, 12]
    C = 4 * len(warm)
    fair, _ = _run("fair", E, H, C, warm)
    greedy, allocs = _run("greedy", E, H, C, warm)
    for f, g, w in zip(fair, greedy, warm):
        assert len(f) == w + E * (C // len(warm)) and np.all(np.isfinite(g)) and len(g) >= w + E
        assert np.array_equal(f[:w], g[:w])                         # same warm-up, bit for bit
    assert any(len(set(a.tolist())) > 1 for a in allocs)            # the allocation is not uniform
    floor = [min(f.min(), g.min()) for f, g in zip(fair, greedy)]

    def mean_norm(hs):
        return float(np.mean([(h[-1] - lo) / (h[0] - lo) for h, lo in zip(hs, floor)]))
    _say(f"  mean normalised loss: equal shares {mean_norm(fair):.4f}, quality-driven {mean_norm(greedy):.4f}; "
         f"allocations {[a.tolist() for a in allocs]}")
    assert mean_norm(greedy) <= mean_norm(fair), (mean_norm(greedy), mean_norm(fair))


def test_normalised_loss_changes_fall_from_one_towards_zero_for_every_kind_of_job():
    # Sec. 2, "Normalizing Quality Metrics" (and the figure it refers to): whatever the range of the
    # loss, the change per iteration, divided by the largest change seen so far, starts at 1 and
    # decays towards 0 for the common algorithms.  Checked on the library's own histories.
    _say("[case] normalised loss changes of GD (logistic, hinge, squared), sparse GD, L-BFGS and K-Means")
    d = "cuda"
    K = 40
    hists = {}
    for name, p in (("logistic", synth.make_glm(synth.LOGISTIC, 20000, 64, 11, lam=1e-4, eta=0.5, K=K, device=d)),
                    ("hinge", synth.make_glm(synth.HINGE, 20000, 64, 12, lam=1e-4, eta=0.05, K=K, device=d)),
                    ("squared", synth.make_glm(synth.SQUARED, 20000, 64, 13, lam=1e-3, eta=0.05, K=K, device=d))):
        j = _Dense(p, K); j.step(K); hists[name] = j.job
    # the sparse problem is badly conditioned (power-law column popularity): it needs more iterations
    s = _Sparse(synth.make_sparse_glm(synth.LOGISTIC, 30000, 5000, 20.0, 14, lam=1e-5, eta=2.0, K=K, device=d), 8 * K)
    s.step(8 * K); hists["sparse logistic"] = s.job
    km = _KMeans(synth.make_kmeans(40000, 32, 24, 15, blobs=12, device=d), K)
    km.step(K); hists["kmeans"] = km.job
    p = synth.make_glm(synth.LOGISTIC, 20000, 64, 16, lam=1e-4, eta=0.0, K=K, device=d)
    lj = glm.Job(p.X, p.y, p.w0.clone(), p.loss, p.lam, 0.0, K)
    glm.glm_lbfgs(lj, glm.glm_lbfgs_state_t(), K, 10, glm.alloc_lbfgs_workspace(lj, 10))
    hists["lbfgs"] = lj
    torch.cuda.synchronize()
    for name, job in hists.items():
        h = job.history().cpu().numpy().astype(np.float64)
        nu, norm = so.normalized_changes(h)
        assert nu[0] == 1.0 and np.all(np.abs(nu) <= 1.0) and norm > 0, name
        head, tail = np.abs(nu[:5]).mean(), np.abs(nu[-5:]).mean()
        _say(f"  {name:16s} loss {h[0]:.4g} -> {h[-1]:.4g}; mean |normalised change| first 5: {head:.3f}, last 5: {tail:.4f}")
        assert tail < 0.25 * head and tail < 0.2, (name, head, tail)
