"""GPU parity of the L-BFGS driver against the fp64 oracle (same readings of the method on both
sides; the library holds iterates, gradients and losses in fp32, so late in a run, when loss
differences approach fp32 resolution, line-search decisions may differ: trajectories are compared
while the loss still moves, the end point by its distance from the optimum)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from oracle import lbfgs_oracle as lb
from paper_1802_04819_amd import glm, synth
from _parity import REL_TOL, rel

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _run(p, iters, memory, splits=None):
    job = glm.Job(p.X.cuda(), p.y.cuda(), p.w0.cuda().clone(), p.loss, p.lam, 0.0, iters)
    ws = glm.alloc_lbfgs_workspace(job, memory)
    st = glm.glm_lbfgs_state_t()
    for n in (splits or (iters,)):
        glm.glm_lbfgs(job, st, n, memory, ws)
    torch.cuda.synchronize()
    return job, st


@pytest.mark.parametrize("loss,N,D,lam", [(synth.LOGISTIC, 4096, 64, 1e-3), (synth.SQUARED, 5000, 100, 1e-2),
                                          (synth.LOGISTIC, 3001, 260, 1e-4), (synth.SQUARED, 2000, 1024, 1e-3)])
def test_trajectory_matches_oracle(loss, N, D, lam):
    _say(f"[case] L-BFGS parity loss={loss} N={N} D={D}")
    p = synth.make_glm(loss, N, D, seed=N + D, lam=lam, eta=0.0, K=1, col_scale=(loss == synth.SQUARED))
    iters, memory = 14, 10
    job, st = _run(p, iters, memory)
    hist, w, info = lb.run(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(D), p.lam, iters, memory)
    got = job.history().cpu().numpy()
    moving = np.abs(hist - info["f_end"]) > 1e-4 * abs(info["f_end"])       # the loss is still far from its limit
    assert moving[:3].all()
    for k in range(iters):
        if moving[k]:
            assert rel(got[k], hist[k]) <= REL_TOL, (k, got[k], hist[k])
    assert st.evals == info["evals"] or not moving.all(), (st.evals, info["evals"])
    assert rel(st.f, info["f_end"]) <= REL_TOL
    # the returned gradient is the gradient at the returned iterate
    L, g = oracle.loss_grad(p.loss, p.X.numpy(), p.y.numpy(), job.w.cpu().numpy().astype(np.float64), p.lam)
    assert rel(st.f, L) <= 1e-5
    assert np.max(np.abs(job.grad.cpu().numpy() - g)) <= 1e-4 * max(np.max(np.abs(g)), 1e-6) + 1e-7


def test_reaches_the_closed_form_optimum_and_beats_gradient_descent():
    _say("[case] L-BFGS: ridge regression optimum, and fewer iterations than gradient descent")
    p = synth.make_glm(synth.SQUARED, 6000, 48, seed=3, lam=1e-2, eta=0.05, K=30)
    job, st = _run(p, 30, 8)
    X64 = p.X.numpy().astype(np.float64); y64 = p.y.numpy().astype(np.float64)
    w_star = np.linalg.solve(X64.T @ X64 / p.N + p.lam * np.eye(p.D), X64.T @ y64 / p.N)
    f_star, _ = oracle.loss_grad(p.loss, p.X.numpy(), p.y.numpy(), w_star, p.lam)
    assert rel(st.f, f_star) <= 1e-5
    assert np.max(np.abs(job.w.cpu().numpy() - w_star)) <= 1e-3 * np.max(np.abs(w_star))
    got = job.history().cpu().numpy()
    assert np.all(np.diff(got) <= 2e-6 * np.abs(got[:-1]))
    gd = glm.Job(p.X.cuda(), p.y.cuda(), p.w0.cuda().clone(), p.loss, p.lam, p.eta, 30)
    glm.glm_step(gd, 30, glm.alloc_workspace([gd]))
    torch.cuda.synchronize()
    assert got[10] < gd.loss_hist[29].item()


def test_memory_zero_is_steepest_descent_with_the_same_line_search():
    _say("[case] L-BFGS memory 0")
    p = synth.make_glm(synth.LOGISTIC, 3000, 32, seed=5, lam=1e-3, eta=0.0, K=1)
    job, st = _run(p, 8, 0)
    hist, w, info = lb.run(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(p.D), p.lam, 8, 0)
    got = job.history().cpu().numpy()
    for k in range(8):
        assert rel(got[k], hist[k]) <= REL_TOL, (k, got[k], hist[k])
    assert st.evals == info["evals"]


def test_split_calls_continue_the_run_bit_identically():
    _say("[case] L-BFGS 3 + 4 iterations = 7, reruns identical")
    p = synth.make_glm(synth.LOGISTIC, 5000, 128, seed=6, lam=1e-4, eta=0.0, K=1)
    a, sa = _run(p, 7, 5)
    b, sb = _run(p, 7, 5)
    c, sc = _run(p, 7, 5, splits=(3, 4))
    for x, s in ((b, sb), (c, sc)):
        assert torch.equal(a.history(), x.history()) and torch.equal(a.w, x.w) and torch.equal(a.grad, x.grad)
        assert s.evals == sa.evals and s.f == sa.f
    assert sa.evals >= 8 and sa.started == 1 and sa.memory == 5


def test_hinge_loss_decreases():
    _say("[case] L-BFGS on the hinge loss (not smooth: only descent is claimed)")
    p = synth.make_glm(synth.HINGE, 4000, 64, seed=7, lam=1e-2, eta=0.0, K=1)
    job, st = _run(p, 12, 10)
    got = job.history().cpu().numpy()
    assert got[0] == 1.0 and np.all(np.isfinite(got)) and got[-1] < 0.8 and np.all(np.diff(got) <= 2e-6 * np.abs(got[:-1]))


def test_histories_fit_the_linear_convergence_class():
    _say("[case] L-BFGS histories through the predictor (class II of Sec. 2)")
    p = synth.make_glm(synth.SQUARED, 8000, 64, seed=8, lam=1e-2, eta=0.0, K=1, col_scale=True)
    job, st = _run(p, 20, 3)
    H = 4
    pred = torch.zeros(1, H, dtype=torch.float64, device="cuda"); gain = torch.zeros_like(pred)
    fit = torch.zeros(1, 8, dtype=torch.float64, device="cuda")
    view = glm.HistoryView(job); view.c.hist_len = 12
    glm.glm_predict_batched([view], glm.GLM_CURVE_LINEAR, 0.9, 128, H, pred, gain, fit)
    torch.cuda.synchronize()
    got = job.history().cpu().numpy()
    span = got[:12].max() - got[:12].min()
    assert np.all(np.isfinite(pred.cpu().numpy())) and abs(pred[0, 0].item() - got[12]) <= 0.05 * span


def test_lbfgs_errors():
    _say("[case] L-BFGS error codes")
    p = synth.make_glm(synth.LOGISTIC, 1000, 16, seed=9, lam=1e-3, eta=0.0, K=1)
    job = glm.Job(p.X.cuda(), p.y.cuda(), p.w0.cuda().clone(), p.loss, p.lam, 0.0, 4)
    ws = glm.alloc_lbfgs_workspace(job, 4)
    lib = glm.load()
    st = glm.glm_lbfgs_state_t()
    wsp, n = ctypes.c_void_p(ws.data_ptr()), ws.numel()
    assert lib.glm_lbfgs(ctypes.byref(job.c), ctypes.byref(st), 1, 33, wsp, n, None) == glm.GLM_EINVAL
    assert lib.glm_lbfgs(ctypes.byref(job.c), ctypes.byref(st), 1, -1, wsp, n, None) == glm.GLM_EINVAL
    assert lib.glm_lbfgs(ctypes.byref(job.c), None, 1, 4, wsp, n, None) == glm.GLM_EINVAL
    assert lib.glm_lbfgs(ctypes.byref(job.c), ctypes.byref(st), 5, 4, wsp, n, None) == glm.GLM_ENOSPC
    assert lib.glm_lbfgs(ctypes.byref(job.c), ctypes.byref(st), 1, 4, wsp, n - 300, None) == glm.GLM_ENOSPC
    assert st.started == 0 and st.evals == 0 and job.hist_len == 0
    glm.glm_lbfgs(job, st, 2, 4, ws)
    assert st.started == 1 and job.hist_len == 2
    assert lib.glm_lbfgs(ctypes.byref(job.c), ctypes.byref(st), 1, 5, wsp, n, None) == glm.GLM_EINVAL    # memory changed
    out = ctypes.c_size_t()
    assert lib.glm_lbfgs_workspace_bytes(ctypes.byref(job.c), 40, ctypes.byref(out)) == glm.GLM_EINVAL
