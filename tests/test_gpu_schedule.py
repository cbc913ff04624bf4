"""Gradient descent with the decaying step eta / sqrt(k + 1) against the oracle's scheduled run:
per step, as a trajectory, split over calls, inside a batched epoch, and what it is for: hinge-loss
jobs whose loss curve flattens (the diminishing returns the scheduler relies on)."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_1802_04819_amd import glm, synth
from _parity import REL_TOL, check_step_against_oracle, rel

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _job(p, cap, schedule, step=None):
    return glm.Job(p.X.cuda(), p.y.cuda(), p.w0.cuda().clone(), p.loss, p.lam, p.eta if step is None else step, cap,
                   schedule=schedule)


@pytest.mark.parametrize("loss,eta", [(synth.LOGISTIC, 1.0), (synth.HINGE, 0.2), (synth.SQUARED, 0.3)])
@pytest.mark.parametrize("N,D", [(5000, 64), (3001, 260)])
def test_each_step_of_the_decaying_schedule(loss, eta, N, D):
    _say(f"[case] step / sqrt(k + 1), per step: loss {loss}, {N} x {D}")
    p = synth.make_glm(loss, N, D, seed=31, lam=1e-3, eta=eta, K=6)
    job = _job(p, 6, glm.GLM_STEP_INV_SQRT)
    ws = glm.alloc_workspace([job])
    Xn, yn = p.X.numpy(), p.y.numpy()
    for k in range(6):
        w_in = job.w.cpu().numpy().astype(np.float64)
        glm.glm_step(job, 1, ws)                      # hist_len carries k into the next call
        torch.cuda.synchronize()
        _, g = check_step_against_oracle(p.loss, Xn, yn, w_in, p.lam, job.loss_hist[k].item(), job.grad.cpu().numpy(),
                                         tag=f"k={k}")
        eta_k = eta / math.sqrt(k + 1)
        w_ref = w_in - eta_k * g
        scale = max(np.max(np.abs(w_ref)), eta_k * np.max(np.abs(g)), 1e-30)
        assert np.max(np.abs(job.w.cpu().numpy() - w_ref)) <= REL_TOL * scale, ("update", k)
        # and it is not the constant step (from the second iteration on)
        if k >= 1:
            w_const = w_in - eta * g
            assert np.max(np.abs(job.w.cpu().numpy() - w_const)) > 10 * REL_TOL * scale


@pytest.mark.parametrize("loss,eta", [(synth.LOGISTIC, 1.0), (synth.SQUARED, 0.3)])
def test_trajectory_matches_the_oracles_scheduled_run(loss, eta):
    _say(f"[case] step / sqrt(k + 1), 40-iteration trajectory, loss {loss}")
    p = synth.make_glm(loss, 8000, 128, seed=32, lam=1e-3, eta=eta, K=40)
    job = _job(p, 40, glm.GLM_STEP_INV_SQRT)
    glm.glm_step(job, 40, glm.alloc_workspace([job]))
    torch.cuda.synchronize()
    lh, gh, w, _ = oracle.run_schedule(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(p.D), p.lam, eta, oracle.INV_SQRT, 40)
    got = job.history().cpu().numpy()
    assert max(rel(a, b) for a, b in zip(got, lh)) <= REL_TOL
    assert np.max(np.abs(job.w.cpu().numpy() - w)) <= REL_TOL * np.max(np.abs(w))
    assert rel(float(np.linalg.norm(job.grad.cpu().numpy().astype(np.float64))), gh[-1]) <= REL_TOL


def test_split_calls_and_batched_epochs_take_the_same_steps():
    _say("[case] step / sqrt(k + 1): 7 = 3 + 4 iterations, alone and inside a batched epoch, bit for bit")
    ps = [synth.make_glm(l, n, d, seed=33 + i, lam=1e-3, eta=e, K=7)
          for i, (l, n, d, e) in enumerate([(synth.LOGISTIC, 4000, 64, 1.0), (synth.HINGE, 2500, 100, 0.2),
                                            (synth.SQUARED, 3000, 256, 0.3)])]
    scheds = [glm.GLM_STEP_INV_SQRT, glm.GLM_STEP_INV_SQRT, glm.GLM_STEP_CONSTANT]
    ref = []
    for p, s in zip(ps, scheds):
        job = _job(p, 7, s)
        glm.glm_step(job, 7, glm.alloc_workspace([job]))
        torch.cuda.synchronize()
        ref.append((job.history().cpu().clone(), job.w.cpu().clone()))
    jobs = [_job(p, 7, s) for p, s in zip(ps, scheds)]
    ws = glm.alloc_workspace(jobs)
    glm.glm_step_batched(jobs, np.array([3, 2, 3], np.int32), ws)
    glm.glm_step_batched(jobs, np.array([4, 5, 4], np.int32), ws)
    torch.cuda.synchronize()
    for job, (h, w) in zip(jobs, ref):
        assert torch.equal(job.history().cpu(), h) and torch.equal(job.w.cpu(), w)


def test_hinge_loss_flattens_under_the_decaying_step():
    """With the small constant steps of the concurrent-jobs mix, subgradient descent on the hinge
    loss falls linearly for hundreds of iterations (every sample stays active, the gradient hardly
    changes); with step / sqrt(k + 1) it can start with a large step and the per-iteration change
    shrinks, which is what the normaliser and the predictor of Sec. 2 assume (Sec. 1: diminishing
    returns)."""
    _say("[case] hinge loss, constant against decaying step: size of the late changes")
    p = synth.make_glm(synth.HINGE, 20000, 128, seed=35, lam=1e-4, eta=0.002, K=120)
    out = {}
    for name, sched, step in (("constant", glm.GLM_STEP_CONSTANT, 0.002), ("decaying", glm.GLM_STEP_INV_SQRT, 0.2)):
        job = _job(p, 120, sched, step=step)
        glm.glm_step(job, 120, glm.alloc_workspace([job]))
        torch.cuda.synchronize()
        h = job.history().cpu().numpy().astype(np.float64)
        d = -np.diff(h)
        out[name] = (d[:10].mean(), d[-20:].mean(), h[-1])
        _say(f"  {name}: mean change of the first 10 iterations {d[:10].mean():.3e}, of the last 20 {d[-20:].mean():.3e}, "
             f"loss {h[0]:.3f} -> {h[-1]:.3f}")
    assert out["constant"][1] > 0.9 * out["constant"][0]          # still falling at the initial rate
    assert out["decaying"][1] < 0.05 * out["decaying"][0]         # flattened
    assert out["decaying"][2] < out["constant"][2]                # and further down


@pytest.mark.parametrize("loss,eta", [(synth.LOGISTIC, 1.0), (synth.HINGE, 0.2)])
def test_sparse_job_with_the_decaying_schedule(loss, eta):
    _say(f"[case] sparse, step / sqrt(k + 1): trajectory against the oracle and 6 = 2 + 4 iterations, loss {loss}")
    p = synth.make_sparse_glm(loss, 20000, 3000, 12.0, seed=36, lam=1e-4, eta=eta, K=6)
    t = lambda x: x.cuda()

    def job():
        return glm.SparseJob(t(p.row_ptr), t(p.col_idx), t(p.row_val), t(p.col_ptr), t(p.row_idx), t(p.col_val), t(p.y),
                             p.w0.cuda().clone(), p.loss, p.lam, eta, 6, schedule=glm.GLM_STEP_INV_SQRT)
    a = job()
    glm.glm_step_sparse(a, 6, glm.alloc_sparse_workspace(a))
    b = job()
    ws = glm.alloc_sparse_workspace(b)
    glm.glm_step_sparse(b, 2, ws); glm.glm_step_sparse(b, 4, ws)
    torch.cuda.synchronize()
    assert torch.equal(a.history(), b.history()) and torch.equal(a.w, b.w)
    lh, gh, w, _ = oracle.sparse_run_schedule(p.loss, p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy(), p.y.numpy(),
                                              p.D, np.zeros(p.D), p.lam, eta, oracle.INV_SQRT, 6)
    got = a.history().cpu().numpy()
    assert max(rel(x, y) for x, y in zip(got, lh)) <= REL_TOL
    assert np.max(np.abs(a.w.cpu().numpy() - w)) <= REL_TOL * np.max(np.abs(w))
    const = oracle.sparse_run(p.loss, p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy(), p.y.numpy(), p.D,
                              np.zeros(p.D), p.lam, eta, 6)[2]
    assert np.max(np.abs(a.w.cpu().numpy() - const)) > 100 * REL_TOL * np.max(np.abs(w))     # not the constant step
