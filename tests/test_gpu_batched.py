"""GPU tests of glm_step_batched: many concurrent jobs driven by an allocation vector."""
import numpy as np
import pytest
import torch

import oracle
from paper_1802_04819_amd import glm, synth
from _parity import REL_TOL, make_job, rel

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _mixed_problems():
    shapes = [(synth.LOGISTIC, 5000, 64), (synth.HINGE, 12000, 128), (synth.SQUARED, 3000, 256),
              (synth.LOGISTIC, 700, 512), (synth.HINGE, 9000, 100), (synth.SQUARED, 1, 8),
              (synth.LOGISTIC, 20000, 1024), (synth.SQUARED, 4097, 20), (synth.HINGE, 2500, 2048)]
    eta = {synth.LOGISTIC: 0.3, synth.HINGE: 0.02, synth.SQUARED: 0.05}
    return [synth.make_glm(l, n, d, seed=100 + i, lam=10.0 ** (-2 - i % 3), eta=eta[l], K=8)
            for i, (l, n, d) in enumerate(shapes)]


def test_batched_equals_looped_single_jobs_bitwise():
    _say("[case] batched == looped glm_step, bit for bit, mixed shapes and losses")
    probs = _mixed_problems()
    alloc = np.array([3, 1, 8, 0, 5, 2, 4, 8, 1], dtype=np.int32)
    batched = [make_job(p, hist_cap=16) for p in probs]
    looped = [make_job(p, hist_cap=16) for p in probs]
    ws = glm.alloc_workspace(batched)
    glm.glm_step_batched(batched, alloc, ws)
    for j, a in zip(looped, alloc):
        ws1 = glm.alloc_workspace([j])
        glm.glm_step(j, int(a), ws1)
    torch.cuda.synchronize()
    for b, l, a in zip(batched, looped, alloc):
        assert b.hist_len == l.hist_len == int(a)
        assert torch.equal(b.history(), l.history())
        assert torch.equal(b.w, l.w) and torch.equal(b.grad, l.grad)
    # a second epoch with another allocation continues every history
    alloc2 = np.array([1, 2, 0, 7, 1, 1, 0, 3, 6], dtype=np.int32)
    glm.glm_step_batched(batched, alloc2, ws)
    for j, a in zip(looped, alloc2):
        glm.glm_step(j, int(a), glm.alloc_workspace([j]))
    torch.cuda.synchronize()
    for b, l, a, a2 in zip(batched, looped, alloc, alloc2):
        assert b.hist_len == int(a) + int(a2)
        assert torch.equal(b.history(), l.history()) and torch.equal(b.w, l.w)


def test_batched_histories_match_oracle_trajectories():
    _say("[case] batched histories vs oracle trajectories")
    probs = _mixed_problems()
    alloc = np.array([4, 4, 6, 3, 5, 2, 3, 8, 2], dtype=np.int32)
    jobs = [make_job(p, hist_cap=8) for p in probs]
    ws = glm.alloc_workspace(jobs)
    glm.glm_step_batched(jobs, alloc, ws)
    torch.cuda.synchronize()
    for p, j, a in zip(probs, jobs, alloc):
        lh, gh, wK, g_last = oracle.run(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(p.D), p.lam, p.eta, int(a))
        got = j.history().cpu().numpy()
        for k in range(int(a)):
            assert rel(got[k], lh[k]) <= REL_TOL, (p.name, k, got[k], lh[k])
        gn = np.linalg.norm(j.grad.cpu().numpy().astype(np.float64))
        assert rel(gn, gh[-1]) <= REL_TOL, (p.name, gn, gh[-1])
        assert np.max(np.abs(j.w.cpu().numpy() - wK)) <= REL_TOL * max(np.max(np.abs(wK)), 1e-30)


def test_all_idle_epoch_is_a_no_op():
    _say("[case] allocation of all zeros")
    probs = _mixed_problems()[:3]
    jobs = [make_job(p, hist_cap=4) for p in probs]
    ws = glm.alloc_workspace(jobs)
    glm.glm_step_batched(jobs, np.zeros(3, np.int32), ws)
    torch.cuda.synchronize()
    assert all(j.hist_len == 0 and j.w.abs().sum().item() == 0 for j in jobs)


def test_batched_reruns_are_bit_identical_with_many_jobs():
    _say("[case] 40 jobs, rerun determinism")
    specs = synth.config3_specs(J=40, scale=0.02)
    probs = [synth.config3_job(s, device="cuda") for s in specs]
    alloc = synth.config3_alloc(0, J=40)
    outs = []
    for _ in range(2):
        jobs = [glm.Job(p.X, p.y, p.w0.clone(), p.loss, p.lam, p.eta, 8) for p in probs]
        ws = glm.alloc_workspace(jobs)
        glm.glm_step_batched(jobs, alloc, ws)
        torch.cuda.synchronize()
        outs.append([(j.history().clone(), j.w.clone()) for j in jobs])
    for (h0, w0), (h1, w1) in zip(*outs):
        assert torch.equal(h0, h1) and torch.equal(w0, w1)
    # spot-check three jobs of the mix against the oracle, per step at the final iterate
    for idx in (0, 17, 39):
        p = probs[idx]
        job = glm.Job(p.X, p.y, outs[0][idx][1].clone(), p.loss, p.lam, 0.0, 1)
        glm.glm_step(job, 1, glm.alloc_workspace([job]))
        torch.cuda.synchronize()
        L, g = oracle.loss_grad(p.loss, p.X.cpu().numpy(), p.y.cpu().numpy(),
                                outs[0][idx][1].cpu().numpy().astype(np.float64), p.lam, chunks=8)
        assert rel(job.loss_hist[0].item(), L) <= REL_TOL
        assert rel(np.linalg.norm(job.grad.cpu().numpy().astype(np.float64)), np.linalg.norm(g)) <= REL_TOL
