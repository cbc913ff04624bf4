"""GPU test of glm_step_noalloc (the entry point for callers that cannot allocate): through the
C ABI, against glm_step on a caller-owned workspace, bit for bit (both run the same kernels in
the same order), and against the fp64 oracle to the stated tolerance.  Two calls in a row on the
same device-resident scratch, the second with a smaller input, then a third with the large one
again: whatever a call leaves in the scratch must not reach the next call's results."""
import numpy as np
import pytest
import torch

import oracle
from paper_1802_04819_amd import glm, synth
from _parity import REL_TOL, make_job, rel

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _run_pair(p, iters):
    """The same job through glm_step (own workspace) and through glm_step_noalloc."""
    a = make_job(p, hist_cap=iters)
    b = make_job(p, hist_cap=iters)
    ws = glm.alloc_workspace([a])
    glm.glm_step(a, iters, ws)
    glm.glm_step_noalloc(b, iters)
    torch.cuda.synchronize()
    assert a.hist_len == iters and b.hist_len == iters
    for name in ("loss_hist", "w", "grad"):
        ta, tb = getattr(a, name).cpu().numpy(), getattr(b, name).cpu().numpy()
        assert ta.tobytes() == tb.tobytes(), (p.name, name)
    return b


def _check_oracle(p, job, iters):
    lh, gh, wK, _ = oracle.run(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(p.D), p.lam, p.eta, iters)
    got = job.history().cpu().numpy()
    for k in range(iters):
        assert rel(got[k], lh[k]) <= REL_TOL, (p.name, k, got[k], lh[k])
    gn = float(np.linalg.norm(job.grad.cpu().numpy().astype(np.float64)))
    assert rel(gn, gh[-1]) <= REL_TOL, (p.name, gn, gh[-1])
    assert np.max(np.abs(job.w.cpu().numpy() - wK)) <= REL_TOL * max(np.max(np.abs(wK)), 1e-30)


def test_two_calls_in_a_row_second_smaller_then_large_again():
    _say("[case] glm_step_noalloc: large, then smaller, then large again, vs glm_step and the oracle")
    assert glm.glm_step_noalloc_scratch_bytes() >= (8 << 20)
    big = synth.make_glm(synth.LOGISTIC, 30011, 1024, seed=5, lam=1e-4, eta=0.3, K=3)
    small = synth.make_glm(synth.SQUARED, 777, 36, seed=6, lam=1e-3, eta=0.1, K=5)
    mid = synth.make_glm(synth.HINGE, 5003, 260, seed=7, lam=1e-3, eta=0.02, K=4)
    jb = _run_pair(big, big.K)
    _check_oracle(big, jb, big.K)
    js = _run_pair(small, small.K)          # the scratch still holds the large job's partial sums
    _check_oracle(small, js, small.K)
    jm = _run_pair(mid, mid.K)
    _check_oracle(mid, jm, mid.K)
    jb2 = _run_pair(big, big.K)
    assert jb2.loss_hist.cpu().numpy().tobytes() == jb.loss_hist.cpu().numpy().tobytes()
    assert jb2.w.cpu().numpy().tobytes() == jb.w.cpu().numpy().tobytes()


def test_split_calls_and_zero_iterations():
    _say("[case] glm_step_noalloc: 2 + 0 + 3 iterations equal 5 at once")
    p = synth.make_glm(synth.LOGISTIC, 4099, 128, seed=8, lam=1e-4, eta=0.5, K=5)
    a = make_job(p, hist_cap=5)
    b = make_job(p, hist_cap=5)
    glm.glm_step_noalloc(a, 5)
    glm.glm_step_noalloc(b, 2)
    glm.glm_step_noalloc(b, 0)
    glm.glm_step_noalloc(b, 3)
    torch.cuda.synchronize()
    assert b.hist_len == 5
    assert a.loss_hist.cpu().numpy().tobytes() == b.loss_hist.cpu().numpy().tobytes()
    assert a.w.cpu().numpy().tobytes() == b.w.cpu().numpy().tobytes()


def test_largest_shape_fits_and_errors_leave_everything_untouched():
    _say("[case] glm_step_noalloc: D = 4096 with the most row blocks fits; error codes")
    p = synth.make_glm(synth.SQUARED, 2600, 4096, seed=9, lam=1e-3, eta=0.05, K=2)
    j = _run_pair(p, 2)
    _check_oracle(p, j, 2)
    before = (j.w.clone(), j.loss_hist.clone(), j.hist_len)
    with pytest.raises(glm.GlmError) as e:          # history full
        glm.glm_step_noalloc(j, 1)
    assert e.value.status == glm.GLM_ENOSPC
    with pytest.raises(glm.GlmError) as e:
        glm.glm_step_noalloc(j, -1)
    assert e.value.status == glm.GLM_EINVAL
    torch.cuda.synchronize()
    assert torch.equal(before[0], j.w) and torch.equal(before[1], j.loss_hist) and before[2] == j.hist_len
