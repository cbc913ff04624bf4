"""GPU tests of glm_sweep (many models sharing one X, matrix-core kernels) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_1802_04819_amd import glm, synth
from _parity import REL_TOL, rel

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _run_sweep(p, lams, etas, K, W0=None):
    X, y = p.X.cuda(), p.y.cuda()
    M = len(lams)
    W = torch.zeros(M, p.D, device="cuda") if W0 is None else W0.cuda().clone()
    G = torch.zeros(M, p.D, device="cuda")
    hist = torch.zeros(max(K, 1), M, device="cuda")
    ws = glm.alloc_sweep_workspace(X, M)
    glm.glm_sweep(X, y, p.loss, W, G, lams, etas, K, hist, ws)
    torch.cuda.synchronize()
    return W, G, hist


@pytest.mark.parametrize("loss,N,D,M", [
    (synth.LOGISTIC, 1000, 64, 5), (synth.LOGISTIC, 4097, 256, 64), (synth.HINGE, 3000, 96, 17),
    (synth.SQUARED, 2500, 320, 33), (synth.LOGISTIC, 129, 32, 1), (synth.SQUARED, 31, 1024, 64),
    (synth.HINGE, 20000, 512, 64),
    # more than one group of 64 models, a last group of at most 32, row lengths that are not multiples of 32
    (synth.LOGISTIC, 3000, 128, 128), (synth.SQUARED, 2000, 96, 100), (synth.LOGISTIC, 5000, 256, 16),
    (synth.HINGE, 1500, 48, 32), (synth.LOGISTIC, 2222, 100, 70), (synth.SQUARED, 900, 4, 3), (synth.LOGISTIC, 700, 1028, 9),
    # groups of at most 16 models on row lengths that are multiples of 16 up to 1024 (one-pass kernel): a last
    # tile of fewer than 16 rows, fewer rows than a tile, several tiles per block, every row-length class,
    # a last group of 6 after a group of 64
    (synth.HINGE, 2007, 1024, 16), (synth.SQUARED, 15, 16, 2), (synth.LOGISTIC, 9601, 512, 9),
    (synth.HINGE, 40000, 768, 12), (synth.LOGISTIC, 3000, 48, 16), (synth.LOGISTIC, 2500, 128, 70),
    (synth.SQUARED, 5000, 272, 7), (synth.LOGISTIC, 16, 1024, 1),
])
def test_sweep_matches_oracle_trajectories(loss, N, D, M):
    _say(f"[case] sweep parity loss={loss} N={N} D={D} M={M}")
    eta_hi = {synth.LOGISTIC: 0.5, synth.HINGE: 0.02, synth.SQUARED: 0.02}[loss]
    p = synth.make_glm(loss, N, D, seed=21 + N, lam=0.0, eta=0.0, K=5)
    rng = np.random.default_rng(3)
    lams = (10.0 ** rng.uniform(-5, -1, M)).astype(np.float32)
    etas = (eta_hi * 10.0 ** rng.uniform(-2, 0, M)).astype(np.float32)
    K = 5
    W, G, hist = _run_sweep(p, lams, etas, K)
    lh, gh, WK, GL = oracle.run_sweep(p.loss, p.X.numpy(), p.y.numpy(), np.zeros((M, D)), lams, etas, K)
    got = hist.cpu().numpy()
    for k in range(K):
        for m in range(M):
            assert rel(got[k, m], lh[k, m]) <= REL_TOL, (k, m, got[k, m], lh[k, m])
    Gn = G.cpu().numpy().astype(np.float64)
    for m in range(M):
        assert rel(np.linalg.norm(Gn[m]), gh[-1, m]) <= REL_TOL, (m,)
        assert np.max(np.abs(Gn[m] - GL[m])) <= REL_TOL * np.max(np.abs(GL[m]))
        assert np.max(np.abs(W.cpu().numpy()[m] - WK[m])) <= REL_TOL * max(np.max(np.abs(WK[m])), 1e-30)


def test_sweep_column_equals_single_job_within_tolerance():
    _say("[case] sweep model m vs glm_step with (lambda_m, step_m)")
    p = synth.make_glm(synth.LOGISTIC, 6000, 128, seed=5, lam=0.0, eta=0.0, K=6)
    lams, etas = synth.sweep_grid(4, 4)
    W, G, hist = _run_sweep(p, lams, etas, 6)
    for m in (0, 7, 15):
        job = glm.Job(p.X.cuda(), p.y.cuda(), torch.zeros(128, device="cuda"), p.loss,
                      float(lams[m]), float(etas[m]), 6)
        glm.glm_step(job, 6, glm.alloc_workspace([job]))
        torch.cuda.synchronize()
        a, b = hist[:, m].cpu().numpy(), job.history().cpu().numpy()
        assert np.max(np.abs(a - b) / np.abs(b)) <= 1e-5
        assert torch.allclose(W[m], job.w, rtol=1e-4, atol=1e-6)


def test_sweep_per_step_from_nonzero_start():
    _say("[case] sweep single step from a random W, per-step oracle check")
    p = synth.make_glm(synth.LOGISTIC, 3333, 160, seed=8, lam=0.0, eta=0.0, K=1)
    M = 12
    g = torch.Generator().manual_seed(2)
    W0 = torch.randn(M, 160, generator=g) * 0.3
    lams = np.full(M, 1e-2, np.float32); etas = np.zeros(M, np.float32)      # step 0: evaluate only
    W, G, hist = _run_sweep(p, lams, etas, 1, W0=W0)
    assert torch.equal(W.cpu(), W0)
    for m in range(M):
        L, gr = oracle.loss_grad(p.loss, p.X.numpy(), p.y.numpy(), W0[m].numpy().astype(np.float64), 1e-2)
        assert rel(hist[0, m].item(), L) <= REL_TOL
        gg = G[m].cpu().numpy().astype(np.float64)
        assert rel(np.linalg.norm(gg), np.linalg.norm(gr)) <= REL_TOL
        assert np.max(np.abs(gg - gr)) <= REL_TOL * np.max(np.abs(gr))


@pytest.mark.parametrize("M", [64, 16])
def test_sweep_reruns_are_bit_identical(M):
    _say(f"[case] sweep rerun determinism, {M} models")
    p = synth.make_glm(synth.LOGISTIC, 50000, 256, seed=4, lam=0.0, eta=0.0, K=4, device="cuda")
    lams, etas = synth.sweep_grid()
    lams, etas = lams[:M], etas[:M]
    outs = [_run_sweep(p, lams, etas, 4) for _ in range(3)]
    for o in outs[1:]:
        assert all(torch.equal(a, b) for a, b in zip(outs[0], o))


@pytest.mark.parametrize("M_full,M_less", [(64, 63), (32, 31), (128, 127), (16, 15), (80, 65)])
def test_sweep_full_and_partial_tiles_give_the_same_bits(M_full, M_less):
    """A tile full of models runs the forward kernel without masks, a partial tile the one with them;
    both add the same numbers in the same order, so a model's trajectory does not depend on how many
    models share its tile."""
    _say(f"[case] sweep, {M_full} models against the first {M_less} of them: same bits per model")
    p = synth.make_glm(synth.LOGISTIC, 3001, 256, seed=77, lam=0.0, eta=0.0, K=4)
    rng = np.random.default_rng(8)
    lams = (10.0 ** rng.uniform(-5, -1, M_full)).astype(np.float32)
    etas = (0.5 * 10.0 ** rng.uniform(-2, 0, M_full)).astype(np.float32)
    Wf, Gf, hf = _run_sweep(p, lams, etas, 4)
    Wl, Gl, hl = _run_sweep(p, lams[:M_less], etas[:M_less], 4)
    assert torch.equal(Wf[:M_less], Wl) and torch.equal(Gf[:M_less], Gl) and torch.equal(hf[:, :M_less], hl)


def test_sweep_argument_errors():
    _say("[case] sweep error codes")
    p = synth.make_glm(synth.LOGISTIC, 100, 64, seed=1, lam=0.0, eta=0.0, K=1)
    X, y = p.X.cuda(), p.y.cuda()
    W = torch.zeros(3, 64, device="cuda"); G = torch.zeros_like(W); h = torch.zeros(2, 3, device="cuda")
    ws = glm.alloc_sweep_workspace(X, 3)
    ok = np.array([1e-3] * 3, np.float32)
    with pytest.raises(glm.GlmError) as e:
        glm.glm_sweep(X, y, 0, W, G, np.array([1e-3, -1.0, 0.0], np.float32), ok, 1, h, ws)
    assert e.value.status == glm.GLM_EINVAL
    with pytest.raises(glm.GlmError) as e:
        glm.glm_sweep(X, y, 0, W, G, ok, ok, 1, h, ws[:1024])
    assert e.value.status == glm.GLM_ENOSPC
    with pytest.raises(glm.GlmError) as e:
        glm.glm_sweep(X, y, 5, W, G, ok, ok, 1, h, ws)
    assert e.value.status == glm.GLM_EINVAL
    with pytest.raises(glm.GlmError):
        glm.sweep_workspace_bytes(10, 46, 3)          # D must be a multiple of 4
    with pytest.raises(glm.GlmError):
        glm.sweep_workspace_bytes(10, 64, 70000)      # more models than a call takes
    assert glm.sweep_workspace_bytes(10, 48, 3) > 0 and glm.sweep_workspace_bytes(10, 64, 65) > 0
    torch.cuda.synchronize()
    assert W.abs().sum().item() == 0
