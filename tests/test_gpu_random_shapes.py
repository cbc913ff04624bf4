"""Seeded random shapes inside the documented limits, every entry point against its oracle.
The hand-picked shapes of the other GPU tests cover the known tile and tail cases; these draws
are there for the combinations nobody thought of."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
from oracle import lbfgs_oracle as lb
from paper_1802_04819_amd import glm, synth
from _parity import REL_TOL, rel, run_and_check_every_step
import test_gpu_kmeans as tk
import test_gpu_sparse as ts

pytestmark = pytest.mark.gpu

DIMS = [4, 8, 12, 20, 36, 60, 64, 68, 100, 128, 132, 200, 256, 260, 384, 512, 516, 700, 1024, 1028, 2048, 3000, 4096]


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("i", range(12))
def test_dense_step(i):
    rng = np.random.default_rng(100 + i)
    loss = int(rng.integers(0, 3)); N = int(rng.integers(1, 30000)); D = int(rng.choice(DIMS))
    N = min(N, max(1, int(2e7 // D)))
    eta = {0: 0.3, 1: 0.02, 2: 0.05}[loss] / max(1.0, D / 256)
    _say(f"[case] random dense loss={loss} N={N} D={D}")
    p = synth.make_glm(loss, N, D, seed=100 + i, lam=float(10 ** rng.uniform(-6, -2)), eta=eta, K=2)
    run_and_check_every_step(p, 2)


@pytest.mark.parametrize("i", range(3))
def test_batched_epoch(i):
    rng = np.random.default_rng(200 + i)
    J = int(rng.integers(2, 10))
    probs = []
    for j in range(J):
        D = int(rng.choice(DIMS[:19])); N = min(int(rng.integers(1, 8000)), max(1, int(4e6 // D)))
        probs.append(synth.make_glm(int(rng.integers(0, 3)), N, D, seed=2000 + 100 * i + j, lam=1e-4, eta=0.01, K=1))
    alloc = rng.integers(0, 4, size=J).astype(np.int32)
    _say(f"[case] random batched epoch J={J} alloc={alloc.tolist()}")
    jobs = [glm.Job(p.X.cuda(), p.y.cuda(), p.w0.cuda().clone(), p.loss, p.lam, p.eta, 4) for p in probs]
    glm.glm_step_batched(jobs, alloc, glm.alloc_workspace(jobs))
    torch.cuda.synchronize()
    for p, j, a in zip(probs, jobs, alloc):
        assert j.hist_len == a
        if a == 0:
            assert not j.w.any()
            continue
        lh, gh, wK, gl = oracle.run(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(p.D), p.lam, p.eta, int(a))
        got = j.history().cpu().numpy()
        for k in range(int(a)):
            assert rel(got[k], lh[k]) <= REL_TOL, (p.name, k, got[k], lh[k])
        assert rel(np.linalg.norm(j.grad.cpu().numpy().astype(np.float64)), gh[-1]) <= REL_TOL


@pytest.mark.parametrize("i", range(3))
def test_sweep(i):
    rng = np.random.default_rng(300 + i)
    D = int(rng.choice([32, 64, 96, 256, 1024, 2048])); N = min(int(rng.integers(1, 6000)), max(1, int(4e6 // D)))
    M = int(rng.integers(1, 65)); loss = int(rng.integers(0, 3))
    _say(f"[case] random sweep N={N} D={D} M={M} loss={loss}")
    p = synth.make_glm(loss, N, D, seed=300 + i, lam=1e-4, eta=0.01, K=1)
    lams = (10 ** rng.uniform(-6, -2, size=M)).astype(np.float32)
    etas = (10 ** rng.uniform(-3, -1.5, size=M)).astype(np.float32)
    X, y = p.X.cuda(), p.y.cuda()
    W = torch.zeros(M, D, device="cuda"); G = torch.zeros(M, D, device="cuda"); hist = torch.zeros(3, M, device="cuda")
    glm.glm_sweep(X, y, loss, W, G, lams, etas, 3, hist, glm.alloc_sweep_workspace(X, M))
    torch.cuda.synchronize()
    lh, gh, WK, GL = oracle.run_sweep(loss, p.X.numpy(), p.y.numpy(), np.zeros((M, D)), lams, etas, 3)
    assert np.max(np.abs(hist.cpu().numpy() - lh) / np.abs(lh)) <= REL_TOL
    gn = np.linalg.norm(G.cpu().numpy().astype(np.float64), axis=1)
    assert np.max(np.abs(gn - gh[-1]) / np.maximum(gh[-1], 1e-300)) <= REL_TOL


@pytest.mark.parametrize("i", range(8))
def test_sparse_step(i):
    rng = np.random.default_rng(400 + i)
    N = int(rng.integers(1, 20000)); D = int(rng.integers(1, 20000)); dens = float(10 ** rng.uniform(-4.5, -1))
    dens = min(dens, 3e6 / (N * D))
    loss = int(rng.integers(0, 3))
    A = sp.random(N, D, dens, format="csr", random_state=int(rng.integers(1 << 30)), dtype=np.float32)
    _say(f"[case] random sparse N={N} D={D} nnz={A.nnz} loss={loss}")
    y = ts._labels(loss, N, rng)
    eta = {0: 0.5, 1: 0.05, 2: 0.02}[loss]
    job, csr = ts._job_from_scipy(A, y, loss, 1e-3, eta, 2)
    ts._check_steps(job, csr, y, D, loss, 1e-3, eta, 2, "random")


@pytest.mark.parametrize("i", range(10))
def test_kmeans_step(i):
    rng = np.random.default_rng(500 + i)
    D = int(rng.choice([4, 8, 20, 32, 60, 64, 100, 128, 132, 256, 300, 512, 1024]))
    N = min(int(rng.integers(1, 40000)), max(1, int(6e6 // D)))
    K = int(min(N, rng.choice([1, 2, 3, 7, 31, 32, 33, 64, 100, 255, 256, 257, 500, 1024])))
    _say(f"[case] random kmeans N={N} D={D} K={K}")
    p = synth.make_kmeans(N, D, K, seed=500 + i, blobs=int(max(2, min(K, 30))), offset=float(rng.choice([0.0, 0.0, 5.0])))
    tk.run_checked(p, 3, "random")


@pytest.mark.parametrize("i", range(3))
def test_lbfgs_run(i):
    rng = np.random.default_rng(600 + i)
    loss = int(rng.choice([0, 2])); D = int(rng.choice(DIMS[:19])); mem = int(rng.integers(0, 12))
    N = min(int(rng.integers(200, 8000)), max(200, int(4e6 // D)))
    _say(f"[case] random L-BFGS loss={loss} N={N} D={D} memory={mem}")
    p = synth.make_glm(loss, N, D, seed=600 + i, lam=1e-3, eta=0.0, K=1)
    job = glm.Job(p.X.cuda(), p.y.cuda(), p.w0.cuda().clone(), p.loss, p.lam, 0.0, 8)
    glm.glm_lbfgs(job, glm.glm_lbfgs_state_t(), 8, mem, glm.alloc_lbfgs_workspace(job, mem))
    torch.cuda.synchronize()
    hist, w, info = lb.run(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(D), p.lam, 8, mem)
    got = job.history().cpu().numpy()
    moving = np.abs(hist - info["f_end"]) > 1e-4 * abs(info["f_end"])
    for k in range(8):
        if moving[: k + 1].all():
            assert rel(got[k], hist[k]) <= REL_TOL, (k, got[k], hist[k])


@pytest.mark.parametrize("i", range(3))
def test_sparse_step_with_row_panels(i):
    rng = np.random.default_rng(700 + i)
    N = int(rng.integers(786_433, 3_500_000)); D = int(rng.integers(1, 5000)); nnz = int(rng.integers(1, 3_000_000))
    loss = int(rng.integers(0, 3))
    rows = rng.integers(0, N, size=nnz); cols = (rng.random(nnz) ** float(rng.uniform(1, 4)) * D).astype(np.int64)
    if i == 0:
        rows[: nnz // 2] = rng.integers(N // 3, N // 3 + 1000, size=nnz // 2)       # one crowded panel
    A = sp.csr_matrix(((rng.standard_normal(nnz) / 3).astype(np.float32), (rows, cols)), shape=(N, D))
    _say(f"[case] random sparse with row panels N={N} D={D} nnz={A.nnz} loss={loss}")
    y = ts._labels(loss, N, rng)
    eta = {0: 0.5, 1: 0.05, 2: 0.02}[loss]
    job, csr = ts._job_from_scipy(A, y, loss, 1e-4, eta, 2)
    ts._check_steps(job, csr, y, D, loss, 1e-4, eta, 2, "random panels")
    assert job.c.prepared == 1
