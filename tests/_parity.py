"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

import oracle
from paper_1802_04819_amd import glm

# Stated tolerance of the method's target: relative error of the loss and of the gradient
# L2 norm, per iteration, against the fp64 oracle.
REL_TOL = 1e-4


def rel(a, b):
    return abs(a - b) / max(abs(b), 1e-300)


def make_job(p, device="cuda", hist_cap=None, step=None, w=None):
    X = p.X.to(device); y = p.y.to(device)
    w0 = (p.w0 if w is None else w).to(device).clone()
    return glm.Job(X, y, w0, p.loss, p.lam, p.eta if step is None else step,
                   p.K if hist_cap is None else hist_cap)


def check_step_against_oracle(loss, X_np, y_np, w_in, lam, L_gpu, g_gpu, chunks=0, tag=""):
    """Per-step parity: the oracle is evaluated at the fp32 iterate the GPU step started from."""
    L, g = oracle.loss_grad(loss, X_np, y_np, np.asarray(w_in, dtype=np.float64), lam, chunks=chunks)
    gn = float(np.linalg.norm(g))
    g_gpu = np.asarray(g_gpu, dtype=np.float64)
    assert rel(float(L_gpu), L) <= REL_TOL, (tag, "loss", float(L_gpu), L)
    assert rel(float(np.linalg.norm(g_gpu)), gn) <= REL_TOL, (tag, "gnorm", np.linalg.norm(g_gpu), gn)
    # element by element: every gradient entry within REL_TOL of the gradient's scale
    err = np.max(np.abs(g_gpu - g))
    assert err <= REL_TOL * max(np.max(np.abs(g)), 1e-300), (tag, "grad entries", err, np.max(np.abs(g)))
    return L, g


def run_and_check_every_step(p, iters, device="cuda", chunks=0):
    """Runs `iters` single iterations through glm_step, checking each against the oracle at
    the same starting iterate, including the update w <- w - eta g."""
    job = make_job(p, device, hist_cap=iters)
    ws = glm.alloc_workspace([job])
    Xn, yn = p.X.numpy(), p.y.numpy()
    for k in range(iters):
        w_in = job.w.cpu().numpy().copy()
        glm.glm_step(job, 1, ws)
        torch.cuda.synchronize()
        L_gpu = job.loss_hist[k].item()
        g_gpu = job.grad.cpu().numpy()
        _, g = check_step_against_oracle(p.loss, Xn, yn, w_in, p.lam, L_gpu, g_gpu, chunks, f"{p.name} k={k}")
        w_ref = w_in.astype(np.float64) - p.eta * g
        w_out = job.w.cpu().numpy().astype(np.float64)
        scale = max(np.max(np.abs(w_ref)), p.eta * np.max(np.abs(g)), 1e-30)
        assert np.max(np.abs(w_out - w_ref)) <= REL_TOL * scale, (p.name, k, "update")
    assert job.hist_len == iters
    return job
