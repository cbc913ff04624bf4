"""fp64 CPU oracle for L-BFGS on the GLM objective (TEST INFRASTRUCTURE: imported only by tests,
the smoke check and the benchmark's CPU leg; shares nothing with the GPU library).

The paper names L-BFGS among the iterative solvers of the jobs it schedules (Sec. 1, "ML training
is typically iterative with diminishing returns") and as an example of its second convergence
class (Sec. 2, "Predicting Quality Improvement": linear or superlinear convergence).  It gives no
detail of the method, so this follows the published algorithm (limited-memory BFGS: the two-loop
recursion over the last m curvature pairs with the initial scaling s.y / y.y, and a backtracking
line search on the sufficient-decrease condition), with these readings, shared with the library:
  - the objective and its gradient are those of the GLM oracle (`oracle.loss_grad`);
  - first iteration: direction -g, first trial step min(1, 1/|g|); later iterations start at 1;
  - a trial step alpha is accepted when it satisfies the sufficient-decrease condition
    f(w + alpha p) <= f(w) + c1 alpha g.p  with c1 = 1e-4; otherwise alpha is halved, at most 30
    times, after which the step is taken anyway;
  - a curvature pair with s.y <= 1e-10 y.y is not stored;
  - the history entry of iteration k is the loss at the iterate that enters it.
Against values printed by the paper: "parity unpinned".  The CPU tests pin the two-loop recursion
to the dense BFGS update formula, and the whole method to closed-form optima and SciPy.
"""
from __future__ import annotations

import numpy as np

import oracle

C1 = 1e-4
MAX_HALVINGS = 30
CURV_EPS = 1e-10


def two_loop(g, S, Y):
    """-H g for the limited-memory inverse Hessian built from pairs (S[i], Y[i]), oldest first."""
    q = np.array(g, dtype=np.float64, copy=True)
    n = len(S)
    alpha = np.zeros(n)
    rho = [1.0 / float(np.dot(S[i], Y[i])) for i in range(n)]
    for i in range(n - 1, -1, -1):
        alpha[i] = rho[i] * float(np.dot(S[i], q))
        q -= alpha[i] * Y[i]
    if n:
        q *= float(np.dot(S[-1], Y[-1])) / float(np.dot(Y[-1], Y[-1]))
    for i in range(n):
        beta = rho[i] * float(np.dot(Y[i], q))
        q += (alpha[i] - beta) * S[i]
    return -q


def minimize(f_and_g, w0, iters, memory=10):
    """`iters` L-BFGS iterations on an arbitrary objective.  Returns (loss_hist, w, info) where
    info holds the accepted step sizes, the number of evaluations and the gradient norms."""
    w = np.array(w0, dtype=np.float64, copy=True)
    f, g = f_and_g(w)
    S, Y = [], []
    hist, steps, gn = np.empty(iters), [], []
    evals = 1
    for k in range(iters):
        hist[k] = f
        gn.append(float(np.linalg.norm(g)))
        p = two_loop(g, S, Y)
        gtp = float(np.dot(g, p))
        alpha = 1.0 if S else min(1.0, 1.0 / max(gn[-1], 1e-300))
        for h in range(MAX_HALVINGS + 1):
            wt = w + alpha * p
            ft, gt = f_and_g(wt)
            evals += 1
            if ft <= f + C1 * alpha * gtp or h == MAX_HALVINGS:
                break
            alpha *= 0.5
        s, y = wt - w, gt - g
        sy, yy = float(np.dot(s, y)), float(np.dot(y, y))
        if sy > CURV_EPS * yy:
            S.append(s); Y.append(y)
            if len(S) > memory:
                S.pop(0); Y.pop(0)
        w, f, g = wt, ft, gt
        steps.append(alpha)
    return hist, w, {"steps": steps, "evals": evals, "gnorm": gn, "f_end": f, "g_end": g}


def run(loss, X, y, w0, lam, iters, memory=10, chunks=0):
    """L-BFGS on the GLM objective of `oracle.loss_grad`."""
    return minimize(lambda w: oracle.loss_grad(loss, X, y, w, lam, chunks), w0, iters, memory)
