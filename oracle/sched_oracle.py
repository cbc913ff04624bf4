"""fp64 CPU oracle for the scheduler-side steps that consume the loss histories
(TEST INFRASTRUCTURE: imported only by tests, the smoke check and the benchmark's CPU leg).

Follows Sec. 2 of the paper:
  * "Normalizing Quality Metrics": the change in loss between iterations is normalised by the
    largest change seen so far.
  * "Predicting Quality Improvement": a curve f(k) = 1/(a k^2 + b k + c) + d (sublinear
    convergence, class I) or f(k) = mu^(k-b) + c (linear/superlinear, class II) is fitted to the
    exponentially weighted loss history and evaluated at future iterations.
  * "Scheduling Based on Quality Improvements": start from one unit per job, repeatedly give
    one more unit to the job whose predicted loss reduction for that unit is largest, until the
    capacity is used up.

The paper states neither the weight decay, nor how the curve is fitted, nor what "normalised
loss reduction" is exactly; the readings taken here (and in the library) are:
  - weight of history point i of n is gamma^(n-1-i); only the last `window` points are used;
  - the fit is a variable projection: for a candidate offset (d, resp. c) the remaining
    parameters enter linearly after the transform u = 1/(L-d) (resp. v = log(L-c)) and are found
    by weighted linear least squares with the first-order weights w (L-d)^4 (resp. w (L-c)^2);
    the offset is chosen on a two-level logarithmic grid of 64 candidates each by the weighted
    squared error of the untransformed curve; ties go to the lower candidate index;
  - iteration numbers are scaled to t = i/(m-1) over the window of m points;
  - the predicted reduction of the h-th further iteration is (f(m-2+h) - f(m-1+h)) divided by
    the largest single-iteration change seen so far in the whole history.
The paper prints no numeric example of any of this: "parity unpinned" against paper values;
the CPU tests pin the routines with exact curves, hand examples and brute force.
"""
from __future__ import annotations

import numpy as np

CLASS_SUBLINEAR, CLASS_LINEAR = 1, 2
N_CAND = 64
EXP_LO, EXP_HI = -4.0, 2.0          # first-level offsets: gap = span * 10**e, e in [EXP_LO, EXP_HI]


def normalized_changes(L):
    """nu_k = (L_{k-1} - L_k) / max_{i<=k} |L_{i-1} - L_i| for k = 1..n-1, and the final normaliser."""
    L = np.asarray(L, dtype=np.float64)
    d = L[:-1] - L[1:]
    run = np.maximum.accumulate(np.abs(d))
    nu = np.where(run > 0, d / np.where(run > 0, run, 1.0), 0.0)
    return nu, (float(run[-1]) if len(run) else 0.0)


def _fit_for_offset(cls, t, L, w, off):
    """Weighted linear least squares in the transformed space for one offset candidate.
    Returns (params, sse) with sse the weighted squared error of the untransformed curve,
    or (None, inf) when the candidate is not admissible."""
    g = L - off
    if np.any(g <= 0):
        return None, np.inf
    if cls == CLASS_SUBLINEAR:
        u = 1.0 / g
        W = w * g ** 4
        A = np.stack([t * t, t, np.ones_like(t)], axis=1)
    else:
        u = np.log(g)
        W = w * g ** 2
        A = np.stack([t, np.ones_like(t)], axis=1)
    AtW = A.T * W
    N = AtW @ A
    rhs = AtW @ u
    try:
        p = np.linalg.solve(N, rhs)
    except np.linalg.LinAlgError:
        return None, np.inf
    lin = A @ p
    if cls == CLASS_SUBLINEAR:
        if np.any(lin <= 0) or not np.all(np.isfinite(lin)):
            return None, np.inf
        f = 1.0 / lin + off
    else:
        if not np.all(np.isfinite(lin)):
            return None, np.inf
        f = np.exp(lin) + off
    sse = float(np.sum(w * (f - L) ** 2))
    if not np.isfinite(sse):
        return None, np.inf
    return p, sse


def fit_curve(L, cls=CLASS_SUBLINEAR, gamma=0.9, window=128):
    """Fit the convergence curve of class `cls` to the last `window` losses.

    Returns a dict with `ok`, `off` (d or c), `p` (linear parameters in scaled time), `m`
    (points used), `sse`.  ok is False when there are fewer than 4 points, the history is
    flat, or no candidate was admissible; predictions then repeat the last loss."""
    L = np.asarray(L, dtype=np.float64)
    L = L[-window:]
    m = len(L)
    out = {"ok": False, "m": m, "cls": cls, "last": float(L[-1]) if m else 0.0}
    if m < 4:
        return out
    lo, hi = float(L.min()), float(L.max())
    span = hi - lo
    if not span > 0:
        return out
    t = np.arange(m, dtype=np.float64) / (m - 1)
    w = gamma ** np.arange(m - 1, -1, -1, dtype=np.float64)
    best = (np.inf, None, None, None)      # sse, exponent, offset, params
    step = (EXP_HI - EXP_LO) / (N_CAND - 1)
    for g in range(N_CAND):                # level 1
        e = EXP_LO + step * g
        off = lo - span * 10.0 ** e
        p, sse = _fit_for_offset(cls, t, L, w, off)
        if sse < best[0]:
            best = (sse, e, off, p)
    if best[1] is None:
        return out
    e0 = best[1]
    step2 = 2.0 * step / (N_CAND - 1)
    for g in range(N_CAND):                # level 2: 64 exponents in [e0 - step, e0 + step]
        e = (e0 - step) + step2 * g
        off = lo - span * 10.0 ** e
        p, sse = _fit_for_offset(cls, t, L, w, off)
        if sse < best[0]:
            best = (sse, e, off, p)
    out.update(ok=True, off=float(best[2]), p=np.asarray(best[3]), sse=float(best[0]))
    return out


def predict(fit, horizon):
    """f at the next `horizon` iterations (h = 1..horizon after the last point of the window)."""
    H = int(horizon)
    if not fit["ok"]:
        return np.full(H, fit["last"])
    m = fit["m"]
    t = (m - 1 + np.arange(1, H + 1, dtype=np.float64)) / (m - 1)
    if fit["cls"] == CLASS_SUBLINEAR:
        a, b, c = fit["p"]
        den = a * t * t + b * t + c
        f = np.where(den > 0, 1.0 / np.where(den > 0, den, 1.0) + fit["off"], fit["last"])
    else:
        p, q = fit["p"]
        f = np.exp(p * t + q) + fit["off"]
    return f


def fitted_value_at_last(fit):
    """f at the last point of the window (t = 1)."""
    if not fit["ok"]:
        return fit["last"]
    if fit["cls"] == CLASS_SUBLINEAR:
        a, b, c = fit["p"]
        den = a + b + c
        return 1.0 / den + fit["off"] if den > 0 else fit["last"]
    p, q = fit["p"]
    return float(np.exp(p + q) + fit["off"])


def predict_job(L, cls=CLASS_SUBLINEAR, gamma=0.9, window=128, horizon=16):
    """(pred[h], gain[h]) for h = 1..horizon: predicted loss and predicted normalised reduction
    contributed by the h-th further iteration."""
    L = np.asarray(L, dtype=np.float64)
    fit = fit_curve(L, cls, gamma, window)
    pred = predict(fit, horizon)
    _, norm = normalized_changes(L) if len(L) >= 2 else (None, 0.0)
    prev = np.concatenate([[fitted_value_at_last(fit)], pred[:-1]])
    gain = (prev - pred) / norm if norm > 0 else np.zeros(int(horizon))
    return pred, gain, fit


def greedy_allocate(gain, capacity):
    """The paper's greedy loop.  gain[j][h-1] is the predicted reduction of job j's h-th unit.
    Starts from one unit per job; each step gives one more unit to the job whose next unit has
    the largest gain (lowest job index on ties); a job holds at most H units.  Stops when the
    capacity is used up or every job holds H units.  Needs capacity >= number of jobs."""
    gain = np.asarray(gain, dtype=np.float64)
    J, H = gain.shape
    if capacity < J:
        raise ValueError("capacity must cover one unit per job")
    a = np.ones(J, dtype=np.int64)
    left = int(capacity) - J
    while left > 0:
        best_j, best_g = -1, -np.inf
        for j in range(J):
            if a[j] < H and gain[j, a[j]] > best_g:
                best_j, best_g = j, gain[j, a[j]]
        if best_j < 0:
            break
        a[best_j] += 1
        left -= 1
    return a
