"""fp64 CPU oracle for the scheduler-side steps that consume the loss histories
(TEST INFRASTRUCTURE: imported only by tests, the smoke check and the benchmark's CPU leg).

Follows Sec. 2 of the paper:
  * "Normalizing Quality Metrics": the change in loss between iterations is normalised by the
    largest change seen so far.
  * "Predicting Quality Improvement": a curve f(k) = 1/(a k^2 + b k + c) + d (sublinear
    convergence, class I) or f(k) = mu^(k-b) + c (linear/superlinear, class II) is fitted to the
    exponentially weighted loss history and evaluated at future iterations.  The fit itself --
    the weighted least-squares problem over all parameters of the curve, the box that keeps the
    asymptote below the observed losses, and how its minimiser is found -- is sched_fit.c (plain
    C loops; it is called several hundred times per test run).
  * "Scheduling Based on Quality Improvements": start from one unit per job, repeatedly give
    one more unit to the job whose predicted loss reduction for that unit is largest, until the
    capacity is used up.

The paper states neither the weight decay, nor what "normalised loss reduction" is exactly; the
readings taken here (and in the library):
  - weight of history point i of n is gamma^(n-1-i); only the last `window` points are used;
  - iteration numbers are scaled to t = i/(m-1) over the window of m points;
  - the predicted reduction of the h-th further iteration is (f(m-2+h) - f(m-1+h)) divided by
    the largest single-iteration change seen so far in the whole history.
The paper prints no numeric example of any of this: "parity unpinned" against paper values;
the CPU tests pin the routines with exact curves, an independent minimiser, hand examples and
brute force.
"""
from __future__ import annotations

import numpy as np

import oracle

CLASS_SUBLINEAR, CLASS_LINEAR = 1, 2
FIT_LIB = None          # a test may point this at a separately compiled copy of sched_fit.c


def normalized_changes(L):
    """nu_k = (L_{k-1} - L_k) / max_{i<=k} |L_{i-1} - L_i| for k = 1..n-1, and the final normaliser."""
    L = np.asarray(L, dtype=np.float64)
    d = L[:-1] - L[1:]
    run = np.maximum.accumulate(np.abs(d))
    nu = np.where(run > 0, d / np.where(run > 0, run, 1.0), 0.0)
    return nu, (float(run[-1]) if len(run) else 0.0)


def weighted_error(L, cls, gamma, window, off, p):
    """E = sum_i w_i (f(t_i) - L_i)^2 of a given curve on the window: the quantity the fit minimises,
    evaluated directly (used to judge a fit someone else produced)."""
    L = np.asarray(L, dtype=np.float64)[-window:]
    m = len(L)
    t = np.arange(m, dtype=np.float64) / (m - 1)
    w = gamma ** np.arange(m - 1, -1, -1, dtype=np.float64)
    if cls == CLASS_SUBLINEAR:
        q = (p[0] * t + p[1]) * t + p[2]
        if np.any(q <= 0):
            return np.inf
        f = 1.0 / q + off
    else:
        f = np.exp(p[0] * t + p[1]) + off
    return float(np.sum(w * (f - L) ** 2))


def fit_curve(L, cls=CLASS_SUBLINEAR, gamma=0.9, window=128):
    """Fit the convergence curve of class `cls` to the last `window` losses.

    Returns a dict with `ok`, `off` (d or c), `p` (the other parameters, in scaled time and in the
    units of L: class I (a, b, c) with f = 1/(a t^2 + b t + c) + off, class II (p, q) with
    f = exp(p t + q) + off), `e` (offset = min L - span 10^e), `m` (points used), `sse`.  ok is
    False when there are fewer than 5 points, the history is flat or not finite, or nothing
    admissible was found; predictions then repeat the last loss."""
    L = np.asarray(L, dtype=np.float64)
    L = L[-window:]
    m = len(L)
    out = {"ok": False, "m": m, "cls": cls, "last": float(L[-1]) if m else 0.0}
    if m < 5:
        return out
    r = oracle.fit_curve_raw(cls, L, gamma, FIT_LIB)
    if r[0] != 1.0:
        return out
    p = r[2:5] if cls == CLASS_SUBLINEAR else r[2:4]
    out.update(ok=True, off=float(r[1]), p=np.array(p), sse=float(r[5]), e=float(r[6]))
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
