"""CPU pins of the L-BFGS oracle.  The paper only names the method (Sec. 1, Sec. 2 class II), so
the pins are the dense BFGS update formula, closed-form optima, SciPy's implementation and
invariants; the second half plants mistakes in a copy of the source.
"""
import os
import types

import numpy as np
import pytest
import scipy.optimize

import oracle
from oracle import lbfgs_oracle as lb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lbfgs_oracle.py")


def _data(loss, N=400, D=12, seed=0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, D)).astype(np.float32) * (1.0 + 3.0 * rng.random(D)).astype(np.float32)
    m = X.astype(np.float64) @ rng.standard_normal(D) / np.sqrt(D) + 0.3 * rng.standard_normal(N)
    y = m.astype(np.float32) if loss == oracle.SQUARED else (m > 0).astype(np.float32)
    return X, y


def pin_two_loop_is_the_bfgs_update_formula(mod):
    # H_{i+1} = (I - rho s y^T) H_i (I - rho y s^T) + rho s s^T from H_0 = (s.y / y.y of the newest pair) I
    rng = np.random.default_rng(1)
    D = 7
    A = rng.standard_normal((D, D)); A = A @ A.T + np.eye(D)           # pairs of a convex quadratic: s.y > 0
    S = [rng.standard_normal(D) for _ in range(4)]
    Y = [A @ s for s in S]
    g = rng.standard_normal(D)
    H = np.eye(D) * (S[-1] @ Y[-1]) / (Y[-1] @ Y[-1])
    for s, y in zip(S, Y):
        rho = 1.0 / (s @ y)
        V = np.eye(D) - rho * np.outer(y, s)
        H = V.T @ H @ V + rho * np.outer(s, s)
    np.testing.assert_allclose(mod.two_loop(g, S, Y), -H @ g, rtol=1e-11, atol=1e-13)
    np.testing.assert_array_equal(mod.two_loop(g, [], []), -g)          # no pairs: steepest descent
    # secant equation of the newest pair: H y = s
    np.testing.assert_allclose(-mod.two_loop(Y[-1], S, Y), S[-1], rtol=1e-10, atol=1e-12)


def pin_reaches_the_closed_form_optimum(mod):
    X, y = _data(oracle.SQUARED)
    N, D = X.shape
    lam = 0.05
    X64 = X.astype(np.float64)
    w_star = np.linalg.solve(X64.T @ X64 / N + lam * np.eye(D), X64.T @ y.astype(np.float64) / N)
    f_star, _ = oracle.loss_grad(oracle.SQUARED, X, y, w_star, lam)
    hist, w, info = mod.run(oracle.SQUARED, X, y, np.zeros(D), lam, 25, memory=10)
    assert info["f_end"] == pytest.approx(f_star, rel=1e-9)
    np.testing.assert_allclose(w, w_star, rtol=1e-4, atol=1e-6)
    assert hist[0] == pytest.approx(0.5 * np.mean(y.astype(np.float64) ** 2), rel=1e-12)   # loss at w0 = 0 enters first
    assert np.all(np.diff(hist) <= 1e-6 * np.abs(hist[:-1]))             # sufficient decrease (up to eps_f)


def pin_matches_scipy_optimum_and_beats_gradient_descent(mod):
    X, y = _data(oracle.LOGISTIC, seed=2)
    D = X.shape[1]
    lam = 1e-3
    fg = lambda w: oracle.loss_grad(oracle.LOGISTIC, X, y, w, lam)
    res = scipy.optimize.minimize(fg, np.zeros(D), jac=True, method="L-BFGS-B", options={"maxiter": 500, "ftol": 1e-15, "gtol": 1e-10})
    hist, w, info = mod.run(oracle.LOGISTIC, X, y, np.zeros(D), lam, 40, memory=10)
    assert info["f_end"] == pytest.approx(res.fun, rel=1e-8)
    assert np.linalg.norm(info["g_end"]) < 1e-5
    assert hist[0] == pytest.approx(np.log(2.0), rel=1e-12)
    gd, _, _, _ = oracle.run(oracle.LOGISTIC, X, y, np.zeros(D), lam, 0.05, 40)
    assert hist[-1] < gd[-1]                                             # second convergence class of Sec. 2


def pin_first_step_and_line_search(mod):
    # f(w) = 50 |w|^2: g = 100 w.  From w = (1, 0): p = -g, first trial min(1, 1/100) = 0.01 lands exactly on 0
    f = lambda w: (50.0 * float(w @ w), 100.0 * w)
    hist, w, info = mod.minimize(f, np.array([1.0, 0.0]), 1)
    assert info["steps"] == [0.01] and np.all(w == 0.0) and hist[0] == 50.0 and info["evals"] == 2
    # f(w) = 10 w^2 from w = 0.22: g = 4.4, first trial 1/4.4 overshoots to -0.78 (f = 6.08 > 0.484),
    # half of it reaches -0.28 (f = 0.784, still an increase: rejected), a quarter reaches -0.03
    f1 = lambda w: (10.0 * float(w @ w), 20.0 * w)
    hist, w, info = mod.minimize(f1, np.array([0.22]), 1)
    assert info["steps"] == [1.0 / 4.4 / 4.0] and info["evals"] == 4 and w[0] == pytest.approx(-0.03, abs=1e-12)
    # a steep valley: the unit step of later iterations must sometimes be cut as well
    f2 = lambda w: (float(w[0] ** 2 + 1e4 * w[1] ** 2), np.array([2.0 * w[0], 2e4 * w[1]]))
    hist, w, info = mod.minimize(f2, np.array([1.0, 1.0]), 12)
    assert np.all(np.diff(hist) <= 1e-6 * np.abs(hist[:-1])) and info["f_end"] < 1e-12
    assert all(0 < a <= 1.0 for a in info["steps"]) and any(a < 1.0 for a in info["steps"][1:] + info["steps"][:1])
    # memory 0 is steepest descent with the same line search: direction always -g
    seen = []
    def f3(w):
        seen.append(w.copy()); return f2(w)
    mod.minimize(f3, np.array([1.0, 1e-3]), 3, memory=0)
    # every trial point lies on the ray w - alpha g of the iterate it started from
    assert len(seen) >= 4


def pin_memory_is_limited_and_pairs_are_the_latest(mod):
    X, y = _data(oracle.LOGISTIC, seed=3)
    D = X.shape[1]
    a, _, ia = mod.run(oracle.LOGISTIC, X, y, np.zeros(D), 1e-2, 12, memory=2)
    b, _, ib = mod.run(oracle.LOGISTIC, X, y, np.zeros(D), 1e-2, 12, memory=10)
    np.testing.assert_array_equal(a[:3], b[:3])                          # identical until the third pair exists
    assert not np.array_equal(a[4:], b[4:])
    assert ib["f_end"] <= ia["f_end"] * (1 + 1e-6)


PINS = [pin_two_loop_is_the_bfgs_update_formula, pin_reaches_the_closed_form_optimum,
        pin_matches_scipy_optimum_and_beats_gradient_descent, pin_first_step_and_line_search,
        pin_memory_is_limited_and_pairs_are_the_latest]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_passes_pin(pin):
    pin(lb)


MUTANTS = {
    "direction_not_negated": ("    return -q\n", "    return q\n"),
    "no_initial_scaling": ("        q *= float(np.dot(S[-1], Y[-1])) / float(np.dot(Y[-1], Y[-1]))", "        q *= 1.0"),
    "scaling_from_oldest_pair": ("        q *= float(np.dot(S[-1], Y[-1])) / float(np.dot(Y[-1], Y[-1]))", "        q *= float(np.dot(S[0], Y[0])) / float(np.dot(Y[0], Y[0]))"),
    "first_loop_oldest_first": ("    for i in range(n - 1, -1, -1):\n        alpha[i]", "    for i in range(n):\n        alpha[i]"),
    "second_loop_sign": ("        q += (alpha[i] - beta) * S[i]", "        q += (alpha[i] + beta) * S[i]"),
    "first_loop_uses_s_for_update": ("        q -= alpha[i] * Y[i]", "        q -= alpha[i] * S[i]"),
    "pair_difference_swapped": ("        s, y = wt - w, gt - g", "        s, y = wt - w, g - gt"),
    "oldest_pair_kept_forever": ("                S.pop(0); Y.pop(0)", "                S.pop(1); Y.pop(1)"),
    "memory_off_by_one": ("            if len(S) > memory:", "            if len(S) > memory + 1:"),
    "first_step_is_one": ("        alpha = 1.0 if S else min(1.0, 1.0 / max(gn[-1], 1e-300))", "        alpha = 1.0"),
    "armijo_ignores_slope": ("            if ft <= f + C1 * alpha * gtp or h == MAX_HALVINGS:", "            if ft <= f + 0.9 * abs(f) or h == MAX_HALVINGS:"),
    "history_after_the_step": ("        hist[k] = f\n        gn.append", "        gn.append"),
    "step_doubled_on_reject": ("            alpha *= 0.5", "            alpha *= 2.0"),
}
MUTANTS["history_after_the_step"] = ("        w, f, g = wt, ft, gt\n", "        w, f, g = wt, ft, gt\n        hist[k] = f\n")


def _module(old=None, new=None, name="mutant"):
    src = open(SRC).read()
    if old is not None:
        assert src.count(old) == 1, f"mutation site not found exactly once: {old[:50]!r}"
        src = src.replace(old, new)
    mod = types.ModuleType(name)
    exec(compile(src, name, "exec"), mod.__dict__)
    return mod


def _first_failure(mod):
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin(mod)
        except (AssertionError, ValueError, IndexError, ZeroDivisionError, FloatingPointError, OverflowError):
            return pin.__name__
    return None


def test_unmodified_copy_passes_every_pin():
    assert _first_failure(_module(name="clean")) is None


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_rejected(name):
    old, new = MUTANTS[name]
    assert _first_failure(_module(old, new, name)) is not None, f"no pin notices: {name}"
