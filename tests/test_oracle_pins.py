"""CPU tests that pin the fp64 oracle to facts it did not produce itself.

The paper prints no value for a training iteration, so the pins are
mathematical: closed forms at w = 0, exact rational arithmetic on a tiny
example, finite differences, the normal equations through a library solver,
library loss metrics, the optimum found by a library optimiser, convexity and
symmetry invariants.
"""
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import HINGE, LOGISTIC, SQUARED


def _rand_problem(loss, N, D, seed, wscale=1.0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, D)).astype(np.float32)
    wt = rng.standard_normal(D) / math.sqrt(D)
    m = X.astype(np.float64) @ wt + 0.3 * rng.standard_normal(N)
    if loss == LOGISTIC:
        y = (m > 0).astype(np.float32)
    elif loss == HINGE:
        y = np.where(m >= 0, 1.0, -1.0).astype(np.float32)
    else:
        y = m.astype(np.float32)
    w = wscale * rng.standard_normal(D)
    return X, y, w


# ---------------------------------------------------------------- closed forms at w = 0

@pytest.mark.parametrize("lam", [0.0, 1e-4, 3.0])
def test_logistic_at_zero_is_ln2(lam):
    X, y, _ = _rand_problem(LOGISTIC, 257, 12, 1)
    L, g = oracle.loss_grad(LOGISTIC, X, y, np.zeros(12), lam)
    assert L == pytest.approx(0.6931471805599453, rel=1e-14)
    g_ref = X.astype(np.float64).T @ (0.5 - y.astype(np.float64)) / 257
    np.testing.assert_allclose(g, g_ref, rtol=0, atol=1e-15)


def test_hinge_at_zero():
    X, y, _ = _rand_problem(HINGE, 300, 7, 2)
    L, g = oracle.loss_grad(HINGE, X, y, np.zeros(7), 0.5)
    assert L == pytest.approx(1.0, abs=1e-15)
    np.testing.assert_allclose(g, -(X.astype(np.float64).T @ y.astype(np.float64)) / 300, atol=1e-15)


def test_squared_at_zero():
    X, y, _ = _rand_problem(SQUARED, 123, 5, 3)
    L, g = oracle.loss_grad(SQUARED, X, y, np.zeros(5), 0.5)
    y64 = y.astype(np.float64)
    assert L == pytest.approx(float(y64 @ y64) / (2 * 123), rel=1e-14)
    np.testing.assert_allclose(g, -(X.astype(np.float64).T @ y64) / 123, atol=1e-14)


# ---------------------------------------------------------------- exact tiny example

_X4 = [[1, 2], [-1, Fraction(1, 2)], [0, -1], [2, 1]]
_W4 = [Fraction(1, 2), Fraction(-1, 4)]
_LAM4 = Fraction(1, 10)


def _exact_margins():
    return [sum(Fraction(x) * w for x, w in zip(row, _W4)) for row in _X4]


def test_worked_example_hinge_exact_rational():
    y = [1, -1, 1, 1]
    z = _exact_margins()
    assert z == [0, Fraction(-5, 8), Fraction(1, 4), Fraction(3, 4)]
    m = [1 - yi * zi for yi, zi in zip(y, z)]
    L = sum(max(Fraction(0), mi) for mi in m) / 4 + _LAM4 / 2 * sum(w * w for w in _W4)
    g = [sum((-yi if mi > 0 else 0) * Fraction(row[j]) for yi, mi, row in zip(y, m, _X4)) / 4
         + _LAM4 * _W4[j] for j in range(2)]
    assert L == Fraction(39, 64) and g == [Fraction(-19, 20), Fraction(-2, 5)]
    Lo, go = oracle.loss_grad(HINGE, np.array(_X4, np.float32), np.array(y, np.float32),
                              [0.5, -0.25], 0.1)
    assert Lo == pytest.approx(float(L), rel=1e-15)
    np.testing.assert_allclose(go, [float(v) for v in g], rtol=1e-15)


def test_worked_example_squared_exact_rational():
    y = [Fraction(1, 2), -1, Fraction(1, 4), 1]
    z = _exact_margins()
    d = [zi - yi for zi, yi in zip(z, y)]
    L = sum(di * di for di in d) / 8 + _LAM4 / 2 * sum(w * w for w in _W4)
    g = [sum(di * Fraction(row[j]) for di, row in zip(d, _X4)) / 4 + _LAM4 * _W4[j] for j in range(2)]
    Lo, go = oracle.loss_grad(SQUARED, np.array(_X4, np.float32),
                              np.array([float(v) for v in y], np.float32), [0.5, -0.25], 0.1)
    assert Lo == pytest.approx(float(L), rel=1e-15)
    np.testing.assert_allclose(go, [float(v) for v in g], rtol=1e-15)


def test_worked_example_logistic_high_precision():
    # independent form: l = ln(1 + exp(-s z)), s = 2y - 1;  r = -s / (1 + exp(s z)); 50-digit decimals
    getcontext().prec = 50
    y = [1, 0, 1, 1]
    z = [Decimal(v.numerator) / Decimal(v.denominator) for v in _exact_margins()]
    L = Decimal(0)
    g = [Decimal(0), Decimal(0)]
    for yi, zi, row in zip(y, z, _X4):
        s = 2 * yi - 1
        L += (1 + (-s * zi).exp()).ln()
        r = -s / (1 + (s * zi).exp())
        for j in range(2):
            g[j] += r * Decimal(float(row[j]))
    lam = Decimal(1) / Decimal(10)
    wd = [Decimal("0.5"), Decimal("-0.25")]
    L = L / 4 + lam / 2 * sum(w * w for w in wd)
    g = [g[j] / 4 + lam * wd[j] for j in range(2)]
    Lo, go = oracle.loss_grad(LOGISTIC, np.array(_X4, np.float32), np.array(y, np.float32),
                              [0.5, -0.25], 0.1)
    assert Lo == pytest.approx(float(L), rel=2e-15)
    np.testing.assert_allclose(go, [float(v) for v in g], rtol=2e-15)


# ---------------------------------------------------------------- finite differences

@pytest.mark.parametrize("loss", [LOGISTIC, SQUARED, HINGE])
def test_gradient_matches_central_differences(loss):
    N, D = 29, 7
    X, y, w = _rand_problem(loss, N, D, 10 + loss, wscale=0.7)
    lam = 0.05
    if loss == HINGE:
        # keep every sample away from the kink so the loss is differentiable at w
        z = X.astype(np.float64) @ w
        assert np.min(np.abs(1.0 - y * z)) > 1e-3
    L, g = oracle.loss_grad(loss, X, y, w, lam)
    h = 1e-6
    for j in range(D):
        e = np.zeros(D); e[j] = h
        Lp, _ = oracle.loss_grad(loss, X, y, w + e, lam)
        Lm, _ = oracle.loss_grad(loss, X, y, w - e, lam)
        fd = (Lp - Lm) / (2 * h)
        assert abs(fd - g[j]) <= 2e-8 * max(1.0, abs(g[j])), (j, fd, g[j])


def test_gradient_matches_scipy_check_grad():
    from scipy.optimize import check_grad
    X, y, w = _rand_problem(LOGISTIC, 40, 6, 77)
    f = lambda v: oracle.loss_grad(LOGISTIC, X, y, v, 0.01)[0]
    gf = lambda v: oracle.loss_grad(LOGISTIC, X, y, v, 0.01)[1]
    assert check_grad(f, gf, w, epsilon=1e-6) < 1e-6


# ---------------------------------------------------------------- library routines

def test_squared_gradient_vanishes_at_normal_equations_solution():
    N, D, lam = 500, 16, 1e-3
    X, y, _ = _rand_problem(SQUARED, N, D, 21)
    X64, y64 = X.astype(np.float64), y.astype(np.float64)
    A = X64.T @ X64 / N + lam * np.eye(D)
    b = X64.T @ y64 / N
    w_opt = np.linalg.solve(A, b)
    _, g = oracle.loss_grad(SQUARED, X, y, w_opt, lam)
    assert np.linalg.norm(g) <= 1e-10 * np.linalg.norm(b)


def test_loss_values_match_sklearn_metrics():
    from sklearn.metrics import hinge_loss, log_loss, mean_squared_error
    N, D = 400, 9
    X, y, w = _rand_problem(LOGISTIC, N, D, 31)
    z = X.astype(np.float64) @ w
    L, _ = oracle.loss_grad(LOGISTIC, X, y, w, 0.0)
    assert L == pytest.approx(log_loss(y, 1.0 / (1.0 + np.exp(-z))), rel=1e-12)
    X, y, w = _rand_problem(HINGE, N, D, 32)
    L, _ = oracle.loss_grad(HINGE, X, y, w, 0.0)
    assert L == pytest.approx(hinge_loss(y, X.astype(np.float64) @ w), rel=1e-12)
    X, y, w = _rand_problem(SQUARED, N, D, 33)
    L, _ = oracle.loss_grad(SQUARED, X, y, w, 0.0)
    assert L == pytest.approx(0.5 * mean_squared_error(y.astype(np.float64), X.astype(np.float64) @ w), rel=1e-12)
    # the L2 term: lam/2 |w|^2 on top of the data term
    L2, _ = oracle.loss_grad(SQUARED, X, y, w, 0.37)
    assert L2 - L == pytest.approx(0.5 * 0.37 * float(w @ w), rel=1e-12)


def test_logistic_gradient_vanishes_at_sklearn_optimum():
    from sklearn.linear_model import LogisticRegression
    N, D, lam = 600, 8, 1e-2
    X, y, _ = _rand_problem(LOGISTIC, N, D, 41)
    clf = LogisticRegression(C=1.0 / (N * lam), fit_intercept=False, tol=1e-12, max_iter=10000)
    clf.fit(X.astype(np.float64), y)
    L, g = oracle.loss_grad(LOGISTIC, X, y, clf.coef_.ravel(), lam)
    assert np.linalg.norm(g) < 1e-6
    # and it is a minimum: any perturbation increases the loss
    rng = np.random.default_rng(0)
    for _ in range(5):
        Lp, _ = oracle.loss_grad(LOGISTIC, X, y, clf.coef_.ravel() + 1e-2 * rng.standard_normal(D), lam)
        assert Lp > L


# ---------------------------------------------------------------- invariants

@pytest.mark.parametrize("loss", [LOGISTIC, HINGE, SQUARED])
def test_first_order_convexity_inequality(loss):
    X, y, _ = _rand_problem(loss, 200, 10, 50 + loss)
    rng = np.random.default_rng(5)
    for _ in range(20):
        w = rng.standard_normal(10); w2 = rng.standard_normal(10) * 2
        L, g = oracle.loss_grad(loss, X, y, w, 0.01)
        L2, _ = oracle.loss_grad(loss, X, y, w2, 0.01)
        assert L2 >= L + g @ (w2 - w) - 1e-12


@pytest.mark.parametrize("loss", [LOGISTIC, SQUARED])
def test_monotone_decrease_for_small_step(loss):
    N, D, lam = 300, 12, 1e-3
    X, y, _ = _rand_problem(loss, N, D, 60 + loss)
    X64 = X.astype(np.float64)
    top = np.linalg.eigvalsh(X64.T @ X64 / N)[-1]
    smooth = (0.25 if loss == LOGISTIC else 1.0) * top + lam
    lh, gh, _, _ = oracle.run(loss, X, y, np.zeros(D), lam, 1.0 / smooth, 60)
    assert np.all(np.diff(lh) <= 1e-15)   # non-increasing up to fp64 rounding once converged
    assert np.all(np.diff(lh[:8]) < 0)
    assert lh[-1] < lh[0] and gh[-1] < gh[0]


def test_hinge_subgradient_method_makes_progress():
    X, y, _ = _rand_problem(HINGE, 400, 10, 70)
    lh, _, _, _ = oracle.run(HINGE, X, y, np.zeros(10), 1e-4, 0.05, 80)
    assert lh[0] == pytest.approx(1.0, abs=1e-15)
    assert lh[1] < lh[0] and lh.min() < 0.7 * lh[0]


def test_label_flip_symmetry():
    X, y, w = _rand_problem(LOGISTIC, 150, 6, 80)
    L, g = oracle.loss_grad(LOGISTIC, X, y, w, 0.02)
    Lf, gf = oracle.loss_grad(LOGISTIC, X, (1 - y).astype(np.float32), -w, 0.02)
    assert Lf == pytest.approx(L, rel=1e-13)
    np.testing.assert_allclose(gf, -g, rtol=1e-12, atol=1e-15)
    X, y, w = _rand_problem(HINGE, 150, 6, 81)
    L, g = oracle.loss_grad(HINGE, X, y, w, 0.02)
    Lf, gf = oracle.loss_grad(HINGE, X, -y, -w, 0.02)
    assert Lf == pytest.approx(L, rel=1e-13)
    np.testing.assert_allclose(gf, -g, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("loss", [LOGISTIC, HINGE, SQUARED])
def test_row_permutation_and_duplication_invariance(loss):
    X, y, w = _rand_problem(loss, 101, 5, 90 + loss)
    L, g = oracle.loss_grad(loss, X, y, w, 0.03)
    p = np.random.default_rng(1).permutation(101)
    Lp, gp = oracle.loss_grad(loss, X[p], y[p], w, 0.03)
    assert Lp == pytest.approx(L, rel=1e-13)
    np.testing.assert_allclose(gp, g, rtol=1e-11, atol=1e-14)
    Ld, gd = oracle.loss_grad(loss, np.concatenate([X, X]), np.concatenate([y, y]), w, 0.03)
    assert Ld == pytest.approx(L, rel=1e-13)      # fails if a sum were used instead of a mean
    np.testing.assert_allclose(gd, g, rtol=1e-11, atol=1e-14)


def test_column_swap_moves_gradient_entries():
    # catches a transposed or mis-strided X: swapping two columns (and the two weights)
    # must swap exactly those gradient entries
    X, y, w = _rand_problem(LOGISTIC, 64, 6, 95)
    L, g = oracle.loss_grad(LOGISTIC, X, y, w, 0.01)
    Xs = X.copy(); Xs[:, [1, 4]] = X[:, [4, 1]]
    ws = w.copy(); ws[[1, 4]] = w[[4, 1]]
    Ls, gs = oracle.loss_grad(LOGISTIC, Xs, y, ws, 0.01)
    assert Ls == pytest.approx(L, rel=1e-13)
    np.testing.assert_allclose(gs[[1, 4]], g[[4, 1]], rtol=1e-12)
    np.testing.assert_allclose(gs[[0, 2, 3, 5]], g[[0, 2, 3, 5]], rtol=1e-12)


def test_logistic_large_margins_are_finite():
    X = np.array([[1000.0], [-1000.0], [1000.0], [-1000.0]], np.float32)
    y = np.array([1, 0, 0, 1], np.float32)
    L, g = oracle.loss_grad(LOGISTIC, X, y, [1.0], 0.0)
    assert math.isfinite(L) and np.all(np.isfinite(g))
    assert L == pytest.approx((0 + 0 + 1000 + 1000) / 4, rel=1e-15)
    assert g[0] == pytest.approx((0 + 0 + 1000 * 1 + (-1000) * (-1)) / 4, rel=1e-15)


def test_hinge_kink_is_inactive():
    # y z = 1 exactly: loss 0 and the subgradient taken is 0 (strict inequality)
    X = np.array([[1.0], [2.0]], np.float32)
    y = np.array([1.0, 1.0], np.float32)
    L, g = oracle.loss_grad(HINGE, X, y, [1.0], 0.0)
    assert L == 0.0 and g[0] == 0.0


# ---------------------------------------------------------------- drivers

@pytest.mark.parametrize("loss", [LOGISTIC, HINGE, SQUARED])
def test_chunked_evaluation_equals_sequential(loss):
    X, y, w = _rand_problem(loss, 1037, 20, 100 + loss)
    L, g = oracle.loss_grad(loss, X, y, w, 0.01)
    for chunks in (2, 7, 16, 5000):
        Lc, gc = oracle.loss_grad(loss, X, y, w, 0.01, chunks=chunks)
        assert Lc == pytest.approx(L, rel=1e-13)
        np.testing.assert_allclose(gc, g, rtol=1e-11, atol=1e-14)


def test_run_replays_loss_grad_and_update():
    X, y, _ = _rand_problem(LOGISTIC, 97, 6, 110)
    lam, eta, K = 0.01, 0.3, 7
    lh, gh, wK, gl = oracle.run(LOGISTIC, X, y, np.zeros(6), lam, eta, K)
    w = np.zeros(6)
    for k in range(K):
        L, g = oracle.loss_grad(LOGISTIC, X, y, w, lam)
        assert lh[k] == L and gh[k] == pytest.approx(np.linalg.norm(g), rel=1e-15)
        w = w - eta * g
    np.testing.assert_array_equal(w, wK)
    np.testing.assert_array_equal(g, gl)


def test_sweep_is_independent_runs():
    X, y, _ = _rand_problem(LOGISTIC, 80, 5, 120)
    lams = [0.0, 0.1, 0.01]; etas = [0.1, 0.2, 0.5]
    lh, gh, WK, GL = oracle.run_sweep(LOGISTIC, X, y, np.zeros((3, 5)), lams, etas, 4)
    for m in range(3):
        a, b, c, d = oracle.run(LOGISTIC, X, y, np.zeros(5), lams[m], etas[m], 4)
        np.testing.assert_array_equal(lh[:, m], a)
        np.testing.assert_array_equal(WK[m], c)


def test_rejects_bad_arguments():
    X = np.zeros((4, 2), np.float32); y = np.zeros(4, np.float32)
    with pytest.raises(ValueError):
        oracle.loss_grad(7, X, y, [0, 0], 0.0)
    with pytest.raises(TypeError):
        oracle.loss_grad(0, X.astype(np.float64), y, [0, 0], 0.0)
    with pytest.raises(ValueError):
        oracle.loss_grad(0, X, y, [0, 0, 0], 0.0)
