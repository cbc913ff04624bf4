"""Do the pins bite?  Each test plants one plausible mistake in a COPY of the oracle's C source
(on the CPU, in a temporary directory), compiles it, and checks that at least one of the
closed-form / library / invariant pins used in test_oracle_pins.py rejects the mutant, while
the unmodified source passes all of them.  Nothing here touches the GPU library.
"""
import ctypes
import math
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "glm_oracle.c")

MUTANTS = {
    "sum_instead_of_mean_loss": ("*L_out = S / (double)N + 0.5 * lambda * ww;",
                                 "*L_out = S + 0.5 * lambda * ww;"),
    "sum_instead_of_mean_grad": ("g[j] = g[j] / (double)N + lambda * w[j];",
                                 "g[j] = g[j] + lambda * w[j];"),
    "dropped_l2_in_gradient": ("g[j] = g[j] / (double)N + lambda * w[j];",
                               "g[j] = g[j] / (double)N;"),
    "dropped_l2_in_loss": ("*L_out = S / (double)N + 0.5 * lambda * ww;", "*L_out = S / (double)N;"),
    "l2_without_half": ("*L_out = S / (double)N + 0.5 * lambda * ww;",
                        "*L_out = S / (double)N + lambda * ww;"),
    "logistic_residual_sign": ("*r = sig - y;", "*r = y - sig;"),
    "logistic_missing_label_term": ("*l = sp - y * z;", "*l = sp;"),
    "sigmoid_of_minus_z": ("sig = 1.0 / (1.0 + exp(-z));", "sig = 1.0 / (1.0 + exp(z));"),
    "hinge_wrong_margin_sign": ("double m = 1.0 - y * z;", "double m = 1.0 + y * z;"),
    "hinge_residual_sign": ("{ *l = m;   *r = -y;  }", "{ *l = m;   *r = y;  }"),
    "hinge_kink_active": ("if (m > 0.0) { *l = m;", "if (m >= 0.0) { *l = m;"),
    "squared_missing_half": ("*l = 0.5 * d * d;", "*l = d * d;"),
    "squared_residual_sign": ("double d = z - y;\n        *l", "double d = y - z;\n        *l"),
    "transposed_row_stride": ("const float *row = X + i * (int64_t)D;", "const float *row = X + i;"),
    "margin_skips_last_column": ("for (int32_t j = 0; j < D; ++j) z += (double)row[j] * w[j];",
                                 "for (int32_t j = 0; j + 1 < D; ++j) z += (double)row[j] * w[j];"),
    "column_pass_off_by_one": ("for (int32_t j = 0; j < D; ++j) s[j] += (double)row[j] * r;",
                               "for (int32_t j = 1; j < D; ++j) s[j] += (double)row[j] * r;"),
    "update_with_plus": ("w[j] -= eta * g[j];", "w[j] += eta * g[j];"),
    "softplus_overflows": ("double sp = (z > 0.0 ? z : 0.0) + log1p(exp(-fabs(z)));",
                           "double sp = log(1.0 + exp(z));"),
}


def _compile(tmp_path, name, old=None, new=None):
    src = open(SRC).read()
    if old is not None:
        # the finalisation lines also occur in the chunked variant, which the pins below do
        # not call (it is pinned to the sequential routine elsewhere): mutate the first site
        assert src.count(old) >= 1, f"mutation site for {name} not found"
        src = src.replace(old, new, 1)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
    lib.oracle_loss_grad.argtypes = [ctypes.c_int, fp, fp, ctypes.c_int64, ctypes.c_int32, dp,
                                     ctypes.c_double, dp, dp]
    lib.oracle_run.argtypes = [ctypes.c_int, fp, fp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_double,
                               ctypes.c_double, ctypes.c_int32, ctypes.c_int32, dp, dp, dp]
    return lib


class _Oracle:
    def __init__(self, lib):
        self.lib = lib

    def loss_grad(self, loss, X, y, w, lam):
        X = np.ascontiguousarray(X, np.float32); y = np.ascontiguousarray(y, np.float32)
        w = np.ascontiguousarray(w, np.float64)
        g = np.empty(X.shape[1]); L = ctypes.c_double()
        fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        self.lib.oracle_loss_grad(loss, X.ctypes.data_as(fp), y.ctypes.data_as(fp), X.shape[0], X.shape[1],
                                  w.ctypes.data_as(dp), lam, ctypes.byref(L), g.ctypes.data_as(dp))
        return L.value, g

    def run(self, loss, X, y, w0, lam, eta, K):
        X = np.ascontiguousarray(X, np.float32); y = np.ascontiguousarray(y, np.float32)
        w = np.array(w0, np.float64); lh = np.empty(K); gh = np.empty(K); gl = np.empty(X.shape[1])
        fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        self.lib.oracle_run(loss, X.ctypes.data_as(fp), y.ctypes.data_as(fp), X.shape[0], X.shape[1],
                            w.ctypes.data_as(dp), lam, eta, K, 0, lh.ctypes.data_as(dp),
                            gh.ctypes.data_as(dp), gl.ctypes.data_as(dp))
        return lh, gh, w


def _data(loss, N, D, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, D)).astype(np.float32)
    m = X.astype(np.float64) @ (rng.standard_normal(D) / math.sqrt(D)) + 0.3 * rng.standard_normal(N)
    y = {0: (m > 0).astype(np.float32), 1: np.where(m >= 0, 1.0, -1.0).astype(np.float32),
         2: m.astype(np.float32)}[loss]
    return X, y, rng.standard_normal(D)


def _pins(o):
    """A condensed set of the pins of test_oracle_pins.py; returns the names of those that fail."""
    failed = []

    def check(name, ok):
        if not ok:
            failed.append(name)

    # closed forms at w = 0 (lambda > 0 must not matter there)
    for loss, L0 in ((0, math.log(2.0)), (1, 1.0)):
        X, y, _ = _data(loss, 301, 7, 1 + loss)
        L, g = o.loss_grad(loss, X, y, np.zeros(7), 0.7)
        ref = X.astype(np.float64).T @ ((0.5 - y) if loss == 0 else -y.astype(np.float64)) / 301
        check(f"w0_loss_{loss}", abs(L - L0) < 1e-12)
        check(f"w0_grad_{loss}", np.allclose(g, ref, rtol=0, atol=1e-13))
    X, y, _ = _data(2, 123, 5, 3)
    L, g = o.loss_grad(2, X, y, np.zeros(5), 0.7)
    y64 = y.astype(np.float64)
    check("w0_loss_2", abs(L - y64 @ y64 / 246) < 1e-12 * max(1.0, abs(L)))
    check("w0_grad_2", np.allclose(g, -(X.astype(np.float64).T @ y64) / 123, atol=1e-13))
    # finite differences, all three losses, lambda > 0
    for loss in (0, 1, 2):
        X, y, w = _data(loss, 29, 7, 10 + loss)
        w = 0.7 * w
        L, g = o.loss_grad(loss, X, y, w, 0.05)
        for j in range(7):
            e = np.zeros(7); e[j] = 1e-6
            fd = (o.loss_grad(loss, X, y, w + e, 0.05)[0] - o.loss_grad(loss, X, y, w - e, 0.05)[0]) / 2e-6
            check(f"fd_{loss}", abs(fd - g[j]) <= 2e-8 * max(1.0, abs(g[j])))
    # normal equations
    X, y, _ = _data(2, 500, 16, 21)
    X64 = X.astype(np.float64)
    A = X64.T @ X64 / 500 + 1e-3 * np.eye(16); b = X64.T @ y.astype(np.float64) / 500
    _, g = o.loss_grad(2, X, y, np.linalg.solve(A, b), 1e-3)
    check("normal_equations", np.linalg.norm(g) <= 1e-10 * np.linalg.norm(b))
    # library loss values
    from sklearn.metrics import hinge_loss, log_loss, mean_squared_error
    X, y, w = _data(0, 400, 9, 31); z = X.astype(np.float64) @ w
    check("sk_logloss", abs(o.loss_grad(0, X, y, w, 0.0)[0] - log_loss(y, 1 / (1 + np.exp(-z)))) < 1e-11)
    X, y, w = _data(1, 400, 9, 32)
    check("sk_hinge", abs(o.loss_grad(1, X, y, w, 0.0)[0] - hinge_loss(y, X.astype(np.float64) @ w)) < 1e-11)
    X, y, w = _data(2, 400, 9, 33)
    L0 = o.loss_grad(2, X, y, w, 0.0)[0]
    check("sk_mse", abs(L0 - 0.5 * mean_squared_error(y.astype(np.float64), X.astype(np.float64) @ w)) < 1e-11)
    check("l2_term", abs(o.loss_grad(2, X, y, w, 0.37)[0] - L0 - 0.5 * 0.37 * float(w @ w)) < 1e-11)
    # duplication invariance, convexity, monotone decrease, large margins, hinge kink
    X, y, w = _data(0, 101, 5, 90)
    L, g = o.loss_grad(0, X, y, w, 0.03)
    Ld, gd = o.loss_grad(0, np.concatenate([X, X]), np.concatenate([y, y]), w, 0.03)
    check("duplication", abs(Ld - L) < 1e-12 and np.allclose(gd, g, atol=1e-13))
    for loss in (0, 1, 2):
        X, y, _ = _data(loss, 200, 10, 50 + loss)
        rng = np.random.default_rng(5)
        for _ in range(10):
            a, b2 = rng.standard_normal(10), 2 * rng.standard_normal(10)
            La, ga = o.loss_grad(loss, X, y, a, 0.01)
            check(f"convex_{loss}", o.loss_grad(loss, X, y, b2, 0.01)[0] >= La + ga @ (b2 - a) - 1e-12)
    X, y, _ = _data(0, 300, 12, 60)
    top = np.linalg.eigvalsh(X.astype(np.float64).T @ X.astype(np.float64) / 300)[-1]
    lh, _, _ = o.run(0, X, y, np.zeros(12), 1e-3, 1.0 / (0.25 * top + 1e-3), 30)
    check("monotone", bool(np.all(np.diff(lh) <= 1e-15)) and lh[-1] < lh[0])
    Xb = np.array([[1000.0], [-1000.0], [1000.0], [-1000.0]], np.float32)
    Lb, gb = o.loss_grad(0, Xb, np.array([1, 0, 0, 1], np.float32), [1.0], 0.0)
    check("large_margin", math.isfinite(Lb) and abs(Lb - 500.0) < 1e-9 and abs(gb[0] - 500.0) < 1e-9)
    Lk, gk = o.loss_grad(1, np.array([[1.0], [2.0]], np.float32), np.array([1.0, 1.0], np.float32), [1.0], 0.0)
    check("hinge_kink", Lk == 0.0 and gk[0] == 0.0)
    return failed


def test_unmodified_oracle_passes_every_pin(tmp_path):
    assert _pins(_Oracle(_compile(tmp_path, "clean"))) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTANTS[name]
    failed = _pins(_Oracle(_compile(tmp_path, name, old, new)))
    assert failed, f"no pin noticed the planted mistake '{name}'"
