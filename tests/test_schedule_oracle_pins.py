"""Pins of the oracle's step schedules (oracle_run_schedule): closed forms on problems whose
iterates can be written down, agreement with the constant-step routine, split runs, and planted
mistakes in a copy of the C source (CPU only)."""
import ctypes
import math
import os
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "glm_oracle.c")
SQUARED, HINGE = 2, 1


def _pins(run):
    """run(loss, X, y, w0, lam, eta, schedule, K, k0) -> (loss_hist, gnorm_hist, w, g_last)."""
    # 1. one sample, one feature, squared loss, no L2: L = w^2 / 2, g = w, so
    #    w_{k+1} = w_k (1 - eta / sqrt(k + 1)) and loss_hist[k] = w_k^2 / 2
    X = np.array([[1.0]], np.float32); y = np.array([0.0], np.float32)
    eta, K = 0.3, 9
    lh, gh, w, _ = run(SQUARED, X, y, np.array([2.0]), 0.0, eta, oracle.INV_SQRT, K, 0)
    wk, want = 2.0, []
    for k in range(K):
        want.append(0.5 * wk * wk)
        wk *= 1.0 - eta / math.sqrt(k + 1)
    assert np.allclose(lh, want, rtol=1e-14, atol=0) and math.isclose(w[0], wk, rel_tol=1e-14)
    assert math.isclose(lh[4] / lh[3], (1.0 - eta / 2.0) ** 2, rel_tol=1e-13)      # the 4th step is eta / 2

    # 2. hinge loss with every sample active throughout: the gradient is the constant -mean(y x),
    #    so w_K = w_0 - g * eta * sum_k 1 / sqrt(k + 1)
    rng = np.random.default_rng(0)
    X = rng.standard_normal((40, 6)).astype(np.float32) * 0.01
    y = np.where(rng.random(40) < 0.5, -1.0, 1.0).astype(np.float32)
    g = -(y[:, None].astype(np.float64) * X.astype(np.float64)).mean(0)
    K, eta = 7, 0.05
    lh, gh, w, gl = run(HINGE, X, y, np.zeros(6), 0.0, eta, oracle.INV_SQRT, K, 0)
    assert np.allclose(gl, g, rtol=1e-13, atol=0)
    assert np.allclose(w, -g * eta * sum(1.0 / math.sqrt(k + 1) for k in range(K)), rtol=1e-12, atol=0)

    # 3. the constant schedule is the constant-step routine, bit for bit
    X = rng.standard_normal((50, 8)).astype(np.float32); y = rng.standard_normal(50).astype(np.float32)
    a = run(SQUARED, X, y, np.zeros(8), 1e-3, 0.1, oracle.CONSTANT, 6, 0)
    b = oracle.run(SQUARED, X, y, np.zeros(8), 1e-3, 0.1, 6)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    assert not np.array_equal(a[2], run(SQUARED, X, y, np.zeros(8), 1e-3, 0.1, oracle.INV_SQRT, 6, 0)[2])

    # 4. a run split into two calls takes the same steps as one call
    one = run(SQUARED, X, y, np.zeros(8), 1e-3, 0.2, oracle.INV_SQRT, 5, 0)
    first = run(SQUARED, X, y, np.zeros(8), 1e-3, 0.2, oracle.INV_SQRT, 2, 0)
    second = run(SQUARED, X, y, first[2], 1e-3, 0.2, oracle.INV_SQRT, 3, 2)
    assert np.array_equal(one[2], second[2]) and np.array_equal(one[0], np.concatenate([first[0], second[0]]))

    # 5. the constant schedule does not look at k0
    c = run(SQUARED, X, y, np.zeros(8), 1e-3, 0.1, oracle.CONSTANT, 6, 17)
    assert all(np.array_equal(u, v) for u, v in zip(a, c))


def test_schedule_pins_hold_for_the_oracle():
    _pins(oracle.run_schedule)


def test_schedule_arguments_are_checked():
    X = np.ones((2, 4), np.float32); y = np.zeros(2, np.float32)
    with pytest.raises(ValueError):
        oracle.run_schedule(SQUARED, X, y, np.zeros(4), 0.0, 0.1, 2, 3)
    with pytest.raises(ValueError):
        oracle.run_schedule(SQUARED, X, y, np.zeros(4), 0.0, 0.1, oracle.INV_SQRT, 3, k0=-1)


def _as_csr(X):
    X = np.asarray(X, np.float32)
    N, D = X.shape
    rp = np.arange(N + 1, dtype=np.int64) * D
    ci = np.tile(np.arange(D, dtype=np.int32), N)
    return rp, ci, np.ascontiguousarray(X.reshape(-1))


def _sparse_pins(srun):
    """srun(loss, rp, ci, v, y, D, w0, lam, eta, schedule, K, k0) -> as run."""
    # the closed form of pin 1 through the CSR routine (the single entry stored explicitly)
    rp, ci, v = _as_csr([[1.0]]); y = np.array([0.0], np.float32)
    eta, K = 0.3, 9
    lh, gh, w, _ = srun(SQUARED, rp, ci, v, y, 1, np.array([2.0]), 0.0, eta, oracle.INV_SQRT, K, 0)
    wk, want = 2.0, []
    for k in range(K):
        want.append(0.5 * wk * wk)
        wk *= 1.0 - eta / math.sqrt(k + 1)
    assert np.allclose(lh, want, rtol=1e-14, atol=0) and math.isclose(w[0], wk, rel_tol=1e-14)
    # a matrix with real zeros: the scheduled CSR run follows the scheduled dense run (pinned above)
    rng = np.random.default_rng(1)
    X = (rng.standard_normal((60, 7)) * (rng.random((60, 7)) < 0.4)).astype(np.float32)
    y = rng.standard_normal(60).astype(np.float32)
    import scipy.sparse as sp
    A = sp.csr_matrix(X)
    args = (A.indptr.astype(np.int64), A.indices.astype(np.int32), A.data.astype(np.float32), y, 7)
    a = srun(SQUARED, *args, np.zeros(7), 1e-3, 0.2, oracle.INV_SQRT, 6, 0)
    b = oracle.run_schedule(SQUARED, X, y, np.zeros(7), 1e-3, 0.2, oracle.INV_SQRT, 6)
    assert np.allclose(a[0], b[0], rtol=1e-12, atol=0) and np.allclose(a[2], b[2], rtol=1e-12, atol=1e-15)
    # constant schedule = the constant-step CSR routine, bit for bit; k0 ignored there
    c = srun(SQUARED, *args, np.zeros(7), 1e-3, 0.2, oracle.CONSTANT, 6, 11)
    d = oracle.sparse_run(SQUARED, *args, np.zeros(7), 1e-3, 0.2, 6)
    assert all(np.array_equal(u, v_) for u, v_ in zip(c, d))
    # split run
    first = srun(SQUARED, *args, np.zeros(7), 1e-3, 0.2, oracle.INV_SQRT, 2, 0)
    second = srun(SQUARED, *args, first[2], 1e-3, 0.2, oracle.INV_SQRT, 4, 2)
    assert np.array_equal(a[2], second[2]) and np.array_equal(a[0], np.concatenate([first[0], second[0]]))


def test_sparse_schedule_pins_hold_for_the_oracle():
    _sparse_pins(oracle.sparse_run_schedule)


SPARSE_MUTANTS = {
    "sqrt_of_k_instead_of_k_plus_1": ("eta / sqrt((double)(ks + 1))", "eta / sqrt((double)(ks > 0 ? ks : 1))"),
    "one_over_k_decay": ("eta / sqrt((double)(ks + 1))", "eta / (double)(ks + 1)"),
    "position_in_call_instead_of_job": ("const int64_t ks = k0 + i;", "const int64_t ks = i;"),
    "decay_applied_to_constant": ("(schedule == 1) ? eta / sqrt((double)(ks", "(schedule >= 0) ? eta / sqrt((double)(ks"),
    "constant_applied_to_decay": ("(schedule == 1) ? eta / sqrt((double)(ks", "(schedule == 2) ? eta / sqrt((double)(ks"),
    "update_with_plus": ("w[j] = w[j] - eta_ks * g[j];", "w[j] = w[j] + eta_ks * g[j];"),
}


@pytest.mark.parametrize("name", sorted(SPARSE_MUTANTS))
def test_each_planted_sparse_schedule_mistake_is_caught(tmp_path, name):
    old, new = SPARSE_MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    c = tmp_path / f"{name}.c"; so = tmp_path / f"{name}.so"
    c.write_text(src.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
    i64p, i32p = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)
    lib.oracle_sparse_run_schedule.restype = ctypes.c_int
    lib.oracle_sparse_run_schedule.argtypes = [ctypes.c_int, i64p, i32p, fp, fp, ctypes.c_int64, ctypes.c_int64, dp,
                                               ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_int64,
                                               ctypes.c_int32, dp, dp, dp]

    def srun(loss, rp, ci, v, y, D, w0, lam, eta, schedule, K, k0):
        rp = np.ascontiguousarray(rp, np.int64); ci = np.ascontiguousarray(ci, np.int32)
        v = np.ascontiguousarray(v, np.float32); y = np.ascontiguousarray(y, np.float32)
        w = np.array(w0, dtype=np.float64, copy=True)
        lh = np.zeros(K); gh = np.zeros(K); gl = np.zeros(D)
        rc = lib.oracle_sparse_run_schedule(loss, rp.ctypes.data_as(i64p), ci.ctypes.data_as(i32p), v.ctypes.data_as(fp),
                                            y.ctypes.data_as(fp), len(y), D, w.ctypes.data_as(dp), lam, eta, schedule, k0,
                                            K, lh.ctypes.data_as(dp), gh.ctypes.data_as(dp), gl.ctypes.data_as(dp))
        assert rc == 0
        return lh, gh, w, gl
    with pytest.raises(AssertionError):
        _sparse_pins(srun)


MUTANTS = {
    "sqrt_of_k_instead_of_k_plus_1": ("eta / sqrt((double)(k + 1))", "eta / sqrt((double)(k > 0 ? k : 1))"),
    "one_over_k_decay": ("eta / sqrt((double)(k + 1))", "eta / (double)(k + 1)"),
    "position_in_call_instead_of_job": ("const int64_t k = k0 + i;", "const int64_t k = i;"),
    "decay_applied_to_constant": ("(schedule == 1) ? eta / sqrt((double)(k +", "(schedule >= 0) ? eta / sqrt((double)(k +"),
    "constant_applied_to_decay": ("(schedule == 1) ? eta / sqrt((double)(k +", "(schedule == 2) ? eta / sqrt((double)(k +"),
    "multiplies_by_sqrt": ("eta / sqrt((double)(k + 1))", "eta * sqrt((double)(k + 1))"),
    "update_with_plus": ("w[j] = w[j] - eta_k * g[j];", "w[j] = w[j] + eta_k * g[j];"),
    "loss_not_recorded": ("loss_hist[i] = L;\n        gnorm_hist[i] = sqrt(gg);\n        const int64_t k = k0",
                              "gnorm_hist[i] = sqrt(gg);\n        const int64_t k = k0"),
}


def _mutant_run(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = src.replace(old, new)
    c = tmp_path / f"{name}.c"; so = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
    lib.oracle_run_schedule.restype = ctypes.c_int
    lib.oracle_run_schedule.argtypes = [ctypes.c_int, fp, fp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_double,
                                        ctypes.c_double, ctypes.c_int, ctypes.c_int64, ctypes.c_int32, dp, dp, dp]

    def run(loss, X, y, w0, lam, eta, schedule, K, k0):
        X = np.ascontiguousarray(X, np.float32); y = np.ascontiguousarray(y, np.float32)
        w = np.array(w0, dtype=np.float64, copy=True)
        lh = np.zeros(K); gh = np.zeros(K); gl = np.zeros(X.shape[1])
        rc = lib.oracle_run_schedule(loss, X.ctypes.data_as(fp), y.ctypes.data_as(fp), X.shape[0], X.shape[1],
                                     w.ctypes.data_as(dp), lam, eta, schedule, k0, K, lh.ctypes.data_as(dp),
                                     gh.ctypes.data_as(dp), gl.ctypes.data_as(dp))
        assert rc == 0
        return lh, gh, w, gl
    return run


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_each_planted_schedule_mistake_is_caught(tmp_path, name):
    old, new = MUTANTS[name]
    run = _mutant_run(tmp_path, name, old, new)
    with pytest.raises(AssertionError):
        _pins(run)
