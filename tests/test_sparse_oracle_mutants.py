"""Do the pins of the sparse oracle bite?  One plausible mistake at a time is planted in a COPY
of the C source (CPU only, temporary directory); the SciPy sparse-algebra pin, the closed form at
w = 0 and the replay pin of test_sparse_oracle_pins.py must reject it, and accept the clean copy.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest
import scipy.sparse as sp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "glm_oracle.c")

MUTANTS = {
    "margin_skips_last_entry": ("for (int64_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {\n            if (col_idx[e] < 0",
                                "for (int64_t e = row_ptr[i]; e + 1 < row_ptr[i + 1]; ++e) {\n            if (col_idx[e] < 0"),
    "margin_uses_entry_index_as_column": ("z += (double)val[e] * w[col_idx[e]];", "z += (double)val[e] * w[e % D];"),
    "gradient_skips_first_entry": ("for (int64_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) g[col_idx[e]] += (double)val[e] * r;",
                                   "for (int64_t e = row_ptr[i] + 1; e < row_ptr[i + 1]; ++e) g[col_idx[e]] += (double)val[e] * r;"),
    "gradient_overwrites_duplicates": ("g[col_idx[e]] += (double)val[e] * r;", "g[col_idx[e]] = (double)val[e] * r;"),
    "gradient_scatter_by_row": ("g[col_idx[e]] += (double)val[e] * r;", "g[i % D] += (double)val[e] * r;"),
    "sparse_sum_instead_of_mean": ("*L_out = S / (double)N + 0.5 * lambda * ww;\n    for (int64_t j", "*L_out = S + 0.5 * lambda * ww;\n    for (int64_t j"),
    "sparse_gradient_not_averaged": ("for (int64_t j = 0; j < D; ++j) g[j] = g[j] / (double)N + lambda * w[j];\n    return 0;\n}\n\n/* K constant-step",
                                     "for (int64_t j = 0; j < D; ++j) g[j] = g[j] + lambda * w[j];\n    return 0;\n}\n\n/* K constant-step"),
    "sparse_update_with_plus": ("for (int64_t j = 0; j < D; ++j) w[j] -= eta * g[j];", "for (int64_t j = 0; j < D; ++j) w[j] += eta * g[j];"),
    "sparse_history_after_update": ("        loss_hist[k] = L;\n        gnorm_hist[k] = sqrt(gg);\n        for (int64_t j = 0; j < D; ++j) w[j] -= eta * g[j];",
                                    "        for (int64_t j = 0; j < D; ++j) w[j] -= eta * g[j];\n        loss_hist[k] = L + 1e-3 * w[0];\n        gnorm_hist[k] = sqrt(gg);"),
}


def _compile(tmp_path, name, old=None, new=None):
    src = open(SRC).read()
    if old is not None:
        assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
        src = src.replace(old, new)
    c = tmp_path / f"{name}.c"; so = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
    lp, ip = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)
    lib.oracle_sparse_loss_grad.argtypes = [ctypes.c_int, lp, ip, fp, fp, ctypes.c_int64, ctypes.c_int64, dp,
                                            ctypes.c_double, dp, dp]
    lib.oracle_sparse_run.argtypes = [ctypes.c_int, lp, ip, fp, fp, ctypes.c_int64, ctypes.c_int64, dp, ctypes.c_double,
                                      ctypes.c_double, ctypes.c_int32, dp, dp, dp]
    return lib


def _ptrs(rp, ci, v, y):
    fp = ctypes.POINTER(ctypes.c_float)
    return (rp.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), ci.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
            v.ctypes.data_as(fp), y.ctypes.data_as(fp))


def _loss_grad(lib, loss, rp, ci, v, y, D, w, lam):
    g = np.empty(D); L = ctypes.c_double()
    w = np.ascontiguousarray(w, np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = lib.oracle_sparse_loss_grad(loss, *_ptrs(rp, ci, v, y), len(y), D, w.ctypes.data_as(dp), lam, ctypes.byref(L),
                                     g.ctypes.data_as(dp))
    assert rc == 0
    return L.value, g


def _matrix(seed):
    """A small CSR matrix with unsorted columns, repeated (row, column) pairs and an empty row."""
    rng = np.random.default_rng(seed)
    N, D = 40, 13
    counts = rng.integers(0, 7, size=N); counts[5] = 0
    rp = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    ci = rng.integers(0, D, size=rp[-1]).astype(np.int32)
    ci[rp[7] + 1] = ci[rp[7]]                                  # a duplicate pair in row 7 (counts[7] >= 2 by seed)
    v = rng.standard_normal(rp[-1]).astype(np.float32)
    return N, D, rp, ci, v


def _pins(lib):
    for loss in (0, 1, 2):
        N, D, rp, ci, v = _matrix(3)
        rng = np.random.default_rng(10 + loss)
        y = {0: (rng.random(N) > 0.5).astype(np.float32), 1: np.where(rng.random(N) > 0.5, 1, -1).astype(np.float32),
             2: rng.standard_normal(N).astype(np.float32)}[loss]
        A = sp.csr_matrix((v.astype(np.float64), ci, rp), shape=(N, D))       # SciPy sums duplicates
        w = rng.standard_normal(D); lam = 0.2
        L, g = _loss_grad(lib, loss, rp, ci, v, y, D, w, lam)
        z = A @ w; yd = y.astype(np.float64)
        if loss == 0:
            l = np.logaddexp(0, z) - yd * z; r = 1 / (1 + np.exp(-z)) - yd
        elif loss == 1:
            m = 1 - yd * z; l = np.maximum(m, 0); r = np.where(m > 0, -yd, 0.0)
        else:
            l = 0.5 * (z - yd) ** 2; r = z - yd
        assert L == pytest.approx(l.mean() + 0.5 * lam * w @ w, rel=1e-12)
        np.testing.assert_allclose(g, A.T @ r / N + lam * w, rtol=1e-10, atol=1e-14)
        # K iterations replay loss_grad and descend
        K = 4; eta = 0.1
        wr = w.copy(); lh = np.empty(K); gh = np.empty(K); gl = np.empty(D)
        dp = ctypes.POINTER(ctypes.c_double)
        rc = lib.oracle_sparse_run(loss, *_ptrs(rp, ci, v, y), N, D, wr.ctypes.data_as(dp), lam, eta, K,
                                   lh.ctypes.data_as(dp), gh.ctypes.data_as(dp), gl.ctypes.data_as(dp))
        assert rc == 0
        ww = w.copy()
        for k in range(K):
            Lk, gk = _loss_grad(lib, loss, rp, ci, v, y, D, ww, lam)
            assert lh[k] == pytest.approx(Lk, rel=1e-14) and gh[k] == pytest.approx(np.linalg.norm(gk), rel=1e-13)
            ww = ww - eta * gk
        np.testing.assert_allclose(wr, ww, rtol=1e-13, atol=1e-15)
        if loss != 1:
            assert lh[-1] < lh[0]


def test_matrix_has_the_intended_structure():
    N, D, rp, ci, v = _matrix(3)
    assert rp[8] - rp[7] >= 2 and ci[rp[7]] == ci[rp[7] + 1] and rp[6] == rp[5]


def test_unmodified_copy_passes(tmp_path):
    _pins(_compile(tmp_path, "clean"))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_rejected(tmp_path, name):
    lib = _compile(tmp_path, name, *MUTANTS[name])
    with pytest.raises(AssertionError):
        _pins(lib)
