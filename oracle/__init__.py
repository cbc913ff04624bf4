"""fp64 CPU oracle for the GLM full-batch iteration and the K-Means iteration (TEST INFRASTRUCTURE).

Thin ctypes wrapper over ``glm_oracle.c`` and ``kmeans_oracle.c``.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the GPU library never
does.  Nothing here depends on the GPU package, and the GPU package does not
depend on anything here.

The paper prints no formula or value for a training iteration (it only states,
Sec. 2 "Normalizing Quality Metrics", that the loss is evaluated every
iteration, and lists the algorithms in Sec. 3 "Setup"), so against paper-printed
values every function here is "parity unpinned"; the CPU tests pin them with
closed forms, finite differences, the normal equations and convexity
invariants instead.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

LOGISTIC, HINGE, SQUARED = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "glm_oracle.c")
_SRCS = [_SRC, os.path.join(_HERE, "kmeans_oracle.c"), os.path.join(_HERE, "sched_fit.c")]
_LIB_PATH = os.path.join(_HERE, "libglm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C sources here with gcc (OpenMP on) into libglm_oracle.so beside them."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < max(os.path.getmtime(f) for f in _SRCS):
        tmp = _LIB_PATH + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", tmp] + _SRCS + ["-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_loss_grad.restype = ctypes.c_int
        lib.oracle_loss_grad.argtypes = [ctypes.c_int, fp, fp, ctypes.c_int64, ctypes.c_int32,
                                         dp, ctypes.c_double, dp, dp]
        lib.oracle_loss_grad_chunked.restype = ctypes.c_int
        lib.oracle_loss_grad_chunked.argtypes = [ctypes.c_int, fp, fp, ctypes.c_int64, ctypes.c_int32,
                                                 dp, ctypes.c_double, ctypes.c_int32, dp, dp]
        lib.oracle_run.restype = ctypes.c_int
        lib.oracle_run.argtypes = [ctypes.c_int, fp, fp, ctypes.c_int64, ctypes.c_int32,
                                   dp, ctypes.c_double, ctypes.c_double, ctypes.c_int32,
                                   ctypes.c_int32, dp, dp, dp]
        lib.oracle_run_schedule.restype = ctypes.c_int
        lib.oracle_run_schedule.argtypes = [ctypes.c_int, fp, fp, ctypes.c_int64, ctypes.c_int32,
                                            dp, ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_int64,
                                            ctypes.c_int32, dp, dp, dp]
        i64p = ctypes.POINTER(ctypes.c_int64)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_sparse_loss_grad.restype = ctypes.c_int
        lib.oracle_sparse_loss_grad.argtypes = [ctypes.c_int, i64p, i32p, fp, fp, ctypes.c_int64,
                                                ctypes.c_int64, dp, ctypes.c_double, dp, dp]
        lib.oracle_sparse_run.restype = ctypes.c_int
        lib.oracle_sparse_run.argtypes = [ctypes.c_int, i64p, i32p, fp, fp, ctypes.c_int64, ctypes.c_int64,
                                          dp, ctypes.c_double, ctypes.c_double, ctypes.c_int32, dp, dp, dp]
        lib.oracle_sparse_run_schedule.restype = ctypes.c_int
        lib.oracle_sparse_run_schedule.argtypes = [ctypes.c_int, i64p, i32p, fp, fp, ctypes.c_int64, ctypes.c_int64,
                                                   dp, ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_int64,
                                                   ctypes.c_int32, dp, dp, dp]
        lib.oracle_kmeans_assign.restype = ctypes.c_int
        lib.oracle_kmeans_assign.argtypes = [fp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_int32, i32p, dp, dp]
        lib.oracle_kmeans_step.restype = ctypes.c_int
        lib.oracle_kmeans_step.argtypes = [fp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_int32, i32p, i64p, dp]
        lib.oracle_fit_curve.restype = ctypes.c_int
        lib.oracle_fit_curve.argtypes = [ctypes.c_int, dp, ctypes.c_int, ctypes.c_double, dp]
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_max_threads.argtypes = []
        _lib = lib
    return _lib


def fit_curve_raw(cls: int, L, gamma: float, lib=None):
    """The convergence-curve fit of sched_fit.c on the window L (fp64, 4..128 values):
    (ok, offset, p0, p1, p2, E, e).  `lib` lets a test run a separately compiled copy."""
    L = np.ascontiguousarray(np.asarray(L, dtype=np.float64))
    out = np.zeros(7, dtype=np.float64)
    (lib or _load()).oracle_fit_curve(int(cls), L.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), int(L.shape[0]),
                                     float(gamma), out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _f32(a, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs X and y must be float32 (the bits the GPU reads)")
    if shape is not None and a.shape != shape:
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _fptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def loss_grad(loss: int, X, y, w, lam: float, chunks: int = 0):
    """(L, g) at w: L = mean_i l_i + lam/2 |w|^2, g = X^T r / N + lam w, all in fp64.

    ``chunks`` > 1 evaluates contiguous row chunks independently (OpenMP) and
    adds them in chunk order; 0/1 is the strictly sequential evaluation.
    """
    X = _f32(X)
    N, D = X.shape
    y = _f32(y, (N,))
    w = np.ascontiguousarray(np.asarray(w, dtype=np.float64))
    if w.shape != (D,):
        raise ValueError("w must have shape (D,)")
    g = np.empty(D, dtype=np.float64)
    L = ctypes.c_double(0.0)
    lib = _load()
    if chunks and chunks > 1:
        rc = lib.oracle_loss_grad_chunked(int(loss), _fptr(X), _fptr(y), N, D, _dptr(w),
                                          float(lam), int(chunks), ctypes.byref(L), _dptr(g))
    else:
        rc = lib.oracle_loss_grad(int(loss), _fptr(X), _fptr(y), N, D, _dptr(w), float(lam),
                                  ctypes.byref(L), _dptr(g))
    if rc != 0:
        raise ValueError("oracle_loss_grad rejected its arguments")
    return float(L.value), g


def run(loss: int, X, y, w0, lam: float, eta: float, K: int, chunks: int = 0):
    """K constant-step GD iterations from w0.

    Returns (loss_hist[K], gnorm_hist[K], w_K, g_last); entry k of the histories
    belongs to the iterate entering iteration k.
    """
    X = _f32(X)
    N, D = X.shape
    y = _f32(y, (N,))
    w = np.array(w0, dtype=np.float64, copy=True)
    if w.shape != (D,):
        raise ValueError("w0 must have shape (D,)")
    lh = np.empty(K, dtype=np.float64)
    gh = np.empty(K, dtype=np.float64)
    gl = np.zeros(D, dtype=np.float64)
    rc = _load().oracle_run(int(loss), _fptr(X), _fptr(y), N, D, _dptr(w), float(lam), float(eta),
                            int(K), int(chunks), _dptr(lh), _dptr(gh), _dptr(gl))
    if rc != 0:
        raise ValueError("oracle_run rejected its arguments")
    return lh, gh, w, gl


CONSTANT, INV_SQRT = 0, 1


def run_schedule(loss: int, X, y, w0, lam: float, eta: float, schedule: int, K: int, k0: int = 0):
    """K gradient-descent iterations from w0 with the step of iteration k (counted from the job's
    start, k0 + position in this call) given by the schedule: CONSTANT eta, INV_SQRT
    eta / sqrt(k + 1).  Returns as run()."""
    X = _f32(X)
    N, D = X.shape
    y = _f32(y, (N,))
    w = np.array(w0, dtype=np.float64, copy=True)
    if w.shape != (D,):
        raise ValueError("w0 must have shape (D,)")
    lh = np.empty(K, dtype=np.float64)
    gh = np.empty(K, dtype=np.float64)
    gl = np.zeros(D, dtype=np.float64)
    rc = _load().oracle_run_schedule(int(loss), _fptr(X), _fptr(y), N, D, _dptr(w), float(lam), float(eta),
                                     int(schedule), int(k0), int(K), _dptr(lh), _dptr(gh), _dptr(gl))
    if rc != 0:
        raise ValueError("oracle_run_schedule rejected its arguments")
    return lh, gh, w, gl


def _csr(row_ptr, col_idx, val, N, D):
    rp = np.ascontiguousarray(row_ptr, dtype=np.int64)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    v = np.ascontiguousarray(val)
    if v.dtype != np.float32:
        raise TypeError("CSR values must be float32 (the bits the GPU reads)")
    if rp.shape != (N + 1,) or rp[0] != 0 or rp[-1] != len(ci) or len(ci) != len(v) or np.any(np.diff(rp) < 0):
        raise ValueError("inconsistent CSR arrays")
    if len(ci) and (ci.min() < 0 or ci.max() >= D):
        raise ValueError("column index out of range")
    return rp, ci, v


def sparse_loss_grad(loss: int, row_ptr, col_idx, val, y, D: int, w, lam: float):
    """(L, g) at w for X given in CSR form (row_ptr [N+1] int64, col_idx int32, val float32)."""
    y = _f32(y)
    N = y.shape[0]
    rp, ci, v = _csr(row_ptr, col_idx, val, N, D)
    w = np.ascontiguousarray(np.asarray(w, dtype=np.float64))
    if w.shape != (D,):
        raise ValueError("w must have shape (D,)")
    g = np.empty(D, dtype=np.float64)
    L = ctypes.c_double(0.0)
    rc = _load().oracle_sparse_loss_grad(int(loss), rp.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                         ci.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _fptr(v), _fptr(y),
                                         N, D, _dptr(w), float(lam), ctypes.byref(L), _dptr(g))
    if rc != 0:
        raise ValueError("oracle_sparse_loss_grad rejected its arguments")
    return float(L.value), g


def sparse_run(loss: int, row_ptr, col_idx, val, y, D: int, w0, lam: float, eta: float, K: int):
    """K constant-step GD iterations on a CSR matrix; returns (loss_hist, gnorm_hist, w_K, g_last)."""
    y = _f32(y)
    N = y.shape[0]
    rp, ci, v = _csr(row_ptr, col_idx, val, N, D)
    w = np.array(w0, dtype=np.float64, copy=True)
    lh = np.empty(K); gh = np.empty(K); gl = np.zeros(D)
    rc = _load().oracle_sparse_run(int(loss), rp.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                   ci.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _fptr(v), _fptr(y), N, D,
                                   _dptr(w), float(lam), float(eta), int(K), _dptr(lh), _dptr(gh), _dptr(gl))
    if rc != 0:
        raise ValueError("oracle_sparse_run rejected its arguments")
    return lh, gh, w, gl


def sparse_run_schedule(loss: int, row_ptr, col_idx, val, y, D: int, w0, lam: float, eta: float, schedule: int,
                        K: int, k0: int = 0):
    """As sparse_run with the step schedule of run_schedule."""
    y = _f32(y)
    N = y.shape[0]
    rp, ci, v = _csr(row_ptr, col_idx, val, N, D)
    w = np.array(w0, dtype=np.float64, copy=True)
    lh = np.empty(K); gh = np.empty(K); gl = np.zeros(D)
    rc = _load().oracle_sparse_run_schedule(int(loss), rp.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                            ci.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _fptr(v), _fptr(y), N, D,
                                            _dptr(w), float(lam), float(eta), int(schedule), int(k0), int(K),
                                            _dptr(lh), _dptr(gh), _dptr(gl))
    if rc != 0:
        raise ValueError("oracle_sparse_run_schedule rejected its arguments")
    return lh, gh, w, gl


def run_sweep(loss: int, X, y, W0, lams: Sequence[float], etas: Sequence[float], K: int,
              chunks: int = 0):
    """M independent models sharing X: model m is ``run`` with (lams[m], etas[m]).

    W0 is [M, D].  Returns (loss_hist[K, M], gnorm_hist[K, M], W_K[M, D], G_last[M, D]).
    """
    W0 = np.asarray(W0, dtype=np.float64)
    M, D = W0.shape
    lh = np.empty((K, M)); gh = np.empty((K, M))
    WK = np.empty((M, D)); GL = np.empty((M, D))
    for m in range(M):
        a, b, c, d = run(loss, X, y, W0[m], float(lams[m]), float(etas[m]), K, chunks)
        lh[:, m], gh[:, m], WK[m], GL[m] = a, b, c, d
    return lh, gh, WK, GL


def kmeans_assign(X, C):
    """(assign [N] int32, best [N], second [N]): nearest centroid (lowest index on ties), the
    squared distance to it and to the nearest other centroid (-1 when K == 1), in fp64."""
    X = _f32(X)
    N, D = X.shape
    C = np.ascontiguousarray(np.asarray(C, dtype=np.float64))
    if C.ndim != 2 or C.shape[1] != D:
        raise ValueError("C must have shape (K, D)")
    K = C.shape[0]
    a = np.empty(N, dtype=np.int32); b = np.empty(N); s = np.empty(N)
    rc = _load().oracle_kmeans_assign(_fptr(X), N, D, _dptr(C), K, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                      _dptr(b), _dptr(s))
    if rc != 0:
        raise ValueError("oracle_kmeans_assign rejected its arguments")
    return a, b, s


def kmeans_step(X, C):
    """One Lloyd iteration from centroids C [K, D]: returns (L, C_new, assign, counts) with L the
    mean squared distance to the nearest ENTERING centroid; empty clusters keep their centroid."""
    X = _f32(X)
    N, D = X.shape
    Cn = np.array(C, dtype=np.float64, copy=True, order="C")
    if Cn.ndim != 2 or Cn.shape[1] != D:
        raise ValueError("C must have shape (K, D)")
    K = Cn.shape[0]
    a = np.empty(N, dtype=np.int32); cnt = np.empty(K, dtype=np.int64); L = ctypes.c_double(0.0)
    rc = _load().oracle_kmeans_step(_fptr(X), N, D, _dptr(Cn), K, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                    cnt.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), ctypes.byref(L))
    if rc != 0:
        raise ValueError("oracle_kmeans_step rejected its arguments")
    return float(L.value), Cn, a, cnt


def kmeans_run(X, C0, iters: int):
    """`iters` Lloyd iterations: (loss_hist [iters], C_final, assign of the last iteration, counts)."""
    C = np.array(C0, dtype=np.float64, copy=True)
    hist = np.empty(iters); a = cnt = None
    for k in range(iters):
        hist[k], C, a, cnt = kmeans_step(X, C)
    return hist, C, a, cnt
