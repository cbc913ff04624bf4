"""ctypes binding of libslaqglm (declared in include/slaqglm.h).

Argument marshalling only: every step of the iteration runs in the library's HIP
kernels.  PyTorch supplies device memory (tensors) and the stream handle.  There
is no fallback: if the library cannot be loaded, or no GPU is present when a
compute entry point is called, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import build as _build

GLM_LOGISTIC, GLM_HINGE, GLM_SQUARED = 0, 1, 2
GLM_OK, GLM_EINVAL, GLM_ENOSPC, GLM_EHIP, GLM_ENOTIMPL = 0, -1, -2, -3, -4

EXPORTS = (
    "glm_workspace_bytes", "glm_step", "glm_step_batched", "glm_sweep", "glm_read_probe",
    "glm_read_probe_sink_floats", "glm_profile_begin", "glm_profile_end", "glm_strerror",
    "glm_predict_batched", "glm_predict_workspace_bytes", "glm_allocate_greedy",
    "glm_sparse_workspace_bytes", "glm_step_sparse",
    "glm_kmeans_workspace_bytes", "glm_kmeans_step",
    "glm_lbfgs_workspace_bytes", "glm_lbfgs",
    "glm_step_noalloc", "glm_step_noalloc_scratch_bytes",
)
GLM_CURVE_SUBLINEAR, GLM_CURVE_LINEAR = 1, 2
GLM_STEP_CONSTANT, GLM_STEP_INV_SQRT = 0, 1


class glm_job_t(ctypes.Structure):
    """Mirror of the C struct glm_job_t."""
    _fields_ = [
        ("X", ctypes.c_void_p), ("y", ctypes.c_void_p), ("w", ctypes.c_void_p),
        ("grad", ctypes.c_void_p), ("loss_hist", ctypes.c_void_p),
        ("N", ctypes.c_int64), ("D", ctypes.c_int32), ("loss", ctypes.c_int32),
        ("lambda_", ctypes.c_float), ("step", ctypes.c_float),
        ("hist_len", ctypes.c_int64), ("hist_cap", ctypes.c_int64), ("schedule", ctypes.c_int32),
    ]


class glm_sparse_job_t(ctypes.Structure):
    """Mirror of the C struct glm_sparse_job_t."""
    _fields_ = [
        ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("row_val", ctypes.c_void_p),
        ("col_ptr", ctypes.c_void_p), ("row_idx", ctypes.c_void_p), ("col_val", ctypes.c_void_p),
        ("y", ctypes.c_void_p), ("w", ctypes.c_void_p), ("grad", ctypes.c_void_p),
        ("loss_hist", ctypes.c_void_p),
        ("N", ctypes.c_int64), ("D", ctypes.c_int64), ("nnz", ctypes.c_int64),
        ("loss", ctypes.c_int32), ("lambda_", ctypes.c_float), ("step", ctypes.c_float),
        ("hist_len", ctypes.c_int64), ("hist_cap", ctypes.c_int64), ("prepared", ctypes.c_int32),
        ("schedule", ctypes.c_int32),
    ]


class glm_kmeans_job_t(ctypes.Structure):
    """Mirror of the C struct glm_kmeans_job_t."""
    _fields_ = [
        ("X", ctypes.c_void_p), ("C", ctypes.c_void_p), ("assign", ctypes.c_void_p),
        ("counts", ctypes.c_void_p), ("loss_hist", ctypes.c_void_p),
        ("N", ctypes.c_int64), ("D", ctypes.c_int32), ("K", ctypes.c_int32),
        ("hist_len", ctypes.c_int64), ("hist_cap", ctypes.c_int64),
    ]


class glm_lbfgs_state_t(ctypes.Structure):
    """Mirror of the C struct glm_lbfgs_state_t (zero-initialised = a new run)."""
    _fields_ = [("started", ctypes.c_int32), ("memory", ctypes.c_int32), ("evals", ctypes.c_int64),
                ("f", ctypes.c_double)]


class GlmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def lib_path() -> str:
    return _build.LIB_PATH


def load():
    """Load libslaqglm.so from the package directory (building it only if it is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build_lib(force=True)
    lib = ctypes.CDLL(_build.LIB_PATH)
    jp = ctypes.POINTER(glm_job_t)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.glm_workspace_bytes.restype = ctypes.c_int
    lib.glm_workspace_bytes.argtypes = [jp, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(sz)]
    lib.glm_step.restype = ctypes.c_int
    lib.glm_step.argtypes = [jp, ctypes.c_int32, vp, sz, vp]
    lib.glm_step_noalloc.restype = ctypes.c_int
    lib.glm_step_noalloc.argtypes = [jp, ctypes.c_int32, vp]
    lib.glm_step_noalloc_scratch_bytes.restype = ctypes.c_size_t
    lib.glm_step_noalloc_scratch_bytes.argtypes = []
    lib.glm_step_batched.restype = ctypes.c_int
    lib.glm_step_batched.argtypes = [jp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), vp, sz, vp]
    lib.glm_sweep.restype = ctypes.c_int
    lib.glm_sweep.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                              vp, vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float),
                              ctypes.c_int32, vp, vp, sz, vp]
    lib.glm_read_probe.restype = ctypes.c_int
    lib.glm_read_probe.argtypes = [vp, sz, vp, vp]
    lib.glm_read_probe_sink_floats.restype = ctypes.c_int32
    lib.glm_read_probe_sink_floats.argtypes = []
    lib.glm_profile_begin.restype = ctypes.c_int
    lib.glm_profile_begin.argtypes = [ctypes.c_int32]
    lib.glm_profile_end.restype = ctypes.c_int
    lib.glm_profile_end.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32)]
    dbl = ctypes.POINTER(ctypes.c_double)
    i32 = ctypes.POINTER(ctypes.c_int32)
    lib.glm_predict_batched.restype = ctypes.c_int
    lib.glm_predict_batched.argtypes = [jp, ctypes.c_int32, i32, ctypes.c_double, ctypes.c_int32,
                                        ctypes.c_int32, vp, vp, vp, vp, sz, vp]
    lib.glm_predict_workspace_bytes.restype = ctypes.c_int
    lib.glm_predict_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.POINTER(sz)]
    lib.glm_allocate_greedy.restype = ctypes.c_int
    lib.glm_allocate_greedy.argtypes = [dbl, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, i32]
    sjp = ctypes.POINTER(glm_sparse_job_t)
    lib.glm_sparse_workspace_bytes.restype = ctypes.c_int
    lib.glm_sparse_workspace_bytes.argtypes = [sjp, ctypes.POINTER(sz)]
    lib.glm_step_sparse.restype = ctypes.c_int
    lib.glm_step_sparse.argtypes = [sjp, ctypes.c_int32, vp, sz, vp]
    lib.glm_lbfgs_workspace_bytes.restype = ctypes.c_int
    lib.glm_lbfgs_workspace_bytes.argtypes = [ctypes.POINTER(glm_job_t), ctypes.c_int32, ctypes.POINTER(sz)]
    lib.glm_lbfgs.restype = ctypes.c_int
    lib.glm_lbfgs.argtypes = [ctypes.POINTER(glm_job_t), ctypes.POINTER(glm_lbfgs_state_t), ctypes.c_int32,
                              ctypes.c_int32, vp, sz, vp]
    kjp = ctypes.POINTER(glm_kmeans_job_t)
    lib.glm_kmeans_workspace_bytes.restype = ctypes.c_int
    lib.glm_kmeans_workspace_bytes.argtypes = [kjp, ctypes.POINTER(sz)]
    lib.glm_kmeans_step.restype = ctypes.c_int
    lib.glm_kmeans_step.argtypes = [kjp, ctypes.c_int32, vp, sz, vp]
    lib.glm_strerror.restype = ctypes.c_char_p
    lib.glm_strerror.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().glm_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != GLM_OK:
        raise GlmError(status, where)


def _stream_handle(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(int(stream.cuda_stream))


def _require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("libslaqglm needs a GPU: torch.cuda.is_available() is False")


class Job:
    """A glm_job_t plus the tensors its pointers refer to (kept alive here)."""

    def __init__(self, X: torch.Tensor, y: torch.Tensor, w: torch.Tensor, loss: int, lam: float,
                 step: float, hist_cap: int, grad: Optional[torch.Tensor] = None,
                 loss_hist: Optional[torch.Tensor] = None, schedule: int = 0):
        for t, name in ((X, "X"), (y, "y"), (w, "w")):
            if t.dtype != torch.float32 or not t.is_contiguous():
                raise TypeError(f"{name} must be a contiguous float32 tensor")
        if X.dim() != 2 or y.shape != (X.shape[0],) or w.shape != (X.shape[1],):
            raise ValueError("expected X [N, D], y [N], w [D]")
        dev = X.device
        self.X, self.y, self.w = X, y, w
        self.grad = grad if grad is not None else torch.zeros(X.shape[1], dtype=torch.float32, device=dev)
        self.loss_hist = (loss_hist if loss_hist is not None
                          else torch.zeros(max(int(hist_cap), 1), dtype=torch.float32, device=dev))
        self.c = glm_job_t(X.data_ptr(), y.data_ptr(), w.data_ptr(), self.grad.data_ptr(),
                           self.loss_hist.data_ptr(), int(X.shape[0]), int(X.shape[1]), int(loss),
                           float(lam), float(step), 0, int(hist_cap), int(schedule))

    @property
    def hist_len(self) -> int:
        return int(self.c.hist_len)

    def history(self) -> torch.Tensor:
        """The loss values appended so far (device tensor view; synchronise before reading)."""
        return self.loss_hist[: self.hist_len]


def _as_array(jobs: Sequence[Job]):
    arr = (glm_job_t * len(jobs))()
    for i, j in enumerate(jobs):
        arr[i] = j.c
    return arr


def _copy_back(arr, jobs: Sequence[Job]):
    for i, j in enumerate(jobs):
        j.c.hist_len = arr[i].hist_len


def glm_workspace_bytes(jobs: Sequence[Job], M_sweep: int = 0) -> int:
    out = ctypes.c_size_t(0)
    arr = _as_array(jobs)
    _check(load().glm_workspace_bytes(arr, len(jobs), int(M_sweep), ctypes.byref(out)),
           "glm_workspace_bytes")
    return int(out.value)


def alloc_workspace(jobs: Sequence[Job], M_sweep: int = 0) -> torch.Tensor:
    """A uint8 device tensor of the size glm_workspace_bytes reports (torch allocations are
    at least 256-byte aligned)."""
    n = glm_workspace_bytes(jobs, M_sweep)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=jobs[0].X.device)


def sweep_workspace_bytes(N: int, D: int, M: int) -> int:
    """glm_workspace_bytes for a sweep of M models over an [N, D] matrix."""
    shape = glm_job_t()
    shape.N, shape.D = int(N), int(D)
    out = ctypes.c_size_t(0)
    _check(load().glm_workspace_bytes(ctypes.byref(shape), 1, int(M), ctypes.byref(out)),
           "glm_workspace_bytes")
    return int(out.value)


def alloc_sweep_workspace(X: torch.Tensor, M: int) -> torch.Tensor:
    n = sweep_workspace_bytes(int(X.shape[0]), int(X.shape[1]), M)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=X.device)


def glm_step(job: Job, iters: int, ws: torch.Tensor, stream=None) -> None:
    _require_gpu()
    _check(load().glm_step(ctypes.byref(job.c), int(iters), ctypes.c_void_p(ws.data_ptr()),
                           ws.numel() * ws.element_size(), _stream_handle(stream)), "glm_step")


def glm_step_noalloc(job: Job, iters: int, stream=None) -> None:
    """glm_step on the library's own device-resident scratch (no workspace argument)."""
    _require_gpu()
    _check(load().glm_step_noalloc(ctypes.byref(job.c), int(iters), _stream_handle(stream)), "glm_step_noalloc")


def glm_step_noalloc_scratch_bytes() -> int:
    return int(load().glm_step_noalloc_scratch_bytes())


def glm_step_batched(jobs: Sequence[Job], alloc, ws: torch.Tensor, stream=None) -> None:
    _require_gpu()
    a = np.ascontiguousarray(np.asarray(alloc, dtype=np.int32))
    if a.shape != (len(jobs),):
        raise ValueError("alloc must have one entry per job")
    arr = _as_array(jobs)
    rc = load().glm_step_batched(arr, len(jobs), a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size(),
                                 _stream_handle(stream))
    _check(rc, "glm_step_batched")
    _copy_back(arr, jobs)


def glm_sweep(X: torch.Tensor, y: torch.Tensor, loss: int, W: torch.Tensor, G: torch.Tensor,
              lambdas, steps, iters: int, loss_hist: torch.Tensor, ws: torch.Tensor,
              stream=None) -> None:
    _require_gpu()
    M, D = int(W.shape[0]), int(W.shape[1])
    lam = np.ascontiguousarray(np.asarray(lambdas, dtype=np.float32))
    eta = np.ascontiguousarray(np.asarray(steps, dtype=np.float32))
    if lam.shape != (M,) or eta.shape != (M,):
        raise ValueError("lambdas and steps must have M entries")
    fp = ctypes.POINTER(ctypes.c_float)
    rc = load().glm_sweep(ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(y.data_ptr()),
                          int(X.shape[0]), D, M, int(loss), ctypes.c_void_p(W.data_ptr()),
                          ctypes.c_void_p(G.data_ptr()), lam.ctypes.data_as(fp), eta.ctypes.data_as(fp),
                          int(iters), ctypes.c_void_p(loss_hist.data_ptr()),
                          ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size(),
                          _stream_handle(stream))
    _check(rc, "glm_sweep")


class SparseJob:
    """A glm_sparse_job_t plus the tensors it points at."""

    def __init__(self, row_ptr, col_idx, row_val, col_ptr, row_idx, col_val, y, w, loss: int, lam: float,
                 step: float, hist_cap: int, schedule: int = 0):
        """col_ptr, row_idx and col_val may all be None: the library then builds the column layout itself."""
        csr_only = col_ptr is None and row_idx is None and col_val is None
        if not csr_only and (col_ptr is None or row_idx is None or col_val is None):
            raise ValueError("give the whole column layout or none of it")
        checks = [(row_ptr, torch.int64), (col_idx, torch.int32), (row_val, torch.float32), (y, torch.float32),
                  (w, torch.float32)]
        if not csr_only:
            checks += [(col_ptr, torch.int64), (row_idx, torch.int32), (col_val, torch.float32)]
        for t, dt in checks:
            if t.dtype != dt or not t.is_contiguous():
                raise TypeError("sparse job tensors must be contiguous int64 / int32 / float32 as declared")
        N, D, nnz = int(y.shape[0]), int(w.shape[0]), int(col_idx.shape[0])
        if row_ptr.shape != (N + 1,) or row_val.shape != (nnz,):
            raise ValueError("inconsistent sparse array shapes")
        if not csr_only and (col_ptr.shape != (D + 1,) or row_idx.shape != (nnz,) or col_val.shape != (nnz,)):
            raise ValueError("inconsistent sparse array shapes")
        dev = y.device
        self.tensors = (row_ptr, col_idx, row_val, col_ptr, row_idx, col_val, y)
        self.w = w
        self.grad = torch.zeros(D, dtype=torch.float32, device=dev)
        self.loss_hist = torch.zeros(max(int(hist_cap), 1), dtype=torch.float32, device=dev)
        ptr = lambda t: None if t is None else t.data_ptr()
        self.c = glm_sparse_job_t(row_ptr.data_ptr(), col_idx.data_ptr(), row_val.data_ptr(),
                                  ptr(col_ptr), ptr(row_idx), ptr(col_val), y.data_ptr(),
                                  w.data_ptr(), self.grad.data_ptr(), self.loss_hist.data_ptr(), N, D, nnz,
                                  int(loss), float(lam), float(step), 0, int(hist_cap), 0, int(schedule))

    @property
    def hist_len(self) -> int:
        return int(self.c.hist_len)

    def history(self) -> torch.Tensor:
        return self.loss_hist[: self.hist_len]


def glm_sparse_workspace_bytes(job: SparseJob) -> int:
    out = ctypes.c_size_t(0)
    _check(load().glm_sparse_workspace_bytes(ctypes.byref(job.c), ctypes.byref(out)), "glm_sparse_workspace_bytes")
    return int(out.value)


def alloc_sparse_workspace(job: SparseJob) -> torch.Tensor:
    return torch.empty(max(glm_sparse_workspace_bytes(job), 256), dtype=torch.uint8, device=job.w.device)


def glm_step_sparse(job: SparseJob, iters: int, ws: torch.Tensor, stream=None) -> None:
    _require_gpu()
    _check(load().glm_step_sparse(ctypes.byref(job.c), int(iters), ctypes.c_void_p(ws.data_ptr()), ws.numel(),
                                  _stream_handle(stream)), "glm_step_sparse")


class KMeansJob:
    """A glm_kmeans_job_t plus the tensors it points at."""

    def __init__(self, X: torch.Tensor, C: torch.Tensor, hist_cap: int):
        for t in (X, C):
            if t.dtype != torch.float32 or not t.is_contiguous() or t.dim() != 2:
                raise TypeError("X and C must be contiguous 2-D float32 tensors")
        if X.shape[1] != C.shape[1]:
            raise ValueError("X and C differ in the number of columns")
        N, D, K = int(X.shape[0]), int(X.shape[1]), int(C.shape[0])
        dev = X.device
        self.X, self.C = X, C
        self.assign = torch.zeros(N, dtype=torch.int32, device=dev)
        self.counts = torch.zeros(K, dtype=torch.int32, device=dev)
        self.loss_hist = torch.zeros(max(int(hist_cap), 1), dtype=torch.float32, device=dev)
        self.c = glm_kmeans_job_t(X.data_ptr(), C.data_ptr(), self.assign.data_ptr(), self.counts.data_ptr(),
                                  self.loss_hist.data_ptr(), N, D, K, 0, int(hist_cap))

    @property
    def hist_len(self) -> int:
        return int(self.c.hist_len)

    def history(self) -> torch.Tensor:
        return self.loss_hist[: self.hist_len]


def glm_kmeans_workspace_bytes(job: KMeansJob) -> int:
    out = ctypes.c_size_t(0)
    _check(load().glm_kmeans_workspace_bytes(ctypes.byref(job.c), ctypes.byref(out)), "glm_kmeans_workspace_bytes")
    return int(out.value)


def alloc_kmeans_workspace(job: KMeansJob) -> torch.Tensor:
    return torch.empty(max(glm_kmeans_workspace_bytes(job), 256), dtype=torch.uint8, device=job.X.device)


def glm_kmeans_step(job: KMeansJob, iters: int, ws: torch.Tensor, stream=None) -> None:
    _require_gpu()
    _check(load().glm_kmeans_step(ctypes.byref(job.c), int(iters), ctypes.c_void_p(ws.data_ptr()), ws.numel(),
                                  _stream_handle(stream)), "glm_kmeans_step")


def glm_lbfgs_workspace_bytes(job: Job, memory: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().glm_lbfgs_workspace_bytes(ctypes.byref(job.c), int(memory), ctypes.byref(out)),
           "glm_lbfgs_workspace_bytes")
    return int(out.value)


def alloc_lbfgs_workspace(job: Job, memory: int) -> torch.Tensor:
    return torch.empty(max(glm_lbfgs_workspace_bytes(job, memory), 256), dtype=torch.uint8, device=job.w.device)


def glm_lbfgs(job: Job, state: glm_lbfgs_state_t, iters: int, memory: int, ws: torch.Tensor, stream=None) -> None:
    _require_gpu()
    _check(load().glm_lbfgs(ctypes.byref(job.c), ctypes.byref(state), int(iters), int(memory),
                            ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream_handle(stream)), "glm_lbfgs")


class HistoryView:
    """The loss history of any job (dense, sparse or K-Means) in the shape the predictor reads:
    a glm_job_t of which only loss_hist and hist_len are set."""

    def __init__(self, job):
        self.job = job
        self.c = glm_job_t()
        self.c.loss_hist = job.loss_hist.data_ptr()
        self.c.hist_len = int(job.c.hist_len)


def glm_predict_batched(jobs: Sequence[Job], curve, gamma: float, window: int, horizon: int,
                        pred: torch.Tensor, gain: torch.Tensor, fit: torch.Tensor,
                        ws: Optional[torch.Tensor] = None, stream=None) -> None:
    """pred, gain: float64 device tensors [J, horizon]; fit: float64 device tensor [J, 8]."""
    _require_gpu()
    J = len(jobs)
    cv = np.ascontiguousarray(np.broadcast_to(np.asarray(curve, dtype=np.int32), (J,)))
    for t, shape in ((pred, (J, horizon)), (gain, (J, horizon)), (fit, (J, 8))):
        if t.dtype != torch.float64 or tuple(t.shape) != shape or not t.is_contiguous():
            raise TypeError("pred/gain/fit must be contiguous float64 tensors of shape [J, horizon] / [J, 8]")
    if ws is None:
        need = ctypes.c_size_t(0)
        _check(load().glm_predict_workspace_bytes(J, ctypes.byref(need)), "glm_predict_workspace_bytes")
        ws = torch.empty(max(int(need.value), 256), dtype=torch.uint8, device=pred.device)
    arr = _as_array(jobs)
    rc = load().glm_predict_batched(arr, J, cv.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), float(gamma),
                                    int(window), int(horizon), ctypes.c_void_p(pred.data_ptr()),
                                    ctypes.c_void_p(gain.data_ptr()), ctypes.c_void_p(fit.data_ptr()),
                                    ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream_handle(stream))
    _check(rc, "glm_predict_batched")


def glm_allocate_greedy(gain, capacity: int) -> np.ndarray:
    """gain: host array [J, H] (float64).  Returns the int32 allocation vector [J]."""
    g = np.ascontiguousarray(np.asarray(gain, dtype=np.float64))
    if g.ndim != 2:
        raise ValueError("gain must be [J, H]")
    J, H = g.shape
    alloc = np.zeros(J, dtype=np.int32)
    rc = load().glm_allocate_greedy(g.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), J, H, int(capacity),
                                    alloc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "glm_allocate_greedy")
    return alloc


def glm_read_probe(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    _require_gpu()
    _check(load().glm_read_probe(ctypes.c_void_p(src.data_ptr()), src.numel(),
                                 ctypes.c_void_p(sink.data_ptr()), _stream_handle(stream)),
           "glm_read_probe")


def glm_read_probe_sink_floats() -> int:
    return int(load().glm_read_probe_sink_floats())


def glm_profile_begin(cap: int) -> None:
    _check(load().glm_profile_begin(int(cap)), "glm_profile_begin")


def glm_profile_end(cap: int) -> List[float]:
    ms = (ctypes.c_float * int(cap))()
    n = ctypes.c_int32(0)
    _check(load().glm_profile_end(ms, ctypes.byref(n)), "glm_profile_end")
    return [float(ms[i]) for i in range(n.value)]
