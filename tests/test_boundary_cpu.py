"""CPU tests of the C-ABI boundary: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

from paper_1802_04819_amd import glm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "slaqglm.h")


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(glm_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = glm.load()
    names = _declared_functions()
    assert set(names) == set(glm.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_strerror_texts():
    assert glm.strerror(glm.GLM_OK) == "ok"
    for s in (glm.GLM_EINVAL, glm.GLM_ENOSPC, glm.GLM_EHIP, glm.GLM_ENOTIMPL, 12345):
        assert isinstance(glm.strerror(s), str) and glm.strerror(s)


def _job(**kw):
    # fake but well-formed device addresses: validation must reject before dereferencing
    f = dict(X=0x10000, y=0x20000, w=0x30000, grad=0x40000, loss_hist=0x50000, N=1000, D=64,
             loss=0, lambda_=1e-3, step=0.1, hist_len=0, hist_cap=10, schedule=0)
    f.update(kw)
    return glm.glm_job_t(f["X"], f["y"], f["w"], f["grad"], f["loss_hist"], f["N"], f["D"],
                         f["loss"], f["lambda_"], f["step"], f["hist_len"], f["hist_cap"], f["schedule"])


def _ws_bytes(job, J=1, M=0):
    out = ctypes.c_size_t(0)
    rc = glm.load().glm_workspace_bytes(ctypes.byref(job), J, M, ctypes.byref(out))
    return rc, out.value


def test_workspace_bytes_depends_on_shape_only():
    rc, a = _ws_bytes(_job())
    assert rc == glm.GLM_OK and a > 0 and a % 256 == 0
    rc, b = _ws_bytes(_job(N=10**6, D=1024))
    assert rc == glm.GLM_OK and b > a
    rc, c = _ws_bytes(_job(loss=2, lambda_=5.0, X=0))      # only N and D are read
    assert rc == glm.GLM_OK and c == a


def test_sweep_workspace_bytes_with_and_without_a_residual_area():
    """A sweep of at most 16 models on rows the one-pass kernel takes (a multiple of 16 floats, at most
    1024) keeps no residuals [N, 64]; every other sweep does, and its areas for the partial sums also
    hold those of a small last group."""
    N, D = 100000, 512
    rc, small = _ws_bytes(_job(N=N, D=D), M=16)
    rc2, big = _ws_bytes(_job(N=N, D=D), M=17)
    assert rc == glm.GLM_OK and rc2 == glm.GLM_OK
    assert big - small >= 4 * N * 64 and small < 4 * N * 64
    # the one-pass kernel's partial gradients: one [16, D] per block, 512 blocks at this row length
    assert small >= 4 * 512 * 16 * D
    # rows the one-pass kernel does not take: the residual area is there whatever the number of models
    for Dx in (520, 2048):
        rc, a = _ws_bytes(_job(N=N, D=Dx), M=16)
        assert rc == glm.GLM_OK and a >= 4 * N * 64
    # tiny N: one block per tile of 16 rows, never fewer bytes than the two-pass areas need
    rc, t1 = _ws_bytes(_job(N=5, D=64), M=3)
    rc2, t2 = _ws_bytes(_job(N=5, D=64), M=64)
    assert rc == glm.GLM_OK and rc2 == glm.GLM_OK and 0 < t1 <= t2


@pytest.mark.parametrize("bad", [dict(N=0), dict(D=0), dict(D=6), dict(D=4100), dict(N=-5)])
def test_workspace_bytes_rejects_bad_shapes(bad):
    rc, _ = _ws_bytes(_job(**bad))
    assert rc == glm.GLM_EINVAL


def test_workspace_bytes_rejects_null_and_counts():
    out = ctypes.c_size_t(0)
    lib = glm.load()
    assert lib.glm_workspace_bytes(None, 1, 0, ctypes.byref(out)) == glm.GLM_EINVAL
    j = _job()
    assert lib.glm_workspace_bytes(ctypes.byref(j), 0, 0, ctypes.byref(out)) == glm.GLM_EINVAL
    assert lib.glm_workspace_bytes(ctypes.byref(j), 1, 0, None) == glm.GLM_EINVAL
    assert lib.glm_workspace_bytes(ctypes.byref(j), 1, -1, ctypes.byref(out)) == glm.GLM_EINVAL


_BAD_JOBS = [
    dict(X=0), dict(y=0), dict(w=0), dict(grad=0), dict(loss_hist=0),
    dict(X=0x10004), dict(w=0x30008), dict(y=0x20002),
    dict(N=0), dict(D=2), dict(D=130), dict(D=8192),
    dict(loss=3), dict(loss=-1),
    dict(lambda_=-1.0), dict(lambda_=float("nan")), dict(lambda_=float("inf")),
    dict(step=-0.1), dict(step=float("nan")),
    dict(hist_len=-1), dict(hist_len=11, hist_cap=10),
    dict(schedule=2), dict(schedule=-1),
]


@pytest.mark.parametrize("bad", _BAD_JOBS)
def test_step_rejects_invalid_jobs_without_side_effects(bad):
    j = _job(**bad)
    before = bytes(j)
    rc = glm.load().glm_step(ctypes.byref(j), 1, ctypes.c_void_p(0x100000), 1 << 30, None)
    assert rc == glm.GLM_EINVAL
    assert bytes(j) == before


def test_step_rejects_negative_iters_history_overflow_and_small_workspace():
    lib = glm.load()
    j = _job()
    assert lib.glm_step(ctypes.byref(j), -1, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_EINVAL
    assert lib.glm_step(None, 1, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_EINVAL
    j = _job(hist_len=8, hist_cap=10)
    assert lib.glm_step(ctypes.byref(j), 3, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_ENOSPC
    assert j.hist_len == 8
    j = _job()
    _, need = _ws_bytes(j)
    assert lib.glm_step(ctypes.byref(j), 1, ctypes.c_void_p(0x100000), need - 1, None) == glm.GLM_ENOSPC
    assert lib.glm_step(ctypes.byref(j), 1, None, need, None) == glm.GLM_EINVAL
    assert lib.glm_step(ctypes.byref(j), 1, ctypes.c_void_p(0x100010), need, None) == glm.GLM_EINVAL
    assert j.hist_len == 0


def test_batched_validates_every_job_before_enqueueing():
    lib = glm.load()
    arr = (glm.glm_job_t * 3)(_job(), _job(D=128), _job(loss=9))
    alloc = (ctypes.c_int32 * 3)(1, 2, 1)
    assert lib.glm_step_batched(arr, 3, alloc, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_EINVAL
    arr = (glm.glm_job_t * 3)(_job(), _job(D=128), _job(hist_len=10))
    assert lib.glm_step_batched(arr, 3, alloc, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_ENOSPC
    alloc = (ctypes.c_int32 * 3)(1, -2, 0)
    assert lib.glm_step_batched(arr, 3, alloc, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_EINVAL
    assert all(arr[i].hist_len == (10 if i == 2 else 0) for i in range(3))
    assert lib.glm_step_batched(arr, 0, alloc, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_EINVAL
    assert lib.glm_step_batched(arr, 3, None, ctypes.c_void_p(0x100000), 1 << 30, None) == glm.GLM_EINVAL


def test_python_binding_refuses_to_run_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    X = torch.zeros(8, 4); y = torch.zeros(8); w = torch.zeros(4)
    job = glm.Job(X, y, w, glm.GLM_SQUARED, 0.0, 0.1, 4)
    ws = torch.zeros(4096, dtype=torch.uint8)
    with pytest.raises(RuntimeError):
        glm.glm_step(job, 1, ws)


def test_probe_and_profile_argument_checks():
    lib = glm.load()
    assert lib.glm_read_probe(None, 1024, ctypes.c_void_p(0x1000), None) == glm.GLM_EINVAL
    assert lib.glm_read_probe(ctypes.c_void_p(0x1000), 1022, ctypes.c_void_p(0x1000), None) == glm.GLM_EINVAL
    assert lib.glm_read_probe_sink_floats() > 0
    assert lib.glm_profile_begin(0) == glm.GLM_EINVAL
    n = ctypes.c_int32(0)
    ms = (ctypes.c_float * 4)()
    assert lib.glm_profile_end(ms, ctypes.byref(n)) == glm.GLM_EINVAL     # not recording


def test_header_is_c_and_the_c_consumer_links():
    """gcc -std=c99 -Wall -Wextra -Werror accepts the header and links a C program against the
    library (the program itself runs in the GPU suite)."""
    from paper_1802_04819_amd import build as b
    path = b.build_c_demo()
    assert os.path.exists(path) and os.access(path, os.X_OK)


def _sparse_ws(N, D, nnz, csr_only=False):
    a = 0x10000
    j = glm.glm_sparse_job_t(a, a, a, 0 if csr_only else a, 0 if csr_only else a, 0 if csr_only else a, a, a, a, a,
                             N, D, nnz, 0, 1e-3, 0.1, 0, 4, 0, 0)
    out = ctypes.c_size_t(0)
    rc = glm.load().glm_sparse_workspace_bytes(ctypes.byref(j), ctypes.byref(out))
    return rc, out.value


def test_sparse_workspace_bytes_over_the_limits_of_the_scatter_path():
    """The size is a function of (N, D, nnz, CSR alone or not); it stays sane on both sides of every
    limit of the scatter path (4,194,304 entries, 1024 panels of outputs, 64 windows of the other
    vector, enough entries per panel and window) and does not shrink when the number of entries grows."""
    shapes = [(1000, 500, 0), (1000, 500, 10_000), (300_000, 200_000, (1 << 22) - 1), (300_000, 200_000, 1 << 22),
              (16_777_216, 300, 20_000_000), (16_777_217, 300, 20_000_000),          # 1024 / 1025 panels, 64 / 65 windows
              (2_000_000, 1_000_000, 199_821_056), (4_194_304, 4_194_304, 5_000_000),  # too few entries per panel and window
              (50_000_000, 100_000, 400_000_000)]
    for N, D, nnz in shapes:
        rc, b = _sparse_ws(N, D, nnz)
        assert rc == glm.GLM_OK and b % 256 == 0, (N, D, nnz)
        assert b < 64 * max(nnz, 1) + 64 * (N + D) + (1 << 30), (N, D, nnz, b)       # a few copies of the matrix at most
        rc2, b2 = _sparse_ws(N, D, nnz, csr_only=True)
        assert rc2 == glm.GLM_OK and b2 >= b
        if nnz > 0:
            rc3, b3 = _sparse_ws(N, D, 2 * nnz)
            assert rc3 == glm.GLM_OK and b3 >= b
    assert _sparse_ws(0, 5, 0)[0] == glm.GLM_EINVAL and _sparse_ws(5, 0, 0)[0] == glm.GLM_EINVAL
    assert _sparse_ws(5, 5, -1)[0] == glm.GLM_EINVAL
