"""GPU tests of glm_step_sparse (CSR + CSC input, chunked deterministic segmented sums)."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
from paper_1802_04819_amd import glm, synth
from _parity import REL_TOL, rel

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _job_from_problem(p, step=None, w=None, hist_cap=None, device="cuda"):
    t = lambda x: x.to(device)
    w0 = (p.w0 if w is None else w).to(device).clone()
    return glm.SparseJob(t(p.row_ptr), t(p.col_idx), t(p.row_val), t(p.col_ptr), t(p.row_idx), t(p.col_val),
                         t(p.y), w0, p.loss, p.lam, p.eta if step is None else step,
                         p.K if hist_cap is None else hist_cap)


def _job_from_scipy(A, y, loss, lam, step, hist_cap, w=None):
    """A: scipy CSR (duplicates allowed, any order).  CSC = stable sort of the entries by column."""
    A = sp.csr_matrix(A)
    N, D = A.shape
    rp = A.indptr.astype(np.int64); ci = A.indices.astype(np.int32); rv = A.data.astype(np.float32)
    rows = np.repeat(np.arange(N, dtype=np.int32), np.diff(rp))
    order = np.argsort(ci, kind="stable")
    cp = np.concatenate([[0], np.cumsum(np.bincount(ci, minlength=D))]).astype(np.int64)
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    w0 = torch.zeros(D, device="cuda") if w is None else torch.from_numpy(np.asarray(w, np.float32)).cuda()
    job = glm.SparseJob(T(rp), T(ci), T(rv), T(cp), T(rows[order]), T(rv[order]), T(np.asarray(y, np.float32)),
                        w0, loss, lam, step, hist_cap)
    return job, (rp, ci, rv)


def _check_steps(job, csr, y, D, loss, lam, eta, iters, tag):
    ws = glm.alloc_sparse_workspace(job)
    rp, ci, rv = csr
    for k in range(iters):
        w_in = job.w.cpu().numpy().astype(np.float64)
        glm.glm_step_sparse(job, 1, ws)
        torch.cuda.synchronize()
        L, g = oracle.sparse_loss_grad(loss, rp, ci, rv, np.asarray(y, np.float32), D, w_in, lam)
        Lg = job.loss_hist[k].item()
        gg = job.grad.cpu().numpy().astype(np.float64)
        assert rel(Lg, L) <= REL_TOL, (tag, k, "loss", Lg, L)
        gn = np.linalg.norm(g)
        if gn > 0:
            assert rel(np.linalg.norm(gg), gn) <= REL_TOL, (tag, k, "gnorm")
        assert np.max(np.abs(gg - g)) <= REL_TOL * max(np.max(np.abs(g)), 1e-300), (tag, k, "grad entries")
        w_ref = w_in - eta * g
        scale = max(np.max(np.abs(w_ref)), eta * np.max(np.abs(g)), 1e-30)
        assert np.max(np.abs(job.w.cpu().numpy() - w_ref)) <= REL_TOL * scale, (tag, k, "update")
    assert job.hist_len == iters


def _labels(loss, N, rng):
    if loss == synth.LOGISTIC:
        return (rng.random(N) > 0.5).astype(np.float32)
    if loss == synth.HINGE:
        return np.where(rng.random(N) > 0.5, 1.0, -1.0).astype(np.float32)
    return rng.standard_normal(N).astype(np.float32)


STRUCTURES = {
    "random 3 percent": lambda rng: sp.random(700, 300, 0.03, format="csr", random_state=1, dtype=np.float32),
    "one entry": lambda rng: sp.csr_matrix(([2.5], ([3], [1])), shape=(9, 4), dtype=np.float32),
    "empty matrix": lambda rng: sp.csr_matrix((5, 7), dtype=np.float32),
    "single row and column": lambda rng: sp.csr_matrix(np.array([[1.5]], np.float32)),
    "dense block": lambda rng: sp.csr_matrix(rng.standard_normal((70, 33)).astype(np.float32)),
    "one long column over many chunks": lambda rng: sp.csr_matrix(
        (rng.standard_normal(5000).astype(np.float32), (np.arange(5000), np.full(5000, 7))), shape=(5000, 20)),
    "one long row over many chunks": lambda rng: sp.csr_matrix(
        (rng.standard_normal(3000).astype(np.float32), (np.full(3000, 2), np.arange(3000))), shape=(6, 3000)),
    "rows of exactly one chunk": lambda rng: sp.csr_matrix(rng.standard_normal((5, 512)).astype(np.float32)),
    "mostly empty rows and columns": lambda rng: sp.random(4000, 5000, 0.0003, format="csr", random_state=2, dtype=np.float32),
    "short rows long columns": lambda rng: sp.csr_matrix(
        (rng.standard_normal(20000).astype(np.float32),
         (np.arange(20000) // 2, (rng.random(20000) ** 6 * 50).astype(int))), shape=(10000, 50)),
}


@pytest.mark.parametrize("loss", [synth.LOGISTIC, synth.HINGE, synth.SQUARED])
@pytest.mark.parametrize("name", sorted(STRUCTURES))
def test_each_step_matches_oracle_on_hand_built_structures(name, loss):
    _say(f"[case] sparse per-step parity: {name}, loss {loss}")
    rng = np.random.default_rng(5)
    A = STRUCTURES[name](rng)
    N, D = A.shape
    y = _labels(loss, N, rng)
    eta = {synth.LOGISTIC: 0.5, synth.HINGE: 0.05, synth.SQUARED: 0.02}[loss]
    job, csr = _job_from_scipy(A, y, loss, 1e-3, eta, 3)
    _check_steps(job, csr, y, D, loss, 1e-3, eta, 3, name)


def test_duplicate_entries_add():
    _say("[case] sparse: repeated (row, column) pairs add")
    rows = np.array([0, 0, 0, 1, 2, 2]); cols = np.array([1, 1, 3, 0, 2, 2])
    vals = np.array([1.0, 2.0, -1.0, 0.5, 4.0, -1.5], np.float32)
    rp = np.array([0, 3, 4, 6], np.int64)
    order = np.argsort(cols, kind="stable")
    cp = np.concatenate([[0], np.cumsum(np.bincount(cols, minlength=4))]).astype(np.int64)
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    y = np.array([1.0, 0.0, 1.0], np.float32)
    w = torch.tensor([0.3, -0.2, 0.1, 0.5], device="cuda")
    job = glm.SparseJob(T(rp), T(cols.astype(np.int32)), T(vals), T(cp), T(rows[order].astype(np.int32)),
                        T(vals[order]), T(y), w, synth.LOGISTIC, 0.1, 0.0, 1)
    glm.glm_step_sparse(job, 1, glm.alloc_sparse_workspace(job))
    torch.cuda.synchronize()
    dense = np.zeros((3, 4), np.float32)
    np.add.at(dense, (rows, cols), vals)
    L, g = oracle.loss_grad(synth.LOGISTIC, dense, y, w.cpu().numpy().astype(np.float64), 0.1)
    assert rel(job.loss_hist[0].item(), L) <= 1e-6
    assert np.max(np.abs(job.grad.cpu().numpy() - g)) <= 1e-6


@pytest.mark.parametrize("loss", [synth.LOGISTIC, synth.SQUARED])
def test_trajectory_on_generated_data(loss):
    _say(f"[case] sparse trajectory parity on generator data, loss {loss}")
    eta = 0.5 if loss == synth.LOGISTIC else 0.1
    p = synth.make_sparse_glm(loss, 20000, 5000, 30.0, seed=4, lam=1e-4, eta=eta, K=15)
    job = _job_from_problem(p)
    glm.glm_step_sparse(job, p.K, glm.alloc_sparse_workspace(job))
    torch.cuda.synchronize()
    lh, gh, wK, g_last = oracle.sparse_run(loss, p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy(),
                                           p.y.numpy(), p.D, np.zeros(p.D), p.lam, p.eta, p.K)
    got = job.history().cpu().numpy()
    assert all(rel(got[k], lh[k]) <= REL_TOL for k in range(p.K)), (got, lh)
    assert rel(np.linalg.norm(job.grad.cpu().numpy().astype(np.float64)), gh[-1]) <= REL_TOL
    assert np.max(np.abs(job.w.cpu().numpy() - wK)) <= REL_TOL * np.max(np.abs(wK))
    assert got[-1] < got[0]


def test_dense_matrix_as_sparse_agrees_with_dense_path():
    _say("[case] a dense matrix stored sparsely gives the dense path's trajectory")
    p = synth.make_glm(synth.LOGISTIC, 3000, 64, seed=2, lam=1e-3, eta=0.3, K=6)
    job, _ = _job_from_scipy(sp.csr_matrix(p.X.numpy()), p.y.numpy(), p.loss, p.lam, p.eta, 6)
    glm.glm_step_sparse(job, 6, glm.alloc_sparse_workspace(job))
    d = glm.Job(p.X.cuda(), p.y.cuda(), p.w0.cuda(), p.loss, p.lam, p.eta, 6)
    glm.glm_step(d, 6, glm.alloc_workspace([d]))
    torch.cuda.synchronize()
    a, b = job.history().cpu().numpy(), d.history().cpu().numpy()
    assert np.max(np.abs(a - b) / b) <= 1e-5
    assert torch.allclose(job.w, d.w, rtol=1e-4, atol=1e-6)


def test_sparse_reruns_bit_identical_and_split_calls():
    _say("[case] sparse rerun determinism and K = 3 + 4")
    p = synth.make_sparse_glm(synth.HINGE, 50000, 20000, 40.0, seed=9, lam=1e-4, eta=0.05, K=7, device="cuda")
    outs = []
    for split in ((7,), (7,), (3, 4)):
        job = _job_from_problem(p)
        ws = glm.alloc_sparse_workspace(job)
        for it in split:
            glm.glm_step_sparse(job, it, ws)
        torch.cuda.synchronize()
        outs.append((job.history().clone(), job.w.clone(), job.grad.clone()))
    for o in outs[1:]:
        assert all(torch.equal(x, y) for x, y in zip(outs[0], o))


def test_sparse_errors():
    _say("[case] sparse error codes")
    p = synth.make_sparse_glm(synth.LOGISTIC, 100, 50, 5.0, seed=1, lam=1e-3, eta=0.1, K=2)
    job = _job_from_problem(p, hist_cap=2)
    ws = glm.alloc_sparse_workspace(job)
    with pytest.raises(glm.GlmError) as e:
        glm.glm_step_sparse(job, 3, ws)
    assert e.value.status == glm.GLM_ENOSPC
    with pytest.raises(glm.GlmError) as e:
        glm.glm_step_sparse(job, 1, ws[:256])
    assert e.value.status == glm.GLM_ENOSPC
    job.c.loss = 7
    with pytest.raises(glm.GlmError) as e:
        glm.glm_step_sparse(job, 1, ws)
    assert e.value.status == glm.GLM_EINVAL
    job.c.loss = 0
    job.c.schedule = 5
    with pytest.raises(glm.GlmError) as e:
        glm.glm_step_sparse(job, 1, ws)
    assert e.value.status == glm.GLM_EINVAL
    job.c.schedule = 0
    job.c.lambda_ = -1.0
    with pytest.raises(glm.GlmError):
        glm.glm_step_sparse(job, 1, ws)
    torch.cuda.synchronize()
    assert job.hist_len == 0 and job.w.abs().sum().item() == 0


def _tall(seed, N=1_200_000, D=300, nnz=3_000_000):
    """More rows than one panel of the column layout holds: a long column through every panel, a
    column that lives in one panel only, empty columns, the rest uniform."""
    rng = np.random.default_rng(seed)
    rows = rng.integers(0, N, size=nnz); cols = rng.integers(3, D - 5, size=nnz)
    rows = np.concatenate([rows, np.arange(0, N, 7), rng.integers(600_000, 700_000, size=5000)])
    cols = np.concatenate([cols, np.zeros(len(np.arange(0, N, 7)), dtype=np.int64), np.ones(5000, dtype=np.int64)])
    vals = (rng.standard_normal(len(rows)) / 3).astype(np.float32)
    return sp.csr_matrix((vals, (rows, cols)), shape=(N, D))


@pytest.mark.parametrize("loss", [synth.LOGISTIC, synth.SQUARED])
def test_row_panelled_column_layout(loss):
    _say(f"[case] sparse, 1.2e6 rows (column layout rebuilt by row panels), loss {loss}")
    A = _tall(11)
    N, D = A.shape
    rng = np.random.default_rng(3)
    y = _labels(loss, N, rng)
    eta = 0.5 if loss == synth.LOGISTIC else 0.05
    job, csr = _job_from_scipy(A, y, loss, 1e-4, eta, 3)
    assert job.c.prepared == 0
    _check_steps(job, csr, y, D, loss, 1e-4, eta, 3, "panels")
    assert job.c.prepared == 1


def test_unsorted_columns_fall_back_to_the_callers_layout():
    _say("[case] sparse, 1.2e6 rows, rows of a column not ascending: caller's layout is used")
    A = _tall(12)
    N, D = A.shape
    rng = np.random.default_rng(4)
    y = _labels(synth.LOGISTIC, N, rng)
    job, csr = _job_from_scipy(A, y, synth.LOGISTIC, 1e-4, 0.5, 2)
    # reverse the entries of every column: same matrix, descending rows
    cp = job.tensors[3].cpu().numpy(); ri = job.tensors[4].cpu().numpy(); cv = job.tensors[5].cpu().numpy()
    ri2, cv2 = ri.copy(), cv.copy()
    for j in range(D):
        ri2[cp[j]:cp[j + 1]] = ri[cp[j]:cp[j + 1]][::-1]; cv2[cp[j]:cp[j + 1]] = cv[cp[j]:cp[j + 1]][::-1]
    job.tensors[4].copy_(torch.from_numpy(ri2)); job.tensors[5].copy_(torch.from_numpy(cv2))
    _check_steps(job, csr, y, D, synth.LOGISTIC, 1e-4, 0.5, 2, "unsorted")
    assert job.c.prepared == 2


def test_panelled_layout_reruns_and_split_calls_bit_identical():
    _say("[case] sparse with panels: reruns and 2 + 3 iterations = 5")
    A = _tall(13)
    N, D = A.shape
    y = _labels(synth.LOGISTIC, N, np.random.default_rng(5))
    outs = []
    for split in ((5,), (5,), (2, 3)):
        job, _ = _job_from_scipy(A, y, synth.LOGISTIC, 1e-4, 0.5, 5)
        ws = glm.alloc_sparse_workspace(job)
        for n in split:
            glm.glm_step_sparse(job, n, ws)
        torch.cuda.synchronize()
        assert job.c.prepared == 1
        outs.append((job.history().cpu().clone(), job.w.cpu().clone(), job.grad.cpu().clone()))
    for o in outs[1:]:
        for x, z in zip(outs[0], o):
            assert torch.equal(x, z)


def test_prepared_flag_is_only_believed_for_the_workspace_it_was_set_on():
    _say("[case] sparse with panels: two jobs taking turns on one workspace; a forged flag on a fresh workspace")
    A, B = _tall(21), _tall(22, N=1_000_003, D=200, nnz=2_000_000)
    ya = _labels(synth.LOGISTIC, A.shape[0], np.random.default_rng(6))
    yb = _labels(synth.LOGISTIC, B.shape[0], np.random.default_rng(7))
    # references: each job alone on a workspace of its own
    refs = []
    for M, y in ((A, ya), (B, yb)):
        job, _ = _job_from_scipy(M, y, synth.LOGISTIC, 1e-4, 0.5, 4)
        glm.glm_step_sparse(job, 4, glm.alloc_sparse_workspace(job))
        torch.cuda.synchronize()
        refs.append((job.history().cpu().clone(), job.w.cpu().clone()))
    ja, _ = _job_from_scipy(A, ya, synth.LOGISTIC, 1e-4, 0.5, 4)
    jb, _ = _job_from_scipy(B, yb, synth.LOGISTIC, 1e-4, 0.5, 4)
    wa, wb = glm.alloc_sparse_workspace(ja), glm.alloc_sparse_workspace(jb)
    shared = wa if wa.numel() >= wb.numel() else wb
    for _ in range(2):                      # A, B, A, B on the same memory, two iterations each
        for job in (ja, jb):
            glm.glm_step_sparse(job, 2, shared)
            assert job.c.prepared == 1
    torch.cuda.synchronize()
    for job, ref in ((ja, refs[0]), (jb, refs[1])):
        assert torch.equal(job.history().cpu(), ref[0]) and torch.equal(job.w.cpu(), ref[1])
    # a struct that claims a layout which this (new, zero-filled) workspace does not hold
    jc, _ = _job_from_scipy(A, ya, synth.LOGISTIC, 1e-4, 0.5, 4)
    jc.c.prepared = 1
    fresh = torch.zeros_like(wa)
    glm.glm_step_sparse(jc, 4, fresh)
    torch.cuda.synchronize()
    assert torch.equal(jc.history().cpu(), refs[0][0]) and torch.equal(jc.w.cpu(), refs[0][1])
    jc.c.prepared = 3
    with pytest.raises(glm.GlmError) as e:
        glm.glm_step_sparse(jc, 0, fresh)
    assert e.value.status == glm.GLM_EINVAL


# ---- products by scatter into LDS with fixed-point sums (at least 2^22 stored entries) ----------

@pytest.mark.parametrize("loss,N,D,mean", [(synth.LOGISTIC, 300_000, 200_000, 20.0), (synth.SQUARED, 250_000, 70_000, 18.0),
                                           (synth.HINGE, 1_500_000, 300, 3.2),
                                           # 18 windows of the gathered residuals and 275 panels of margins
                                           (synth.SQUARED, 4_500_000, 200, 1.2),
                                           # too few entries for the 306 panels of the row product: only the column product takes the path
                                           (synth.LOGISTIC, 5_000_000, 200, 0.9)])
def test_scatter_path_each_step_matches_oracle(loss, N, D, mean):
    _say(f"[case] sparse, fixed-point scatter path: loss {loss}, {N} x {D}, about {mean} entries per row")
    eta = {synth.LOGISTIC: 0.5, synth.HINGE: 0.05, synth.SQUARED: 0.05}[loss]
    p = synth.make_sparse_glm(loss, N, D, mean, seed=41, lam=1e-4, eta=eta, K=3)
    assert p.col_idx.numel() >= (1 << 22)
    job = _job_from_problem(p)
    _check_steps(job, (p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy()), p.y.numpy(), D, loss, p.lam, eta, 3,
                 "scatter")
    assert job.c.prepared == 1


def test_scatter_path_reruns_split_calls_and_duplicates():
    _say("[case] sparse, fixed-point scatter path: duplicates, empty rows and columns, reruns and 2 + 3 = 5, bit for bit")
    rng = np.random.default_rng(42)
    N, D, nnz = 120_000, 50_000, 5_000_000
    rows = rng.integers(0, N - 500, size=nnz); cols = rng.integers(100, D, size=nnz)      # rows / columns left empty
    rows[:1000] = 7; cols[:1000] = 123                                                    # a thousand duplicates
    vals = (rng.standard_normal(nnz) * np.exp(rng.uniform(-6, 6, size=nnz))).astype(np.float32)   # 5 decades of sizes
    coo = sp.coo_matrix((vals, (rows, cols)), shape=(N, D))
    # CSR with the duplicates kept (scipy would add them up)
    order = np.lexsort((cols, rows))
    rp = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=N))]).astype(np.int64)
    ci = cols[order].astype(np.int32); rv = vals[order]
    corder = np.argsort(ci, kind="stable")
    cp = np.concatenate([[0], np.cumsum(np.bincount(ci, minlength=D))]).astype(np.int64)
    ri = np.repeat(np.arange(N, dtype=np.int32), np.diff(rp))[corder]
    y = _labels(synth.SQUARED, N, rng)
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def job():
        return glm.SparseJob(T(rp), T(ci), T(rv), T(cp), T(ri), T(rv[corder]), T(y), torch.zeros(D, device="cuda"),
                             synth.SQUARED, 1e-4, 1e-6, 5)
    outs = []
    for split in ((5,), (5,), (2, 3)):
        jb = job()
        ws = glm.alloc_sparse_workspace(jb)
        for n in split:
            glm.glm_step_sparse(jb, n, ws)
        torch.cuda.synchronize()
        assert jb.c.prepared == 1
        outs.append((jb.history().cpu().clone(), jb.w.cpu().clone(), jb.grad.cpu().clone()))
    for o in outs[1:]:
        for x, z in zip(outs[0], o):
            assert torch.equal(x, z)
    # and the numbers are the oracle's
    jb = job()
    _check_steps(jb, (rp, ci, rv), y, D, synth.SQUARED, 1e-4, 1e-6, 2, "scatter duplicates")
    del coo


def test_scatter_path_with_an_empty_window_and_empty_panels():
    _say("[case] sparse, fixed-point scatter path: 262144 consecutive empty rows (a whole window of the gathered "
         "residuals, sixteen output panels), columns left empty at both ends")
    rng = np.random.default_rng(44)
    N, D, nnz = 600_000, 40_000, 4_500_000
    rows = rng.integers(0, 262_144 + (N - 524_288), size=nnz)
    rows = np.where(rows >= 262_144, rows + 262_144, rows)               # nothing in [262144, 524288)
    cols = rng.integers(20_000, D - 3_000, size=nnz)                      # the first column panel and the last columns empty
    vals = rng.standard_normal(nnz).astype(np.float32) / 3
    order = np.lexsort((cols, rows))
    rp = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=N))]).astype(np.int64)
    ci = cols[order].astype(np.int32); rv = vals[order]
    corder = np.argsort(ci, kind="stable")
    cp = np.concatenate([[0], np.cumsum(np.bincount(ci, minlength=D))]).astype(np.int64)
    ri = np.repeat(np.arange(N, dtype=np.int32), np.diff(rp))[corder]
    y = _labels(synth.LOGISTIC, N, rng)
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    job = glm.SparseJob(T(rp), T(ci), T(rv), T(cp), T(ri), T(rv[corder]), T(y), torch.zeros(D, device="cuda"),
                        synth.LOGISTIC, 1e-4, 0.5, 3)
    _check_steps(job, (rp, ci, rv), y, D, synth.LOGISTIC, 1e-4, 0.5, 3, "scatter, empty window")
    assert job.c.prepared == 1
    w = job.w.cpu().numpy()
    assert not np.any(w[:20_000]) and not np.any(w[D - 3_000:])           # columns without entries never move from 0


# ---- CSR alone: the library builds the column layout itself -------------------------------------

def _csr_only_twin(job):
    """The same job without its column arrays (fresh weights, gradient and history)."""
    rp, ci, rv, _, _, _, y = job.tensors
    return glm.SparseJob(rp, ci, rv, None, None, None, y, torch.zeros_like(job.w), job.c.loss, job.c.lambda_,
                         job.c.step, job.c.hist_cap, job.c.schedule)


def _same_bits(a, b):
    return (a.loss_hist.cpu().numpy().tobytes() == b.loss_hist.cpu().numpy().tobytes()
            and a.w.cpu().numpy().tobytes() == b.w.cpu().numpy().tobytes()
            and a.grad.cpu().numpy().tobytes() == b.grad.cpu().numpy().tobytes())


@pytest.mark.parametrize("which", ["segmented sums", "row panels", "scatter"])
def test_csr_only_input_equals_csr_plus_csc_bit_for_bit_and_matches_oracle(which):
    """The column layout the library builds is the stable sort of the entries by column, which is what
    the generators hand over as CSC: the two ways in must then agree bit for bit, on each of the three
    internal paths; the CSR-only job is also held to the oracle step by step."""
    _say(f"[case] sparse, CSR alone ({which})")
    if which == "segmented sums":
        p = synth.make_sparse_glm(synth.LOGISTIC, 5000, 700, 9.0, seed=5, lam=1e-3, eta=0.5, K=4)
        full = _job_from_problem(p)
        csr, y, D, loss, lam, eta = (p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy()), p.y.numpy(), p.D, p.loss, p.lam, 0.5
    elif which == "row panels":
        A = _tall(13)
        rng = np.random.default_rng(4)
        y = _labels(synth.SQUARED, A.shape[0], rng)
        full, csr = _job_from_scipy(A, y, synth.SQUARED, 1e-4, 0.05, 4)
        D, loss, lam, eta = A.shape[1], synth.SQUARED, 1e-4, 0.05
    else:
        p = synth.make_sparse_glm(synth.LOGISTIC, 300_000, 200_000, 20.0, seed=43, lam=1e-4, eta=0.5, K=4)
        full = _job_from_problem(p)
        csr, y, D, loss, lam, eta = (p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy()), p.y.numpy(), p.D, p.loss, p.lam, 0.5
    alone = _csr_only_twin(full)
    assert glm.glm_sparse_workspace_bytes(alone) > glm.glm_sparse_workspace_bytes(full)
    ws_full, ws_alone = glm.alloc_sparse_workspace(full), glm.alloc_sparse_workspace(alone)
    glm.glm_step_sparse(full, 3, ws_full)
    glm.glm_step_sparse(alone, 2, ws_alone)          # split calls: the second one finds the layout in the workspace
    assert alone.c.prepared == 1
    glm.glm_step_sparse(alone, 1, ws_alone)
    torch.cuda.synchronize()
    assert _same_bits(full, alone), which
    fresh = _csr_only_twin(full)
    _check_steps(fresh, csr, y, D, loss, lam, eta, 2, f"csr only, {which}")


def test_csr_only_hand_built_structures_and_errors():
    _say("[case] sparse, CSR alone: duplicates, empty rows and columns, unsorted columns inside a row, nnz = 0")
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    rp = np.array([0, 3, 3, 6, 7], np.int64)                    # row 1 empty
    ci = np.array([4, 0, 4, 2, 0, 2, 5], np.int32)              # column 4 twice in row 0, columns not ascending, 1 and 3 empty
    rv = np.array([0.5, -1.0, 0.25, 2.0, 1.5, -0.5, 1.0], np.float32)
    y = np.array([1, 0, 1, 0], np.float32)
    job = glm.SparseJob(T(rp), T(ci), T(rv), None, None, None, T(y), torch.zeros(6, device="cuda"), synth.LOGISTIC,
                        1e-2, 0.5, 4)
    _check_steps(job, (rp, ci, rv), y, 6, synth.LOGISTIC, 1e-2, 0.5, 4, "csr only, hand-built")
    empty = glm.SparseJob(T(np.zeros(4, np.int64)), T(np.zeros(0, np.int32)), T(np.zeros(0, np.float32)), None, None,
                          None, T(np.array([1, 0, 1], np.float32)), torch.zeros(5, device="cuda"), synth.LOGISTIC, 0.0,
                          0.5, 2)
    glm.glm_step_sparse(empty, 2, glm.alloc_sparse_workspace(empty))
    torch.cuda.synchronize()
    assert abs(empty.loss_hist[0].item() - np.log(2.0)) < 1e-6 and empty.grad.abs().sum().item() == 0
    half = glm.SparseJob(T(rp), T(ci), T(rv), None, None, None, T(y), torch.zeros(6, device="cuda"), synth.LOGISTIC,
                         1e-2, 0.5, 4)
    half.c.row_idx = T(np.zeros(7, np.int32)).data_ptr()         # a column array without the others
    with pytest.raises(glm.GlmError) as e:
        glm.glm_step_sparse(half, 1, glm.alloc_sparse_workspace(job))
    assert e.value.status == glm.GLM_EINVAL
