"""CPU pins of the sparse (CSR) oracle routines and of the sparse input generator."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
from paper_1802_04819_amd import synth


def _problem(loss, seed=0, N=300, D=80, mean=6.0):
    return synth.make_sparse_glm(loss, N, D, mean, seed, lam=1e-2, eta=0.1, K=5)


def _scipy_csr(p):
    return sp.csr_matrix((p.row_val.numpy().astype(np.float64), p.col_idx.numpy(), p.row_ptr.numpy()),
                         shape=(p.N, p.D))


@pytest.mark.parametrize("loss", [0, 1, 2])
def test_sparse_oracle_equals_dense_oracle_on_the_densified_matrix(loss):
    p = _problem(loss, seed=loss)
    A = _scipy_csr(p)                                   # duplicates are summed by toarray()
    Xd = A.toarray().astype(np.float32)
    # summing duplicates in fp64 then rounding to fp32 would change bits: compare in fp64 instead
    rng = np.random.default_rng(1)
    w = rng.standard_normal(p.D)
    L, g = oracle.sparse_loss_grad(loss, p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy(),
                                   p.y.numpy(), p.D, w, p.lam)
    z = A @ w
    y = p.y.numpy().astype(np.float64)
    if loss == 0:
        l = np.logaddexp(0, z) - y * z; r = 1 / (1 + np.exp(-z)) - y
    elif loss == 1:
        m = 1 - y * z; l = np.maximum(m, 0); r = np.where(m > 0, -y, 0.0)
    else:
        l = 0.5 * (z - y) ** 2; r = z - y
    assert L == pytest.approx(l.mean() + 0.5 * p.lam * w @ w, rel=1e-13)
    np.testing.assert_allclose(g, A.T @ r / p.N + p.lam * w, rtol=1e-11, atol=1e-14)
    # and the dense C oracle on a duplicate-free matrix gives the same numbers
    B = sp.random(200, 50, 0.1, format="csr", random_state=3, dtype=np.float32)
    yb = {0: (rng.random(200) > 0.5).astype(np.float32),
          1: np.where(rng.random(200) > 0.5, 1, -1).astype(np.float32),
          2: rng.standard_normal(200).astype(np.float32)}[loss]
    wb = rng.standard_normal(50)
    Ls, gs = oracle.sparse_loss_grad(loss, B.indptr, B.indices, B.data, yb, 50, wb, 0.1)
    Ld, gd = oracle.loss_grad(loss, B.toarray(), yb, wb, 0.1)
    assert Ls == pytest.approx(Ld, rel=1e-14)
    np.testing.assert_allclose(gs, gd, rtol=1e-12, atol=1e-15)


def test_closed_forms_at_zero_and_finite_differences():
    p = _problem(0, seed=5)
    L, g = oracle.sparse_loss_grad(0, p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy(), p.y.numpy(),
                                   p.D, np.zeros(p.D), 0.3)
    assert L == pytest.approx(np.log(2.0), rel=1e-14)
    A = _scipy_csr(p)
    np.testing.assert_allclose(g, A.T @ (0.5 - p.y.numpy().astype(np.float64)) / p.N, atol=1e-15)
    rng = np.random.default_rng(2)
    w = 0.5 * rng.standard_normal(p.D)
    args = (p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy(), p.y.numpy(), p.D)
    L, g = oracle.sparse_loss_grad(0, *args, w, 0.05)
    for j in rng.choice(p.D, 10, replace=False):
        e = np.zeros(p.D); e[j] = 1e-6
        fd = (oracle.sparse_loss_grad(0, *args, w + e, 0.05)[0] - oracle.sparse_loss_grad(0, *args, w - e, 0.05)[0]) / 2e-6
        assert abs(fd - g[j]) <= 2e-8 * max(1.0, abs(g[j]))


def test_sparse_run_replays_loss_grad():
    p = _problem(2, seed=7)
    args = (p.row_ptr.numpy(), p.col_idx.numpy(), p.row_val.numpy(), p.y.numpy(), p.D)
    lh, gh, wK, gl = oracle.sparse_run(2, *args, np.zeros(p.D), p.lam, p.eta, 4)
    w = np.zeros(p.D)
    for k in range(4):
        L, g = oracle.sparse_loss_grad(2, *args, w, p.lam)
        assert lh[k] == L
        w = w - p.eta * g
    np.testing.assert_array_equal(w, wK)
    assert np.all(np.diff(lh) < 0)


def test_generator_layouts_describe_the_same_matrix():
    p = synth.make_sparse_glm(0, 500, 3000, 8.0, 3, lam=0, eta=0, K=0)
    q = synth.make_sparse_glm(0, 500, 3000, 8.0, 3, lam=0, eta=0, K=0)
    assert torch.equal(p.col_idx, q.col_idx) and torch.equal(p.row_val, q.row_val) and torch.equal(p.y, q.y)
    A = _scipy_csr(p)
    C = sp.csc_matrix((p.col_val.numpy().astype(np.float64), p.row_idx.numpy(), p.col_ptr.numpy()), shape=(p.N, p.D))
    assert abs(A - C).max() < 1e-15
    assert p.row_ptr[-1].item() == p.nnz == p.col_ptr[-1].item()
    # rows of a column are listed in increasing order (stable sort), columns are skewed, some are empty
    cp, ri = p.col_ptr.numpy(), p.row_idx.numpy()
    assert all(np.all(np.diff(ri[cp[j]:cp[j + 1]]) >= 0) for j in range(p.D))
    per_col = np.diff(cp)
    assert per_col.max() > 20 * max(np.median(per_col), 1) and (per_col == 0).any()
    assert set(p.y.unique().tolist()) == {0.0, 1.0} and 0.3 < p.y.mean().item() < 0.7
