"""CPU tests of the seeded input generators and of the stored oracle trajectory."""
import os

import numpy as np
import torch

import oracle
from paper_1802_04819_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_make_glm_is_seeded_and_shaped():
    a = synth.make_glm(synth.LOGISTIC, 1000, 64, 3, lam=0.1, eta=0.1, K=1)
    b = synth.make_glm(synth.LOGISTIC, 1000, 64, 3, lam=0.1, eta=0.1, K=1)
    c = synth.make_glm(synth.LOGISTIC, 1000, 64, 4, lam=0.1, eta=0.1, K=1)
    assert torch.equal(a.X, b.X) and torch.equal(a.y, b.y)
    assert not torch.equal(a.X, c.X)
    assert a.X.shape == (1000, 64) and a.X.dtype == torch.float32 and a.X.is_contiguous()
    assert a.y.shape == (1000,) and a.w0.abs().sum() == 0


def test_label_encodings_and_balance():
    lo = synth.make_glm(synth.LOGISTIC, 20000, 32, 0, lam=0, eta=0, K=0)
    hi = synth.make_glm(synth.HINGE, 20000, 32, 0, lam=0, eta=0, K=0)
    sq = synth.make_glm(synth.SQUARED, 20000, 32, 0, lam=0, eta=0, K=0)
    assert set(lo.y.unique().tolist()) == {0.0, 1.0}
    assert set(hi.y.unique().tolist()) == {-1.0, 1.0}
    assert 0.45 < lo.y.mean().item() < 0.55
    assert abs(hi.y.mean().item()) < 0.1
    # same seed: the three label kinds come from the same margins
    assert torch.equal(lo.y * 2 - 1, hi.y)
    assert torch.equal((sq.y > 0).float(), lo.y)
    assert 0.8 < sq.y.var().item() < 1.4      # var(X.w*) ~ 1 plus noise variance 0.1


def test_config2_columns_are_badly_scaled():
    p = synth.config2(scale=2000 / 4_000_000)
    assert p.X.shape == (2000, 1024) and p.eta == 1e-4 and p.lam == 1e-5 and p.K == 20
    rms = p.X.pow(2).mean(0).sqrt()
    assert rms.min() < 0.05 and rms.max() > 20 and rms.min() > 0.005 and rms.max() < 150


def test_config3_specs_and_alloc():
    specs = synth.config3_specs()
    assert len(specs) == 160
    assert {s.loss for s in specs} == {0, 1, 2}
    assert {s.D for s in specs} == {64, 128, 256, 512}
    assert all(50_000 <= s.N <= 500_000 for s in specs)
    assert all(1e-6 <= s.lam <= 1e-3 for s in specs)
    assert specs == synth.config3_specs()
    a = synth.config3_alloc(0)
    assert a.shape == (160,) and a.dtype == np.int32 and a.min() >= 1 and a.max() <= 8
    assert not np.array_equal(a, synth.config3_alloc(1))
    tot = sum(4 * s.N * s.D for s in specs)
    assert 30e9 < tot < 55e9


def test_sweep_grid():
    lams, etas = synth.sweep_grid()
    assert lams.shape == (64,) and etas.shape == (64,)
    assert np.isclose(lams[0], 1e-6) and np.isclose(lams[-1], 1e-1)
    assert np.isclose(etas[0], 1e-3) and np.isclose(etas[7], 1.0) and np.isclose(etas[8], 1e-3)
    assert len({(float(a), float(b)) for a, b in zip(lams, etas)}) == 64


def _read_history(name):
    rows = [l.split() for l in open(os.path.join(GOLDEN, name)) if not l.startswith("#")]
    return np.array([[float(v) for v in r[1:]] for r in rows])


def test_cfg0_stored_history_is_what_the_oracle_computes():
    p = synth.config0()
    assert (p.N, p.D, p.K, p.lam, p.eta) == (4096, 128, 50, 1e-4, 0.1)
    h = _read_history("cfg0_history.txt")
    assert h.shape == (50, 2)
    lh, gh, _, _ = oracle.run(p.loss, p.X.numpy(), p.y.numpy(), np.zeros(p.D), p.lam, p.eta, p.K)
    np.testing.assert_allclose(lh, h[:, 0], rtol=1e-13)
    np.testing.assert_allclose(gh, h[:, 1], rtol=1e-12)
    # facts the file must satisfy whatever wrote it: ln 2 at w = 0, decreasing loss with
    # diminishing returns (Sec. 1: quality improvement diminishes with iterations)
    assert abs(h[0, 0] - np.log(2)) < 1e-13
    d = np.diff(h[:, 0])
    assert np.all(d < 0) and np.all(np.diff(d) > 0)
