"""The library driven from a plain C program (tests/c_abi_demo.c): no Python binding, no torch in
the process.  The test rebuilds the program's inputs from its generator and holds the ten losses
it prints to the oracle's, at the same bar as every other parity test."""
import os
import subprocess

import numpy as np
import pytest

import oracle
from paper_1802_04819_amd import build as b
from _parity import REL_TOL

pytestmark = pytest.mark.gpu


def _demo_inputs(N=20000, D=64):
    """The demo's linear congruential stream, replayed: w*, then row by row X with the label taken
    from a float32 running sum in column order, as the C loop does."""
    s = 12345
    vals = np.empty(D + N * D, dtype=np.float64)
    for i in range(vals.size):
        s = (s * 1664525 + 1013904223) & 0xFFFFFFFF
        vals[i] = ((s >> 8) & 0xFFFFFF) / 8388608.0 - 1.0
    wstar = vals[:D].astype(np.float32)
    X = vals[D:].astype(np.float32).reshape(N, D)
    m = np.cumsum(X * wstar[None, :], axis=1, dtype=np.float32)[:, -1]
    return X, (m > 0).astype(np.float32)


def test_c_program_matches_the_oracle():
    print("[case] plain C consumer: 10 logistic iterations on 20000 x 64", flush=True)
    if not os.path.exists(b.C_DEMO_BIN):
        b.build_c_demo()                     # gcc only; the library itself is loaded as built
    res = subprocess.run([b.C_DEMO_BIN], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=100)
    assert res.returncode == 0, res.stderr
    got = np.array([float(t) for t in res.stdout.split()])
    assert got.shape == (10,)
    assert abs(got[0] - np.log(2.0)) < 1e-6 and np.all(np.diff(got) < 0)
    X, y = _demo_inputs()
    assert 0.3 < y.mean() < 0.7
    lh, _, _, _ = oracle.run(0, X, y, np.zeros(64), 1e-4, 1.0, 10)
    assert np.max(np.abs(got - lh) / np.abs(lh)) <= REL_TOL
