"""Pins of the K-Means oracle (CPU only).

The paper prints no value for a K-Means iteration (it only lists the algorithm, Sec. 3 "Setup"),
so the oracle is held against things other than itself: a hand-worked example, scikit-learn and
SciPy routines that implement the same textbook definitions independently, closed forms (K = 1,
K = N) and invariants.  The second half plants mistakes in a copy of the C source and checks that
the pins reject each of them.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
from paper_1802_04819_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kmeans_oracle.c")


class _Lib:
    """The oracle's two routines from an arbitrary shared object (the real one or a mutant)."""

    def __init__(self, lib):
        fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        ip, lp = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        lib.oracle_kmeans_assign.argtypes = [fp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_int32, ip, dp, dp]
        lib.oracle_kmeans_step.argtypes = [fp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_int32, ip, lp, dp]
        self.lib = lib

    def assign(self, X, C):
        X = np.ascontiguousarray(X, np.float32); C = np.ascontiguousarray(C, np.float64)
        N, D = X.shape
        a = np.empty(N, np.int32); b = np.empty(N); s = np.empty(N)
        fp, dp, ip = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        rc = self.lib.oracle_kmeans_assign(X.ctypes.data_as(fp), N, D, C.ctypes.data_as(dp), C.shape[0],
                                           a.ctypes.data_as(ip), b.ctypes.data_as(dp), s.ctypes.data_as(dp))
        assert rc == 0
        return a, b, s

    def step(self, X, C):
        X = np.ascontiguousarray(X, np.float32); C = np.array(C, np.float64, copy=True, order="C")
        N, D = X.shape
        a = np.empty(N, np.int32); cnt = np.empty(C.shape[0], np.int64); L = ctypes.c_double()
        fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        rc = self.lib.oracle_kmeans_step(X.ctypes.data_as(fp), N, D, C.ctypes.data_as(dp), C.shape[0],
                                         a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                         cnt.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), ctypes.byref(L))
        assert rc == 0
        return L.value, C, a, cnt

    def run(self, X, C, iters):
        hist = []
        for _ in range(iters):
            L, C, a, cnt = self.step(X, C)
            hist.append(L)
        return np.array(hist), C, a, cnt


def _problem(N=3000, D=12, K=7, seed=3, **kw):
    p = synth.make_kmeans(N, D, K, seed, **kw)
    return p.X.numpy(), p.C0.numpy().astype(np.float64)


# ---- the pins, written against any implementation `o` with assign/step/run ---------------------

def pin_hand_example(o):
    # five points on a line and in the plane, worked by hand
    X = np.array([[0, 0], [0, 1], [10, 10], [10, 11], [5, 5]], np.float32)
    C = np.array([[0, 0], [10, 10]], np.float64)
    L, Cn, a, cnt = o.step(X, C)
    assert a.tolist() == [0, 0, 1, 1, 0]              # (5,5) is 50 away from both: lowest index wins
    assert cnt.tolist() == [3, 2]
    assert L == pytest.approx((0 + 1 + 0 + 1 + 50) / 5, rel=1e-15)
    assert np.allclose(Cn, [[5 / 3, 2.0], [10.0, 10.5]], rtol=1e-15)
    a2, best, second = o.assign(X, C)
    assert best.tolist() == [0, 1, 0, 1, 50] and second.tolist() == [200, 181, 200, 221, 50]
    # three centroids, asymmetric coordinates: catches a transposed centroid matrix
    X = np.array([[1, 0, 0], [0, 2, 0], [0, 0, 3], [1, 2, 3]], np.float32)
    C = np.array([[1, 0, 0], [0, 2, 0], [0, 0, 3]], np.float64)
    L, Cn, a, cnt = o.step(X, C)
    assert a.tolist() == [0, 1, 2, 2]                 # (1,2,3): distances 13, 10, 5
    assert L == pytest.approx(5 / 4, rel=1e-15)
    assert np.allclose(Cn, [[1, 0, 0], [0, 2, 0], [0.5, 1, 3]])


def pin_library_assignments(o):
    from scipy.cluster.vq import vq
    from sklearn.metrics import pairwise_distances_argmin_min
    X, C = _problem()
    a, best, second = o.assign(X, C)
    a_sk, d_sk = pairwise_distances_argmin_min(X.astype(np.float64), C, metric="sqeuclidean")
    assert np.array_equal(a, a_sk)
    assert np.allclose(best, d_sk, rtol=1e-12)
    code, dist = vq(X.astype(np.float64), C)          # SciPy returns the (unsquared) distance
    assert np.array_equal(a, code)
    assert np.allclose(np.sqrt(best), dist, rtol=1e-12)
    full = ((X.astype(np.float64)[:, None, :] - C[None]) ** 2).sum(-1)
    full.sort(axis=1)
    assert np.allclose(second, full[:, 1], rtol=1e-12)


def pin_library_iteration(o):
    from scipy.cluster.vq import kmeans2
    from sklearn.cluster import KMeans
    X, C = _problem()
    L, Cn, a, cnt = o.step(X, C)
    C_sp, lab_sp = kmeans2(X.astype(np.float64), C.copy(), iter=1, minit="matrix")
    assert np.allclose(Cn, C_sp, rtol=1e-10)
    km = KMeans(n_clusters=C.shape[0], init=C, n_init=1, max_iter=1, algorithm="lloyd", tol=0.0).fit(X.astype(np.float64))
    assert np.allclose(Cn, km.cluster_centers_, rtol=1e-6, atol=1e-6)
    # scikit-learn's score is minus the SUM of squared distances to the nearest given centre
    km0 = KMeans(n_clusters=C.shape[0], init=C, n_init=1, max_iter=1).fit(X.astype(np.float64))
    km0.cluster_centers_ = C.copy()
    assert L == pytest.approx(-km0.score(X.astype(np.float64)) / X.shape[0], rel=1e-6)
    # several iterations against scikit-learn's fixed point
    hist, CK, aK, cntK = o.run(X, C, 60)
    kmf = KMeans(n_clusters=C.shape[0], init=C, n_init=1, max_iter=300, algorithm="lloyd", tol=0.0).fit(X.astype(np.float64))
    assert hist[-1] == pytest.approx(kmf.inertia_ / X.shape[0], rel=1e-5)


def pin_closed_forms(o):
    X, _ = _problem(N=500, D=5, K=3)
    X64 = X.astype(np.float64)
    # K = 1: any centroid c gives L = mean |x - c|^2 and the update is the mean of the data
    c = np.full((1, 5), 0.25)
    L, Cn, a, cnt = o.step(X, c)
    assert L == pytest.approx(((X64 - c) ** 2).sum(1).mean(), rel=1e-13)
    assert np.allclose(Cn[0], X64.mean(0), rtol=1e-13) and cnt.tolist() == [500] and not a.any()
    L2, _, _, _ = o.step(X, Cn)
    assert L2 == pytest.approx(X64.var(0).sum(), rel=1e-12)         # total variance
    # K = N with the points as centroids: zero loss, every point its own cluster
    Xs = X[:40]
    L, Cn, a, cnt = o.step(Xs, Xs.astype(np.float64))
    assert L == 0.0 and a.tolist() == list(range(40)) and np.array_equal(Cn, Xs.astype(np.float64))


def pin_invariants(o):
    X, C = _problem(N=2000, D=6, K=5, seed=11)
    hist, CK, aK, cntK = o.run(X, C, 25)
    assert np.all(np.diff(hist) <= 1e-12 * hist[0]) and hist[-1] < 0.9 * hist[0]   # Lloyd never increases the loss
    L, Cn, a, cnt = o.step(X, C)
    assert cnt.sum() == X.shape[0] and np.array_equal(cnt, np.bincount(a, minlength=5))
    # the update is the minimiser for fixed assignments: the loss at (a, Cn) is not above (a, C)
    X64 = X.astype(np.float64)
    assert ((X64 - Cn[a]) ** 2).sum(1).mean() <= L + 1e-12
    # translation: shifting points and centroids alike changes nothing but the centroids' position
    sh = np.arange(6, dtype=np.float64) * 0.5 - 1.0            # exactly representable
    Ls, Cs, as_, cs = o.step((X64 + sh).astype(np.float32).astype(np.float64).astype(np.float32), C + sh)
    Xs64 = (X64 + sh).astype(np.float32).astype(np.float64)
    Lr = ((Xs64 - (C + sh)[as_]) ** 2).sum(1).mean()
    assert Ls == pytest.approx(Lr, rel=1e-12)
    assert np.mean(as_ == a) > 0.999
    # relabelling: permuting the centroids permutes assignments and updated centroids
    perm = np.array([3, 0, 4, 1, 2])
    Lp, Cp, ap, cp = o.step(X, C[perm])
    assert Lp == pytest.approx(L, rel=1e-14)
    assert np.array_equal(perm[ap], a) and np.allclose(Cp, Cn[perm], rtol=1e-13) and np.array_equal(cp, cnt[perm])
    # duplicating every point changes neither loss nor centroids (mean, not sum)
    Ld, Cd, ad, cd = o.step(np.concatenate([X, X]), C)
    assert Ld == pytest.approx(L, rel=1e-13) and np.allclose(Cd, Cn, rtol=1e-13) and np.array_equal(cd, 2 * cnt)


def pin_empty_cluster_and_ties(o):
    X = np.array([[0.0], [1.0], [2.0], [3.0]], np.float32)
    C = np.array([[1.0], [100.0], [2.0]], np.float64)
    L, Cn, a, cnt = o.step(X, C)
    assert a.tolist() == [0, 0, 2, 2] and cnt.tolist() == [2, 0, 2]
    assert Cn[:, 0].tolist() == [0.5, 100.0, 2.5]      # the empty cluster keeps its centroid
    assert L == pytest.approx((1 + 0 + 0 + 1) / 4)
    # identical centroids: the lower index takes every point
    C = np.array([[1.5], [1.5]], np.float64)
    L, Cn, a, cnt = o.step(X, C)
    assert a.tolist() == [0, 0, 0, 0] and cnt.tolist() == [4, 0] and Cn[:, 0].tolist() == [1.5, 1.5]
    # a point exactly between two centroids, the farther-indexed one listed first
    C = np.array([[2.0], [0.0]], np.float64)
    a, best, second = o.assign(np.array([[1.0]], np.float32), C)
    assert a.tolist() == [0] and best.tolist() == [1.0] and second.tolist() == [1.0]


PINS = [pin_hand_example, pin_library_assignments, pin_library_iteration, pin_closed_forms, pin_invariants,
        pin_empty_cluster_and_ties]


class _Real:
    assign = staticmethod(lambda X, C: oracle.kmeans_assign(np.ascontiguousarray(X, np.float32), C))
    step = staticmethod(lambda X, C: oracle.kmeans_step(np.ascontiguousarray(X, np.float32), C))
    run = staticmethod(lambda X, C, n: oracle.kmeans_run(np.ascontiguousarray(X, np.float32), C, n))


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_passes_pin(pin):
    pin(_Real)


MUTANTS = {
    "sum_instead_of_mean_loss": ("*loss_out = S / (double)N;", "*loss_out = S;"),
    "unsquared_distance_terms": ("d += t * t;", "d += (t < 0 ? -t : t);"),
    "farthest_instead_of_nearest": ("else if (d < b) { s = b; b = d; a = k; }", "else if (d > b) { s = b; b = d; a = k; }"),
    "ties_to_higher_index": ("else if (d < b) { s = b; b = d; a = k; }", "else if (d <= b) { s = b; b = d; a = k; }"),
    "second_not_tracked_on_improvement": ("else if (d < b) { s = b; b = d; a = k; }", "else if (d < b) { b = d; a = k; }"),
    "transposed_centroids": ("const double *c = C + (int64_t)k * D;", "const double *c = C + k;"),
    "skips_last_coordinate": ("for (int32_t j = 0; j < D; ++j) {\n                double t", "for (int32_t j = 0; j + 1 < D; ++j) {\n                double t"),
    "skips_first_centroid_in_sums": ("counts[a] += 1;", "if (a > 0) counts[a] += 1;"),
    "mean_over_all_points": ("sums[(int64_t)k * D + j] / (double)counts[k];", "sums[(int64_t)k * D + j] / (double)N;"),
    "sum_instead_of_mean_centroid": ("sums[(int64_t)k * D + j] / (double)counts[k];", "sums[(int64_t)k * D + j];"),
    "empty_cluster_zeroed": ("if (counts[k] == 0) continue;", "if (counts[k] == 0) { for (int32_t j = 0; j < D; ++j) C[(int64_t)k * D + j] = 0.0; continue; }"),
    "sums_use_wrong_row": ("+= (double)X[i * (int64_t)D + j];", "+= (double)X[(i > 0 ? i - 1 : 0) * (int64_t)D + j];"),
    "sums_transposed_x": ("+= (double)X[i * (int64_t)D + j];", "+= (double)X[i + j * N >= N * D ? 0 : i + j * N];"),
}


def _compile(tmp_path, name, old=None, new=None):
    src = open(SRC).read()
    if old is not None:
        assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
        src = src.replace(old, new)
    c = tmp_path / f"{name}.c"; so = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(c)], check=True)
    return _Lib(ctypes.CDLL(str(so)))


def _rejected(o):
    for pin in PINS:
        try:
            pin(o)
        except AssertionError:
            return pin.__name__
    return None


def test_unmodified_copy_passes_every_pin(tmp_path):
    assert _rejected(_compile(tmp_path, "clean")) is None


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_rejected(tmp_path, name):
    old, new = MUTANTS[name]
    assert _rejected(_compile(tmp_path, name, old, new)) is not None, f"no pin notices: {name}"


def test_generator_shapes_and_seed():
    p = synth.make_kmeans(5000, 16, 9, 4, blobs=5, offset=2.0)
    q = synth.make_kmeans(5000, 16, 9, 4, blobs=5, offset=2.0)
    assert tuple(p.X.shape) == (5000, 16) and tuple(p.C0.shape) == (9, 16) and p.X.numpy().dtype == np.float32
    assert bool((p.X == q.X).all()) and bool((p.C0 == q.C0).all())
    # the starting centroids are distinct rows of X
    Xn, Cn = p.X.numpy(), p.C0.numpy()
    rows = {Xn[i].tobytes() for i in range(Xn.shape[0])}
    assert all(Cn[k].tobytes() in rows for k in range(9)) and len({Cn[k].tobytes() for k in range(9)}) == 9
