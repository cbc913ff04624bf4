"""Seeded synthetic inputs for the GLM jobs (shared by the GPU path's tests, the
oracle's tests and the benchmark).

This module only draws random inputs; it contains none of the method's
arithmetic (no loss, residual, gradient or update) and imports neither the GPU
binding nor the oracle.  The paper's own datasets (Sec. 3 "Setup": more than
200 GB of text, image and audio features) are not available, and the paper
states no shapes for them; these generators stand in for them with dense fp32
matrices of the shapes used by the benchmark configurations.

Recipe for one job (``make_glm``):
  X   ~ N(0,1) entries, fp32, [N, D] row-major; optionally each column j is
        multiplied by 10**u_j with u_j ~ U(-2, 2)  (badly scaled features)
  w*  ~ N(0, 1/D) entries (variance 1/D)
  m_i = X_i . w* + e_i,  e_i ~ N(0, 0.1) (variance 0.1), evaluated in fp64
  y_i = 1[m_i > 0]            logistic   (labels in {0, 1})
        +1 if m_i >= 0 else -1 hinge      (labels in {-1, +1})
        m_i                    squared    (real targets)
  w0  = 0
The draw order from the one seeded generator is: column scales (if any), X, w*,
noise.  The stream of a ``torch.Generator`` depends on the device it lives on,
so a problem is reproducible for a given (seed, device) pair; small problems
that are compared with stored values are always drawn on the CPU.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

LOGISTIC, HINGE, SQUARED = 0, 1, 2
LOSS_NAMES = {LOGISTIC: "logistic", HINGE: "hinge", SQUARED: "squared"}


@dataclass
class GLMProblem:
    """One training job: data, labels, start point and hyper-parameters."""
    name: str
    loss: int
    X: torch.Tensor          # [N, D] fp32
    y: torch.Tensor          # [N] fp32
    w0: torch.Tensor         # [D] fp32
    lam: float
    eta: float
    K: int
    seed: int

    @property
    def N(self) -> int:
        return int(self.X.shape[0])

    @property
    def D(self) -> int:
        return int(self.X.shape[1])


def _matvec_f64(X: torch.Tensor, v: torch.Tensor, chunk_rows: int = 1 << 18) -> torch.Tensor:
    """X . v accumulated in fp64, by row chunks so no fp64 copy of X is held."""
    out = torch.empty(X.shape[0], dtype=torch.float64, device=X.device)
    v64 = v.to(torch.float64)
    for i0 in range(0, X.shape[0], chunk_rows):
        i1 = min(i0 + chunk_rows, X.shape[0])
        out[i0:i1] = X[i0:i1].to(torch.float64) @ v64
    return out


def make_glm(loss: int, N: int, D: int, seed: int, *, lam: float, eta: float, K: int,
             col_scale: bool = False, device: str = "cpu", name: str = "") -> GLMProblem:
    """Draw one job as described in the module docstring."""
    if loss not in LOSS_NAMES:
        raise ValueError("unknown loss type")
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    scale = None
    if col_scale:
        u = torch.rand(D, generator=g, device=dev, dtype=torch.float32) * 4.0 - 2.0
        scale = torch.pow(torch.tensor(10.0, device=dev), u)
    X = torch.randn((N, D), generator=g, device=dev, dtype=torch.float32)
    if scale is not None:
        X.mul_(scale)
    w_star = torch.randn(D, generator=g, device=dev, dtype=torch.float32) / math.sqrt(D)
    noise = torch.randn(N, generator=g, device=dev, dtype=torch.float32) * math.sqrt(0.1)
    m = _matvec_f64(X, w_star) + noise.to(torch.float64)
    if loss == LOGISTIC:
        y = (m > 0).to(torch.float32)
    elif loss == HINGE:
        y = torch.where(m >= 0, 1.0, -1.0).to(torch.float32)
    else:
        y = m.to(torch.float32)
    w0 = torch.zeros(D, dtype=torch.float32, device=dev)
    return GLMProblem(name or f"{LOSS_NAMES[loss]}_{N}x{D}", loss, X, y.contiguous(), w0,
                      float(lam), float(eta), int(K), int(seed))


# --------------------------------------------------------------------------- configs

def _scaled(n: int, scale: float, lo: int = 1) -> int:
    return max(lo, int(round(n * scale)))


def config0(device: str = "cpu") -> GLMProblem:
    """Logistic, 4096 x 128, lambda 1e-4, step 0.1, 50 iterations, seed 0."""
    return make_glm(LOGISTIC, 4096, 128, 0, lam=1e-4, eta=0.1, K=50, device=device,
                    name="cfg0_logistic_4096x128")


def config1(scale: float = 1.0, device: str = "cpu") -> GLMProblem:
    """Linear SVM (hinge), 1e6 x 256, lambda 1e-4, step 0.01, 100 subgradient iterations."""
    N = _scaled(1_000_000, scale)
    return make_glm(HINGE, N, 256, 0, lam=1e-4, eta=0.01, K=100, device=device,
                    name=f"cfg1_hinge_{N}x256")


def config2(scale: float = 1.0, device: str = "cpu") -> GLMProblem:
    """Logistic, 4e6 x 1024 with columns scaled by 10**U(-2,2), lambda 1e-5, 20 iterations.

    The step is not part of the configuration's statement; 1e-4 is used because
    the largest column scale (100) bounds the logistic curvature by about
    0.25 * 1e4, so a stable constant step must stay below 8e-4.
    """
    N = _scaled(4_000_000, scale)
    return make_glm(LOGISTIC, N, 1024, 0, lam=1e-5, eta=1e-4, K=20, col_scale=True,
                    device=device, name=f"cfg2_logistic_{N}x1024_colscaled")


@dataclass
class JobSpec:
    """Shape and hyper-parameters of one job of the concurrent-jobs configuration."""
    index: int
    seed: int
    loss: int
    N: int
    D: int
    lam: float
    eta: float


def config3_specs(J: int = 160, scale: float = 1.0) -> List[JobSpec]:
    """The 160 mixed jobs: loss ~ U{logistic, hinge, squared}, N ~ U[50k, 500k],
    D ~ U{64,128,256,512}, lambda = 10**U(-6,-3), step = 10**U(-2,-1) (hinge:
    10**U(-3,-2)); job j draws from its own generator seeded 1000 + j."""
    specs = []
    for j in range(J):
        rng = np.random.default_rng(1000 + j)
        loss = int(rng.integers(0, 3))
        N = _scaled(int(rng.integers(50_000, 500_001)), scale)
        D = int(rng.choice([64, 128, 256, 512]))
        lam = float(10.0 ** rng.uniform(-6.0, -3.0))
        if loss == HINGE:
            eta = float(10.0 ** rng.uniform(-3.0, -2.0))
        else:
            eta = float(10.0 ** rng.uniform(-2.0, -1.0))
        specs.append(JobSpec(j, 1000 + j, loss, N, D, lam, eta))
    return specs


def config3_job(spec: JobSpec, device: str = "cpu") -> GLMProblem:
    return make_glm(spec.loss, spec.N, spec.D, spec.seed, lam=spec.lam, eta=spec.eta, K=0,
                    device=device, name=f"cfg3_job{spec.index}_{LOSS_NAMES[spec.loss]}_{spec.N}x{spec.D}")


def config3_alloc(epoch: int, J: int = 160) -> np.ndarray:
    """Allocation vector of one scheduling epoch: per-job iteration counts ~ U{1..8},
    seeded 2000 + epoch."""
    rng = np.random.default_rng(2000 + epoch)
    return rng.integers(1, 9, size=J).astype(np.int32)


@dataclass
class SweepProblem:
    """M models sharing one X: per-model lambda and step."""
    base: GLMProblem
    lams: np.ndarray = field(default_factory=lambda: np.zeros(0, np.float32))
    etas: np.ndarray = field(default_factory=lambda: np.zeros(0, np.float32))

    @property
    def M(self) -> int:
        return int(self.lams.shape[0])


def sweep_grid(n_lam: int = 8, n_eta: int = 8):
    """lambda log-spaced 1e-6..1e-1, step log-spaced 1e-3..1; model m = n_eta*i_lam + i_eta."""
    lam_axis = np.logspace(-6.0, -1.0, n_lam)
    eta_axis = np.logspace(-3.0, 0.0, n_eta)
    lams = np.repeat(lam_axis, n_eta).astype(np.float32)
    etas = np.tile(eta_axis, n_lam).astype(np.float32)
    return lams, etas


def config4(scale: float = 1.0, device: str = "cpu", D: int = 1024,
            n_lam: int = 8, n_eta: int = 8) -> SweepProblem:
    """Hyper-parameter sweep: 64 logistic models on one 1e6 x 1024 X, 30 iterations."""
    N = _scaled(1_000_000, scale)
    base = make_glm(LOGISTIC, N, D, 0, lam=0.0, eta=0.0, K=30, device=device,
                    name=f"cfg4_sweep_{N}x{D}_M{n_lam * n_eta}")
    lams, etas = sweep_grid(n_lam, n_eta)
    return SweepProblem(base, lams, etas)


# --------------------------------------------------------------------------- sparse inputs

@dataclass
class SparseGLMProblem:
    """A job whose X is sparse: the same matrix in CSR (rows) and CSC (columns) form."""
    name: str
    loss: int
    row_ptr: torch.Tensor    # [N+1] int64
    col_idx: torch.Tensor    # [nnz] int32
    row_val: torch.Tensor    # [nnz] fp32
    col_ptr: torch.Tensor    # [D+1] int64
    row_idx: torch.Tensor    # [nnz] int32
    col_val: torch.Tensor    # [nnz] fp32
    y: torch.Tensor          # [N] fp32
    w0: torch.Tensor         # [D] fp32
    N: int
    D: int
    lam: float
    eta: float
    K: int
    seed: int

    @property
    def nnz(self) -> int:
        return int(self.col_idx.shape[0])


def make_sparse_glm(loss: int, N: int, D: int, mean_nnz: float, seed: int, *, lam: float, eta: float,
                    K: int, skew: float = 3.0, device: str = "cpu", name: str = "") -> SparseGLMProblem:
    """Sparse stand-in for the paper's text / LIBSVM-style data (Sec. 3 "Setup"), whose shapes are
    not stated.  Row i stores n_i entries, n_i = round(mean_nnz * exp(0.5 g_i - 0.125)), g_i ~ N(0,1)
    (log-normal lengths, a few rows empty or long); each entry's column is floor(D * u**skew),
    u ~ U(0,1) (a few columns are very popular, most are rare, many are empty); values ~ N(0,1)
    scaled by 1/sqrt(mean_nnz) so margins stay O(1).  The columns of a row are stored in increasing
    order (canonical CSR).  A column may repeat inside a row; repeated
    entries add, in both layouts.  The CSC arrays are the same entries sorted by column with a
    stable sort, so a column lists its rows in increasing order.  Labels as in make_glm from
    w* ~ N(0,1) and noise of variance 0.1.  Draw order: lengths, columns, values, w*, noise."""
    if loss not in LOSS_NAMES:
        raise ValueError("unknown loss type")
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    ln = torch.randn(N, generator=g, device=dev, dtype=torch.float32)
    counts = torch.round(mean_nnz * torch.exp(0.5 * ln - 0.125)).to(torch.int64).clamp_(min=0)
    row_ptr = torch.zeros(N + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=row_ptr[1:])
    nnz = int(row_ptr[-1].item())
    u = torch.rand(nnz, generator=g, device=dev, dtype=torch.float32)
    col = torch.clamp((u.double() ** skew * D).to(torch.int64), max=D - 1)
    del u
    # canonical CSR: the columns of a row in increasing order (values are i.i.d., so they stay put)
    rows64 = torch.repeat_interleave(torch.arange(N, device=dev, dtype=torch.int64), counts)
    col = torch.sort(rows64 * D + col).values - rows64 * D
    del rows64
    val = torch.randn(nnz, generator=g, device=dev, dtype=torch.float32) / math.sqrt(max(mean_nnz, 1.0))
    w_star = torch.randn(D, generator=g, device=dev, dtype=torch.float32)
    noise = torch.randn(N, generator=g, device=dev, dtype=torch.float32) * math.sqrt(0.1)
    # margins by a prefix sum over the entries (deterministic, fp64)
    prod = val.double() * w_star.double()[col]
    pref = torch.zeros(nnz + 1, dtype=torch.float64, device=dev)
    torch.cumsum(prod, 0, out=pref[1:])
    m = pref[row_ptr[1:]] - pref[row_ptr[:-1]] + noise.double()
    del prod, pref
    if loss == LOGISTIC:
        y = (m > 0).to(torch.float32)
    elif loss == HINGE:
        y = torch.where(m >= 0, 1.0, -1.0).to(torch.float32)
    else:
        y = m.to(torch.float32)
    # the same entries by column
    order = torch.sort(col, stable=True).indices
    rows_of = torch.repeat_interleave(torch.arange(N, device=dev, dtype=torch.int32), counts)
    row_idx = rows_of[order].contiguous()
    col_val = val[order].contiguous()
    del rows_of, order
    col_ptr = torch.zeros(D + 1, dtype=torch.int64, device=dev)
    torch.cumsum(torch.bincount(col, minlength=D), 0, out=col_ptr[1:])
    return SparseGLMProblem(name or f"sparse_{LOSS_NAMES[loss]}_{N}x{D}_nnz{nnz}", loss, row_ptr,
                            col.to(torch.int32).contiguous(), val.contiguous(), col_ptr, row_idx, col_val,
                            y.contiguous(), torch.zeros(D, dtype=torch.float32, device=dev), N, D,
                            float(lam), float(eta), int(K), int(seed))


def sparse_config(scale: float = 1.0, device: str = "cpu") -> SparseGLMProblem:
    """The sparse measurement workload: logistic regression on 2,000,000 x 1,000,000 with about
    100 stored entries per row (about 2e8 entries, 1.6 GB per layout)."""
    N = max(1000, int(2_000_000 * scale))
    D = max(100, int(1_000_000 * scale))
    return make_sparse_glm(LOGISTIC, N, D, 100.0, 0, lam=1e-5, eta=0.5, K=20, device=device,
                           name=f"sparse_logistic_{N}x{D}")


@dataclass
class KMeansProblem:
    """A clustering job: points X [N, D] fp32 and the starting centroids C0 [K, D] fp32."""
    name: str
    X: torch.Tensor
    C0: torch.Tensor
    iters: int
    seed: int

    @property
    def N(self) -> int:
        return int(self.X.shape[0])

    @property
    def D(self) -> int:
        return int(self.X.shape[1])

    @property
    def K(self) -> int:
        return int(self.C0.shape[0])


def make_kmeans(N: int, D: int, K: int, seed: int, *, iters: int = 10, blobs: int = 0, spread: float = 3.0,
                offset: float = 0.0, device: str = "cpu", name: str = "") -> KMeansProblem:
    """Seeded Gaussian-mixture points: `blobs` (default K) true centres ~ N(0, (4 spread)^2 / D) per
    coordinate (centre-to-centre distance about 5.7 spread whatever D is, against a noise radius of
    sqrt(D)), uneven blob sizes (weights ~ u^2 + 0.05), unit-variance noise per coordinate, every
    coordinate shifted by `offset`.  The starting
    centroids are K distinct points of X picked by a seeded permutation (the random draw of the
    usual initialisation is an input of the method, not part of it)."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    B = blobs if blobs > 0 else K
    centres = torch.randn(B, D, generator=g, device=dev, dtype=torch.float32) * (spread / D ** 0.5) * 4.0
    wts = torch.rand(B, generator=g, device=dev, dtype=torch.float32) ** 2 + 0.05
    z = torch.multinomial(wts, N, replacement=True, generator=g)
    X = torch.empty(N, D, device=dev, dtype=torch.float32)
    step = max(1, (1 << 26) // max(D, 1))
    for i0 in range(0, N, step):
        i1 = min(N, i0 + step)
        X[i0:i1] = centres[z[i0:i1]] + torch.randn(i1 - i0, D, generator=g, device=dev, dtype=torch.float32)
    if offset != 0.0:
        X += offset
    pick = torch.randperm(N, generator=g, device=dev)[:K]
    C0 = X[pick].clone()
    return KMeansProblem(name or f"kmeans_{N}x{D}_k{K}", X, C0, iters, seed)


def kmeans_config(scale: float = 1.0, device: str = "cpu") -> KMeansProblem:
    """The clustering measurement workload: 4,000,000 points in 128 dimensions, 256 centroids."""
    return make_kmeans(max(1024, int(4_000_000 * scale)), 128, 256, 0, iters=10, device=device,
                       name=f"kmeans_{max(1024, int(4_000_000 * scale))}x128_k256")
