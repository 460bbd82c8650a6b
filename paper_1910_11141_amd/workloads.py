"""Seeded synthetic workloads: the five benchmark configurations, and the shape of the paper's own
logistic-regression experiment as a sixth.

This module only *generates inputs* (target data and sampler settings).  It
contains none of the sampler's arithmetic, and it is the one piece shared by
the HIP path and the CPU oracle: both are handed the very same arrays.

The paper's own test problems were synthetic and unspecified beyond their
shape (a correlated Gaussian in 100 dimensions; Bayesian logistic regression
on 10,000 synthetic points with 100 regressors; Section 4), so these
generators *are* the workloads; nothing stands in for a public dataset.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

STD_NORMAL, GAUSS_DENSE, GAUSS_DIAG, LOGREG = 0, 1, 2, 3
KIND_NAMES = {STD_NORMAL: "std_normal", GAUSS_DENSE: "gauss_dense", GAUSS_DIAG: "gauss_diag", LOGREG: "logreg"}

DATA_SEED_BASE = 1910_11141
SAMPLER_SEED = 12345


@dataclass
class Workload:
    name: str
    kind: int
    dim: int
    dtype: np.dtype
    n_chains: int
    n_iters: int
    step_size: float
    max_tree_depth: int
    seed: int = SAMPLER_SEED
    precision: np.ndarray | None = None   # GAUSS_DENSE: [dim, dim]
    scales: np.ndarray | None = None      # GAUSS_DIAG: sigma_i
    X: np.ndarray | None = None           # LOGREG: [n_data, dim]
    y: np.ndarray | None = None           # LOGREG: [n_data] in {0, 1}
    prior_scale: float = 1.0
    extras: dict = field(default_factory=dict)

    @property
    def n_data(self) -> int:
        return 0 if self.X is None else int(self.X.shape[0])


def ar1_precision(dim: int, rho: float) -> np.ndarray:
    """Inverse of Sigma_ij = rho^|i-j|: tridiagonal, written in closed form."""
    P = np.zeros((dim, dim), dtype=np.float64)
    s = 1.0 / (1.0 - rho * rho)
    idx = np.arange(dim)
    P[idx, idx] = (1.0 + rho * rho) * s
    P[0, 0] = P[-1, -1] = s
    if dim > 1:
        P[idx[:-1], idx[1:]] = -rho * s
        P[idx[1:], idx[:-1]] = -rho * s
    if dim == 1:
        P[0, 0] = 1.0
    return P


def logreg_data(n_data: int, dim: int, w_std: float, rng: np.random.Generator, standardize: bool):
    """dim-1 N(0,1) feature columns (optionally centred and scaled to unit sample
    std) plus a last column of ones; labels are Bernoulli(sigmoid(X w_true))."""
    F = rng.standard_normal((n_data, dim - 1))
    if standardize:
        F = (F - F.mean(axis=0)) / F.std(axis=0)
    X = np.concatenate([F, np.ones((n_data, 1))], axis=1)
    w_true = w_std * rng.standard_normal(dim)
    p = 1.0 / (1.0 + np.exp(-(X @ w_true)))
    y = (rng.random(n_data) < p).astype(np.float64)
    return X, y, w_true


def make(config: int, *, n_chains: int | None = None, n_iters: int | None = None) -> Workload:
    """Configuration 1..5 as listed in the benchmark definition (6: the paper's own experiment shape); chain
    and iteration counts can be reduced for tests (the data do not change)."""
    rng = np.random.default_rng(DATA_SEED_BASE + config)
    if config == 1:
        w = Workload("cfg1_std_normal_d2", STD_NORMAL, 2, np.dtype(np.float64), 4, 100, 0.5, 6)
    elif config == 2:
        w = Workload("cfg2_ar1_gauss_d100", GAUSS_DENSE, 100, np.dtype(np.float64), 1024, 1000, 0.1, 10,
                     precision=ar1_precision(100, 0.9))
    elif config == 3:
        X, y, wt = logreg_data(1000, 25, 1.0, rng, standardize=True)
        w = Workload("cfg3_logreg_1000x25", LOGREG, 25, np.dtype(np.float64), 4096, 1000, 0.05, 10, X=X, y=y,
                     extras={"w_true": wt})
    elif config == 4:
        X, y, wt = logreg_data(100000, 100, 0.5, rng, standardize=False)
        w = Workload("cfg4_logreg_100000x100", LOGREG, 100, np.dtype(np.float32), 256, 200, 0.005, 10,
                     X=X.astype(np.float32), y=y.astype(np.float32), extras={"w_true": wt})
    elif config == 5:
        sig = 10.0 ** (-2.0 + 4.0 * rng.random(1000))
        w = Workload("cfg5_diag_gauss_d1000", GAUSS_DIAG, 1000, np.dtype(np.float32), 16384, 500, 0.01, 10,
                     scales=sig.astype(np.float32))
    elif config == 6:
        # the shape of the experiment of Section 4.1 of the paper (binary32; the chain count is what it sweeps)
        X, y, wt = logreg_data(10000, 100, 0.5, rng, standardize=False)
        w = Workload("paper_logreg_10000x100", LOGREG, 100, np.dtype(np.float32), 1024, 100, 0.015, 10,
                     X=X.astype(np.float32), y=y.astype(np.float32), extras={"w_true": wt})
    else:
        raise ValueError(f"unknown config {config}")
    if n_chains is not None:
        w.n_chains = int(n_chains)
    if n_iters is not None:
        w.n_iters = int(n_iters)
    return w


def small_logreg(n_data: int, dim: int, seed: int, dtype=np.float64, w_std: float = 1.0) -> Workload:
    """A logistic-regression problem of arbitrary (small) shape for tests."""
    rng = np.random.default_rng(seed)
    X, y, wt = logreg_data(n_data, dim, w_std, rng, standardize=n_data > 2 and dim > 1)
    return Workload(f"logreg_{n_data}x{dim}", LOGREG, dim, np.dtype(dtype), 8, 10, 0.1, 6,
                    X=X.astype(dtype), y=y.astype(dtype), extras={"w_true": wt})


def random_spd_precision(dim: int, seed: int) -> np.ndarray:
    """A well-conditioned random symmetric positive-definite matrix."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((dim, dim))
    P = A @ A.T / dim + np.eye(dim)
    return 0.5 * (P + P.T)
