"""Seeded synthetic regression workloads (inputs only).

This module builds the arrays that BOTH the fp64 CPU oracle and the HIP library
are fed in tests and benchmarks: training inputs X, targets y, kernel
hyperparameters and the +-1 base noise for the probe vectors.  It contains none
of the method's arithmetic (no kernel evaluation, no solves) and imports
neither the oracle nor the HIP binding.

The recipes mirror the shape of the paper's regression experiments (tabular
regression, standardised features, Sec. "Results": t = 10 Rademacher probes,
rank-5 preconditioner, p = 20 iterations for the smallest case).  The paper's
UCI datasets are not available offline; these synthetic sets stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 180911165

RBF = 0
MATERN52 = 1

MATERIALISED = 0
ONTHEFLY = 1
SGPR = 2                        # subset-of-regressors covariance K_XU K_UU^-1 K_UX + sigma^2 I


@dataclass
class Workload:
    """One synthetic problem instance; every array is host memory."""

    name: str
    kernel: int                 # RBF or MATERN52
    X: np.ndarray               # (n, d) float32
    y: np.ndarray               # (n,) float32
    lengthscale: np.ndarray     # (1,) or (d,) float64 (ARD when d entries)
    outputscale: float
    noise: float                # sigma^2
    t: int                      # number of probe vectors
    k: int                      # preconditioner rank
    iters: int                  # mBCG iteration cap p
    tol: float                  # <= 0: run exactly `iters` iterations
    E1: np.ndarray              # (k, t) float32, entries +-1
    E2: np.ndarray              # (n, t) float32, entries +-1
    modes: tuple = (MATERIALISED, ONTHEFLY)
    meta: dict = field(default_factory=dict)
    Uind: Optional[np.ndarray] = None   # (m, d) float32 inducing inputs (SGPR workloads only)
    jitter_rel: float = 0.0             # K_UU gets jitter_rel * outputscale on its diagonal

    @property
    def n(self) -> int:
        return int(self.X.shape[0])

    @property
    def d(self) -> int:
        return int(self.X.shape[1])


def _streams(cfg: int, salt: int = 0):
    """Independent Philox sub-streams in the fixed order X, weights, noise, E2, E1."""
    root = np.random.SeedSequence([BASE_SEED + cfg, salt])
    return [np.random.Generator(np.random.Philox(s)) for s in root.spawn(5)]


def rademacher(rng: np.random.Generator, shape) -> np.ndarray:
    """i.i.d. +-1 entries as float32."""
    return (rng.integers(0, 2, size=shape, dtype=np.int8) * 2 - 1).astype(np.float32)


def _finish(name, kernel, X, y, ls, s, noise, t, k, iters, tol, rng_e2, rng_e1,
            modes=(MATERIALISED, ONTHEFLY), **meta) -> Workload:
    n = X.shape[0]
    E2 = rademacher(rng_e2, (n, t))
    E1 = rademacher(rng_e1, (max(k, 1), t))[:k]
    return Workload(name=name, kernel=kernel,
                    X=np.ascontiguousarray(X, dtype=np.float32),
                    y=np.ascontiguousarray(y, dtype=np.float32),
                    lengthscale=np.atleast_1d(np.asarray(ls, dtype=np.float64)),
                    outputscale=float(s), noise=float(noise), t=int(t), k=int(k),
                    iters=int(iters), tol=float(tol), E1=E1, E2=E2, modes=tuple(modes),
                    meta=dict(meta))


def config1(n: int = 1000, t: int = 10, k: int = 5, iters: int = 20, salt: int = 0) -> Workload:
    """RBF, d = 4, X ~ U[0,1]^d, y = sin(2 pi x.w) + 0.1 N(0,1); l = 0.3, s = 1, sigma^2 = 0.01."""
    rx, rw, rn, re2, re1 = _streams(1, salt)
    d = 4
    X = rx.random((n, d))
    w = rw.standard_normal(d)
    y = np.sin(2.0 * np.pi * (X @ w)) + 0.1 * rn.standard_normal(n)
    return _finish("cfg1_rbf_n%d_d4" % n, RBF, X, y, [0.3], 1.0, 0.01, t, k, iters, 0.0, re2, re1)


def config2(n: int = 10000, t: int = 10, k: int = 10, iters: int = 50, tol: float = 1e-2,
            salt: int = 0) -> Workload:
    """RBF, d = 8, X ~ N(0,I) standardised per column, y = sum_j sin(x_j) a_j + 0.05 N(0,1)."""
    rx, rw, rn, re2, re1 = _streams(2, salt)
    d = 8
    X = rx.standard_normal((n, d))
    X = (X - X.mean(axis=0)) / X.std(axis=0)
    a = rw.standard_normal(d)
    y = np.sin(X) @ a + 0.05 * rn.standard_normal(n)
    return _finish("cfg2_rbf_n%d_d8" % n, RBF, X, y, [1.0], 1.0, 0.05, t, k, iters, tol, re2, re1,
                   modes=(MATERIALISED, ONTHEFLY))


def config3(n: int = 50000, t: int = 10, k: int = 20, iters: int = 50, salt: int = 0) -> Workload:
    """Matern-5/2 ARD, d = 16, X ~ N(0,I), y from a random 2-layer tanh MLP (width 32) + 0.1 N(0,1)."""
    rx, rw, rn, re2, re1 = _streams(3, salt)
    d, width = 16, 32
    X = rx.standard_normal((n, d))
    W1 = rw.standard_normal((d, width)) / np.sqrt(d)
    b1 = rw.standard_normal(width)
    w2 = rw.standard_normal(width) / np.sqrt(width)
    ls = rw.uniform(0.5, 2.0, size=d)
    y = np.tanh(X @ W1 + b1) @ w2 + 0.1 * rn.standard_normal(n)
    return _finish("cfg3_matern52ard_n%d_d16" % n, MATERN52, X, y, ls, 1.0, 0.1, t, k, iters, 0.0,
                   re2, re1)


def config4(n: int = 200000, t: int = 16, k: int = 20, iters: int = 100, salt: int = 0) -> Workload:
    """RBF, d = 8, mixture of 20 Gaussian clusters (within-cluster sigma 0.3), smooth radial target."""
    rx, rw, rn, re2, re1 = _streams(4, salt)
    d, ncl = 8, 20
    centres = rw.standard_normal((ncl, d))
    lab = rx.integers(0, ncl, size=n)
    X = centres[lab] + 0.3 * rx.standard_normal((n, d))
    r = np.sqrt((X * X).sum(axis=1))
    y = np.sin(2.0 * r) / (1.0 + r) + 0.05 * rn.standard_normal(n)
    return _finish("cfg4_rbf_clusters_n%d_d8" % n, RBF, X, y, [1.0], 1.0, 0.05, t, k, iters, 0.0,
                   re2, re1, modes=(ONTHEFLY,))


def with_inducing(w: Workload, m: int, rng: np.random.Generator, jitter_rel: float = 1e-6) -> Workload:
    """Turns `w` into an SGPR workload: m inducing inputs = rows of X chosen by a seeded permutation."""
    rows = np.sort(rng.permutation(w.n)[:m])
    w.Uind = np.ascontiguousarray(w.X[rows])
    w.jitter_rel = float(jitter_rel)
    w.modes = (SGPR,)
    w.meta["inducing_rows"] = rows
    return w


def config5(n: int = 500000, m: int = 1024, t: int = 10, k: int = 10, iters: int = 50,
            salt: int = 0) -> Workload:
    """SGPR, RBF, d = 8, X ~ U[-1,1]^d, y = prod_j cos(x_j) + 0.1 N(0,1); l = 1, s = 1, sigma^2 = 0.01;
    m inducing inputs drawn from X; K_UU jitter 1e-6 s."""
    rx, rw, rn, re2, re1 = _streams(5, salt)
    d = 8
    X = rx.uniform(-1.0, 1.0, size=(n, d))
    y = np.prod(np.cos(X), axis=1) + 0.1 * rn.standard_normal(n)
    w = _finish("cfg5_sgpr_rbf_n%d_m%d_d8" % (n, m), RBF, X, y, [1.0], 1.0, 0.01, t, k, iters, 0.0,
                re2, re1)
    return with_inducing(w, m, rw)


def make(cfg: int, n: Optional[int] = None, **kw) -> Workload:
    """Workload `cfg` (1..5); `n` overrides the number of points, keeping the recipe."""
    fn = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}[cfg]
    if n is not None:
        kw["n"] = n
    return fn(**kw)


def tiny(n: int, d: int, kernel: int = RBF, ard: bool = False, t: int = 3, k: int = 2,
         iters: int = 5, noise: float = 0.1, seed: int = 0) -> Workload:
    """Small generic instance for identity / enumeration tests."""
    rx, rw, rn, re2, re1 = _streams(90 + kernel, 1000 * seed + n)
    X = rx.standard_normal((n, d))
    y = np.sin(X.sum(axis=1)) + 0.1 * rn.standard_normal(n)
    ls = rw.uniform(0.6, 1.6, size=d) if ard else np.array([0.9])
    return _finish("tiny_n%d_d%d" % (n, d), kernel, X, y, ls, 1.3, noise, t, k, iters, 0.0, re2, re1)


def tiny_sgpr(n: int, d: int, m: int, kernel: int = RBF, ard: bool = False, t: int = 3, k: int = 2,
              iters: int = 5, noise: float = 0.1, seed: int = 0, jitter_rel: float = 1e-6) -> Workload:
    """Small SGPR instance: `tiny` plus m inducing inputs drawn from its X."""
    w = tiny(n, d, kernel=kernel, ard=ard, t=t, k=k, iters=iters, noise=noise, seed=seed)
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([BASE_SEED + 95, seed, n, m])))
    return with_inducing(w, m, rng, jitter_rel)
