"""Hyperparameter learning on top of the BBMM call: Adam on the log of the raw hyperparameters,
driven by the stochastic NLML gradient that bbmm_solve_logdet_grad returns (Sec. 2, Eq. (2);
the paper trains with 20 mBCG iterations and a rank-5 preconditioner, Sec. "Results").

Host-side control only: every numerical step of an evaluation runs in the HIP library; this
module draws fresh +-1 base noise per step (seeded), applies the chain rule
d/d log(theta) = theta d/d theta and the Adam update, and keeps the trajectory.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

from . import binding, inputs


@dataclass
class Trajectory:
    lengthscale: List[np.ndarray] = field(default_factory=list)
    outputscale: List[float] = field(default_factory=list)
    noise: List[float] = field(default_factory=list)
    nlml: List[float] = field(default_factory=list)      # stochastic estimate of each step
    grad_norm: List[float] = field(default_factory=list)


def fit(ctx: "binding.Context", kernel: int, mode: int, X, y, lengthscale, outputscale: float,
        noise: float, steps: int = 30, lr: float = 0.1, t: int = 10, k: int = 5, iters: int = 20,
        seed: int = 0, device: str = "cuda:0") -> Trajectory:
    """Runs `steps` Adam updates (beta1 0.9, beta2 0.999) and returns the trajectory; its last
    entries are the learned hyperparameters.  X (n x d), y (n): host float32 arrays."""
    import torch
    dev = torch.device(device)
    Xd = torch.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).to(dev)
    yd = torch.from_numpy(np.ascontiguousarray(y, dtype=np.float32)).to(dev)
    n = Xd.shape[0]
    ls = np.atleast_1d(np.asarray(lengthscale, dtype=np.float64)).copy()
    nl = ls.shape[0]
    theta = np.log(np.concatenate([ls, [outputscale, noise]]))
    m1 = np.zeros_like(theta)
    m2 = np.zeros_like(theta)
    rng = np.random.Generator(np.random.Philox(inputs.BASE_SEED + 7919 * (seed + 1)))
    traj = Trajectory()
    for step in range(1, steps + 1):
        raw = np.exp(theta)
        E1 = torch.from_numpy(inputs.rademacher(rng, (max(k, 1), t))).to(dev)
        E2 = torch.from_numpy(inputs.rademacher(rng, (n, t))).to(dev)
        prob = binding.Problem(kernel=kernel, mode=mode, X=Xd, y=yd, lengthscale=raw[:nl].copy(),
                               outputscale=float(raw[nl]), noise=float(raw[nl + 1]), E1=E1, E2=E2, k=k,
                               max_iters=iters, tol=0.0)
        res = ctx.bbmm_solve_logdet_grad(prob, want_U=False)
        g = np.asarray(res.grad_nlml, dtype=np.float64) * raw          # chain rule to log-parameters
        traj.lengthscale.append(raw[:nl].copy())
        traj.outputscale.append(float(raw[nl]))
        traj.noise.append(float(raw[nl + 1]))
        traj.nlml.append(float(res.nlml))
        traj.grad_norm.append(float(np.linalg.norm(g)))
        m1 = 0.9 * m1 + 0.1 * g
        m2 = 0.999 * m2 + 0.001 * g * g
        theta = theta - lr * (m1 / (1 - 0.9 ** step)) / (np.sqrt(m2 / (1 - 0.999 ** step)) + 1e-8)
    raw = np.exp(theta)
    traj.lengthscale.append(raw[:nl].copy())
    traj.outputscale.append(float(raw[nl]))
    traj.noise.append(float(raw[nl + 1]))
    return traj
