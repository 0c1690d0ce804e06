"""fp64 CPU oracle for BBMM inference with the subset-of-regressors (SoR / SGPR) kernel
(arXiv 1809.11165, Sec. 5 "Programmability", paragraph on sparse GP regression).
TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's cpu_baseline
leg, never by the product path; shares no code with the HIP library.

The training covariance is replaced by

    K_hat = Q + sigma^2 I,    Q = K_XU K_UU^{-1} K_UX,

with m inducing inputs U.  Everything else of the method (rank-k pivoted Cholesky of the
noise-free matrix, here Q; probes from N(0,P); mBCG; Lanczos tridiagonals; SLQ log-det;
stochastic traces) is the paper's algorithm unchanged, so this file only supplies the operator,
its diagonal and rows (App. C, "time complexity": a row of Q costs O(nm)), its hyperparameter
derivatives, and the plain definitions to compare against:

  (I)  sor_exact_inference: Q formed densely, K_hat factorised by Cholesky (tiny n), and
       sor_woodbury: the same solve and log-determinant through the m x m matrix
       sigma^2 K_UU + K_UX K_XU (matrix inversion and determinant lemmas), usable at full size;
  (II) sor_bbmm_inference: the paper's algorithm with matrix products "distributed and grouped"
       as the paragraph says, K_XU (K_UU^{-1} (K_UX M)) + sigma^2 M.

Readings where the paper is silent:
  * K_UU gets the diagonal jitter  jitter_rel * s  (s the outputscale) before it is factorised;
    because the jitter scales with s, Q is exactly linear in s and dQ/ds = Q/s.
  * The inducing inputs are fixed (a subset of X drawn by the input recipe), not hyperparameters.
  * Derivative of Q for a kernel hyperparameter theta (product rule, dA^{-1} = -A^{-1} dA A^{-1}):
        dQ = dK_XU Kinv K_UX + K_XU Kinv dK_UX - K_XU Kinv dK_UU Kinv K_UX.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional, Sequence

import numpy as np
import scipy.linalg as sla

from . import bbmm_oracle as O


@dataclass
class SorParts:
    """The pieces every SoR computation is made of (all fp64)."""
    KXU: np.ndarray        # n x m
    KUU: np.ndarray        # m x m, jitter included
    chol_UU: np.ndarray    # lower Cholesky factor of KUU
    noise: float

    def kuu_solve(self, M: np.ndarray) -> np.ndarray:
        return sla.cho_solve((self.chol_UU, True), M)

    def q_matmul(self, M: np.ndarray) -> np.ndarray:
        """Q M, grouped right to left: K_XU (K_UU^{-1} (K_UX M)), O(nm) per column."""
        return self.KXU @ self.kuu_solve(self.KXU.T @ M)

    def khat_matmul(self, M: np.ndarray) -> np.ndarray:
        return self.q_matmul(M) + self.noise * M

    def q_diag(self) -> np.ndarray:
        """Q_ii = k_{U x_i}^T K_UU^{-1} k_{U x_i}."""
        return np.sum(self.KXU * self.kuu_solve(self.KXU.T).T, axis=1)

    def q_row(self, i: int) -> np.ndarray:
        return self.KXU @ self.kuu_solve(self.KXU[i])


def sor_parts(kernel: int, X, Uind, ls, s: float, noise: float, jitter_rel: float) -> SorParts:
    X = np.asarray(X, dtype=np.float64)
    Uind = np.asarray(Uind, dtype=np.float64)
    KXU = O.kernel_block(kernel, X, Uind, ls, s)
    KUU = O.kernel_block(kernel, Uind, Uind, ls, s)
    KUU[np.diag_indices(Uind.shape[0])] += jitter_rel * s
    return SorParts(KXU=KXU, KUU=KUU, chol_UU=sla.cholesky(KUU, lower=True), noise=float(noise))


def sor_dense_q(parts: SorParts) -> np.ndarray:
    """Q as a dense n x n matrix (small n only): the definition, K_XU K_UU^{-1} K_UX."""
    return parts.KXU @ np.linalg.solve(parts.KUU, parts.KXU.T)


def sor_khat_derivatives(kernel: int, X, Uind, ls, s: float, jitter_rel: float) -> list:
    """Dense dK_hat/dtheta_h for lengthscale(s), outputscale, noise (small n only)."""
    X = np.asarray(X, dtype=np.float64)
    Uind = np.asarray(Uind, dtype=np.float64)
    n, m = X.shape[0], Uind.shape[0]
    KXU = O.kernel_block(kernel, X, Uind, ls, s)
    KUU = O.kernel_block(kernel, Uind, Uind, ls, s) + jitter_rel * s * np.eye(m)
    A = np.linalg.solve(KUU, KXU.T)                        # K_UU^{-1} K_UX, m x n
    dXU = O.kernel_derivative_blocks(kernel, X, Uind, ls, s)
    dUU = O.kernel_derivative_blocks(kernel, Uind, Uind, ls, s)
    dUU[-1] = dUU[-1] + jitter_rel * np.eye(m)             # the jitter is jitter_rel * s
    mats = []
    for dxu, duu in zip(dXU, dUU):
        first = dxu @ A
        mats.append(first + first.T - A.T @ duu @ A)
    mats.append(np.eye(n))
    return mats


def sor_exact_inference(kernel: int, X, Uind, y, ls, s: float, noise: float, jitter_rel: float,
                        with_traces: bool = True) -> O.ExactResult:
    """Plain definition: dense K_hat = Q + sigma^2 I, Cholesky (Sec. 3, "Required operations")."""
    y = np.asarray(y, dtype=np.float64)
    n = y.shape[0]
    parts = sor_parts(kernel, X, Uind, ls, s, noise, jitter_rel)
    Khat = sor_dense_q(parts) + noise * np.eye(n)
    Khat = 0.5 * (Khat + Khat.T)
    u0, logdet, factor = O.exact_solve_logdet(Khat, y)
    yKinvy = float(y @ u0)
    if with_traces:
        Kinv = sla.cho_solve(factor, np.eye(n))
        mats = sor_khat_derivatives(kernel, X, Uind, ls, s, jitter_rel)
        trace = np.array([np.sum(Kinv * M) for M in mats])
        quad = np.array([u0 @ (M @ u0) for M in mats])
    else:
        trace = np.zeros(0)
        quad = np.zeros(0)
    return O.ExactResult(u0=u0, logdet=float(logdet), yKinvy=yKinvy, trace=trace, quad=quad,
                         nlml=O.nlml_from_terms(yKinvy, logdet, n), grad=0.5 * (trace - quad))


def sor_woodbury(parts: SorParts, y: np.ndarray):
    """K_hat^{-1} y and log|K_hat| in O(n m^2) through B = sigma^2 K_UU + K_UX K_XU:
        K_hat^{-1} = (I - K_XU B^{-1} K_UX) / sigma^2,
        log|K_hat| = log|B| - log|K_UU| + (n - m) log sigma^2.
    Returns (u0, logdet)."""
    y = np.asarray(y, dtype=np.float64)
    n, m = parts.KXU.shape
    B = parts.noise * parts.KUU + parts.KXU.T @ parts.KXU
    GB = sla.cholesky(B, lower=True)
    u0 = (y - parts.KXU @ sla.cho_solve((GB, True), parts.KXU.T @ y)) / parts.noise
    logdet = (2.0 * np.sum(np.log(np.diag(GB))) - 2.0 * np.sum(np.log(np.diag(parts.chol_UU)))
              + (n - m) * np.log(parts.noise))
    return u0, float(logdet)


def sor_derivative_matvec(kernel: int, X, Uind, ls, s: float, jitter_rel: float, parts: SorParts,
                          W: np.ndarray, row_chunk: int = 16384) -> list:
    """[(dQ/dtheta_h) W for every kernel hyperparameter h] (lengthscale(s), outputscale), each
    n x c, matrix-free: the three terms of dQ applied right to left, with the n x m derivative
    blocks formed a block of rows at a time."""
    X = np.asarray(X, dtype=np.float64)
    Uind = np.asarray(Uind, dtype=np.float64)
    ls = np.atleast_1d(np.asarray(ls, dtype=np.float64))
    W = np.asarray(W, dtype=np.float64)
    m = Uind.shape[0]
    n = X.shape[0]
    H = ls.shape[0] + 1
    AW = parts.kuu_solve(parts.KXU.T @ W)              # K_UU^{-1} K_UX W, m x c
    out = [np.empty((n, W.shape[1])) for _ in range(H)]
    dKW = [np.zeros((m, W.shape[1])) for _ in range(H)]      # dK_UX W, summed over the row blocks
    for a in range(0, n, row_chunk):
        b = min(n, a + row_chunk)
        dXU = O.kernel_derivative_blocks(kernel, X[a:b], Uind, ls, s)
        for h in range(H):
            out[h][a:b] = dXU[h] @ AW                        # dK_XU (Kinv K_UX W)
            dKW[h] += dXU[h].T @ W[a:b]
    dUU = O.kernel_derivative_blocks(kernel, Uind, Uind, ls, s)
    dUU[-1] = dUU[-1] + jitter_rel * np.eye(m)
    for h in range(H):
        # + K_XU Kinv (dK_UX W) - K_XU Kinv dK_UU (Kinv K_UX W)
        out[h] += parts.KXU @ parts.kuu_solve(dKW[h] - dUU[h] @ AW)
    return out


def sor_derivative_products(kernel: int, X, Uind, ls, s: float, jitter_rel: float, parts: SorParts,
                            Ucols: np.ndarray, Wcols: np.ndarray, row_chunk: int = 16384):
    """sum_c Ucols[:, c]^T (dQ/dtheta_h) Wcols[:, c] for every kernel hyperparameter
    (lengthscale(s), outputscale)."""
    MW = sor_derivative_matvec(kernel, X, Uind, ls, s, jitter_rel, parts, Wcols, row_chunk)
    return np.array([np.sum(np.asarray(Ucols, dtype=np.float64) * M) for M in MW])


def sor_term_sensitivity(kernel: int, X, Uind, ls, s: float, jitter_rel: float, parts: SorParts,
                         U: np.ndarray, W: np.ndarray):
    """First-order bounds on how far the trace and quadratic terms can move when the solves move:
    if every column u_i changes by at most eps |u_i| (W = P^{-1} Z is fixed), then
        |delta trace_h| <= eps * (1/t) sum_i |u_i| |M_h w_i|,
        |delta quad_h|  <= eps * 2 |u_0| |M_h u_0|          (plus O(eps^2)),
    by Cauchy-Schwarz.  U: n x (t+1) (column 0 = u_0), W: n x t.  Returns (trace_sens, quad_sens),
    one entry per hyperparameter, noise (M = I) last.  Test infrastructure: the parity tests use it
    to turn the bound on the iterate into a bound on terms that cancel heavily."""
    U = np.asarray(U, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    t = W.shape[1]
    norm = lambda A: np.linalg.norm(A, axis=0)
    MW = sor_derivative_matvec(kernel, X, Uind, ls, s, jitter_rel, parts, W) + [W]
    Mu = sor_derivative_matvec(kernel, X, Uind, ls, s, jitter_rel, parts, U[:, :1]) + [U[:, :1]]
    tr = np.array([np.sum(norm(U[:, 1:]) * norm(M)) / t for M in MW])
    qd = np.array([2.0 * norm(U[:, :1])[0] * norm(M)[0] for M in Mu])
    return tr, qd


def sor_bbmm_inference(kernel: int, X, Uind, y, ls, s: float, noise: float, jitter_rel: float,
                       E1, E2, k: int, p: int, tol: float = 0.0,
                       forced_pivots: Optional[Sequence[int]] = None,
                       progress: Optional[Callable[[str], None]] = None,
                       via_root: bool = False) -> O.BbmmResult:
    """One BBMM call on the SoR covariance: the steps of bbmm_oracle.bbmm_inference with the
    operator, diagonal, rows and derivative products of Q.

    via_root=True forms the products of the iteration as A (A^T M) with A = K_XU G^{-T},
    K_UU = G G^T -- the same operator in another fp64 rounding order.  Tests use the distance
    between the two runs as the measure of how sharply a quantity is defined at an unconverged
    iteration count."""
    say = progress if progress is not None else (lambda msg: None)
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    ls = np.atleast_1d(np.asarray(ls, dtype=np.float64))
    n = X.shape[0]
    t = np.asarray(E2).shape[1]
    parts = sor_parts(kernel, X, Uind, ls, s, noise, jitter_rel)
    say("K_XU, K_UU ready")

    L, pivots, dmax = O.pivoted_cholesky(parts.q_diag(), parts.q_row, k, forced_pivots)
    P = O.make_preconditioner(L, noise)
    Zp = O.make_probes(L, noise, np.asarray(E1)[:L.shape[1]], E2)
    B = np.concatenate([y[:, None], Zp], axis=1)
    say("preconditioner and probes ready")

    matmul = parts.khat_matmul
    if via_root:
        A = sla.solve_triangular(parts.chol_UU, parts.KXU.T, lower=True).T
        matmul = lambda M: A @ (A.T @ M) + noise * M
    res = O.mbcg(matmul, B, P.solve, p, tol)
    say("mBCG done: %d iterations" % res.iters_run)

    terms = np.zeros(t)
    for i in range(t):
        col = i + 1
        mv = int(res.m_valid[col])
        dg, off = O.tridiag_from_cg(res.alpha[:, col], res.beta[:, col], mv)
        terms[i] = res.rho0[col] * O.e1_logT_e1(dg, off)
    logdet = P.logdet + float(np.mean(terms))

    U = res.U
    u0 = U[:, 0]
    W = res.Z0[:, 1:]
    trace = list(sor_derivative_products(kernel, X, Uind, ls, s, jitter_rel, parts, U[:, 1:], W) / t)
    quad = list(sor_derivative_products(kernel, X, Uind, ls, s, jitter_rel, parts, u0[:, None], u0[:, None]))
    trace.append(float(np.sum(U[:, 1:] * W) / t))     # dK_hat/dsigma^2 = I
    quad.append(float(u0 @ u0))
    trace = np.array(trace)
    quad = np.array(quad)
    yKinvy = float(y @ u0)
    return O.BbmmResult(u0=u0, U=U, W=W, logdet=logdet, logdet_precond=P.logdet, slq_terms=terms,
                        yKinvy=yKinvy, trace=trace, quad=quad,
                        nlml=O.nlml_from_terms(yKinvy, logdet, n), grad=0.5 * (trace - quad),
                        L=L, pivots=pivots, pivot_dmax=dmax, mbcg=res, B=B)


# ----------------------------------------------------------------------------
# Predictive distribution at test inputs under the SoR prior (Sec. 2, Eq. (1), with every
# covariance replaced by its subset-of-regressors form q(a, b) = k_{aU} K_UU^{-1} k_{Ub}):
#   mean(x*)     = q_{x* X} K_hat^{-1} y
#   var(x*)      = q(x*, x*) - q_{x* X} K_hat^{-1} q_{X x*}          (latent f; add sigma^2 for y)
# ----------------------------------------------------------------------------
def sor_cross(kernel: int, Xs, Uind, ls, s: float, parts: SorParts):
    """(Q_{X x*} as an n x ns matrix, q(x*, x*) as ns values)."""
    Xs = np.asarray(Xs, dtype=np.float64)
    Uind = np.asarray(Uind, dtype=np.float64)
    KUs = O.kernel_block(kernel, Uind, Xs, ls, s)                   # m x ns
    W = parts.kuu_solve(KUs)
    return parts.KXU @ W, np.sum(KUs * W, axis=0)


def sor_exact_predict(kernel: int, X, Uind, y, ls, s: float, noise: float, jitter_rel: float, Xs):
    """The plain definition through the dense Cholesky factor of K_hat = Q + sigma^2 I (small n).
    Returns (mean, var)."""
    y = np.asarray(y, dtype=np.float64)
    parts = sor_parts(kernel, X, Uind, ls, s, noise, jitter_rel)
    n = y.shape[0]
    Khat = sor_dense_q(parts) + noise * np.eye(n)
    Khat = 0.5 * (Khat + Khat.T)
    QXs, qss = sor_cross(kernel, Xs, Uind, ls, s, parts)
    u0, _, factor = O.exact_solve_logdet(Khat, y)
    mean = QXs.T @ u0
    var = qss - np.sum(QXs * sla.cho_solve(factor, QXs), axis=0)
    return mean, var


def sor_bbmm_predict(kernel: int, X, Uind, ls, s: float, noise: float, jitter_rel: float, Xs,
                     u0: np.ndarray, P: "O.Preconditioner", p: int, tol: float = 0.0):
    """The same two quantities the way the method obtains them: the mean from a solve u0 that is
    already there, the variances from one more preconditioned mBCG run (Alg. 2) whose right-hand
    sides are the columns Q_{X x*}.  Returns (mean, var, MbcgResult)."""
    parts = sor_parts(kernel, X, Uind, ls, s, noise, jitter_rel)
    QXs, qss = sor_cross(kernel, Xs, Uind, ls, s, parts)
    mean = QXs.T @ np.asarray(u0, dtype=np.float64)
    res = O.mbcg(parts.khat_matmul, QXs, P.solve, p, tol)
    var = qss - np.sum(QXs * res.U, axis=0)
    return mean, var, res
