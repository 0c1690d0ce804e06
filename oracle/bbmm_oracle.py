"""fp64 CPU oracle for BBMM inference (arXiv 1809.11165).  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct numpy code written from the paper.  It shares no
code with the HIP library and must only be imported by tests, the smoke check
and the benchmark's cpu_baseline leg.

Two halves:
  (I)  exact_inference: the plain definition -- dense Cholesky of K_hat gives
       K_hat^{-1} y, log|K_hat| and Tr(K_hat^{-1} dK_hat/dtheta)  (Sec. 3,
       "Required operations"; Eq. (2) for the loss and its derivative).
  (II) bbmm_inference: the paper's algorithm step by step -- rank-k pivoted
       Cholesky (App. C), Woodbury solve and determinant lemma (App. C), probes
       z = L e1 + sigma e2 (App. C, "drawing samples"), preconditioned mBCG
       (Alg. 2), Lanczos tridiagonals from the CG coefficients (Observation 3 in
       App. A), stochastic Lanczos quadrature for log|K_hat| (Eq. (5) with the
       preconditioned form Eq. (7) and the log|P| correction) and the stochastic
       trace estimate with preconditioned probes (Eq. (8)).

Readings of passages where the printed text is garbled or silent (all pinned by
tests/test_oracle_pins.py):
  * RBF kernel uses the squared distance, s exp(-|x-x'|^2 / (2 l^2)).
  * Alg. 1/2 follow the textbook PCG the paper cites: r0 = b - A u0,
    d <- z + beta d, beta = r_j.z_j / r_{j-1}.z_{j-1}.
  * T off-diagonal is sqrt(beta_{j-1}) / alpha_{j-1} (the Observation's matrix).
  * Woodbury / determinant lemma use (I + L^T L / sigma^2), i.e. the capacitance
    matrix C = sigma^2 I + L^T L.
  * Each SLQ term carries |P^{-1/2} z_i|^2 = z_i^T P^{-1} z_i, and the sum over
    probes is a mean.
  * Loss is the standard negative log marginal likelihood
    1/2 (y^T K_hat^{-1} y + log|K_hat| + n log 2 pi); gradient 1/2 (Tr - quad).
  * Matern-5/2 with ARD lengthscales in the Rasmussen-Williams form.
  * Probes are built from +-1 base noise (the experiments' Rademacher probes)
    through the reparameterisation z = L e1 + sigma e2, which has mean 0 and
    covariance exactly P.
  * Pivot ties: lowest index wins.
  * Stop rule: relative recurrence residual |r_j| / |b| < tol for ALL columns,
    tested after alpha_j is recorded; tol <= 0 runs exactly p iterations.
  * A column whose rho or d^T K d becomes non-positive or non-finite is frozen
    (alpha = beta = 0 afterwards, its tridiagonal truncated).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional, Sequence

import numpy as np
import scipy.linalg as sla

RBF = 0
MATERN52 = 1
SQRT5 = np.sqrt(5.0)


# ----------------------------------------------------------------------------
# Kernel functions and their hyperparameter derivatives (Sec. 2, "Notation").
# Hyperparameter order everywhere: lengthscale(s) (1 or d), outputscale, noise.
# ----------------------------------------------------------------------------
def _scaled_sqdist(Xa: np.ndarray, Xb: np.ndarray, ls: np.ndarray) -> np.ndarray:
    """rho^2_ij = sum_d ((xa_id - xb_jd) / l_d)^2 by explicit differences."""
    d = Xa.shape[1]
    l = np.broadcast_to(np.asarray(ls, dtype=np.float64), (d,))
    out = np.zeros((Xa.shape[0], Xb.shape[0]))
    for q in range(d):
        diff = (Xa[:, q:q + 1] - Xb[None, :, q]) / l[q]
        out += diff * diff
    return out


def kernel_block(kernel: int, Xa, Xb, ls, s: float) -> np.ndarray:
    """k(xa_i, xb_j) for all pairs; no noise term."""
    Xa = np.asarray(Xa, dtype=np.float64)
    Xb = np.asarray(Xb, dtype=np.float64)
    rho2 = _scaled_sqdist(Xa, Xb, ls)
    if kernel == RBF:
        return s * np.exp(-0.5 * rho2)
    if kernel == MATERN52:
        rho = np.sqrt(rho2)
        return s * (1.0 + SQRT5 * rho + (5.0 / 3.0) * rho2) * np.exp(-SQRT5 * rho)
    raise ValueError("unknown kernel")


def kernel_matrix(kernel: int, X, ls, s: float, row_chunk: int = 2048) -> np.ndarray:
    """K_XX (n x n).  Rows are produced in chunks only to bound temporaries."""
    X = np.asarray(X, dtype=np.float64)
    n = X.shape[0]
    K = np.empty((n, n))
    for a in range(0, n, row_chunk):
        K[a:a + row_chunk] = kernel_block(kernel, X[a:a + row_chunk], X, ls, s)
    return K


def kernel_derivative_blocks(kernel: int, Xa, Xb, ls, s: float) -> list:
    """[dK/dl_1..dK/dl_L, dK/ds] for the block (Xa, Xb); L = len(ls) (1 or d).

    RBF:      dk/dl_d = k * Delta_d^2 / l_d^3          (sum over d when isotropic)
    Matern52: dk/dl_d = s (5/3)(1 + sqrt5 rho) exp(-sqrt5 rho) * Delta_d^2 / l_d^3
    both:     dk/ds   = k / s
    """
    Xa = np.asarray(Xa, dtype=np.float64)
    Xb = np.asarray(Xb, dtype=np.float64)
    ls = np.atleast_1d(np.asarray(ls, dtype=np.float64))
    d = Xa.shape[1]
    l = np.broadcast_to(ls, (d,))
    rho2 = _scaled_sqdist(Xa, Xb, ls)
    if kernel == RBF:
        K = s * np.exp(-0.5 * rho2)
        g = K
    elif kernel == MATERN52:
        rho = np.sqrt(rho2)
        e = np.exp(-SQRT5 * rho)
        K = s * (1.0 + SQRT5 * rho + (5.0 / 3.0) * rho2) * e
        g = s * (5.0 / 3.0) * (1.0 + SQRT5 * rho) * e
    else:
        raise ValueError("unknown kernel")
    per_dim = []
    for q in range(d):
        diff = Xa[:, q:q + 1] - Xb[None, :, q]
        per_dim.append(g * diff * diff / l[q] ** 3)
    if ls.shape[0] == 1:
        out = [sum(per_dim)]
    else:
        out = per_dim
    out.append(K / s)
    return out


def khat_derivatives(kernel: int, X, ls, s: float) -> list:
    """Dense dK_hat/dtheta_h for every hyperparameter, noise last (= identity)."""
    n = np.asarray(X).shape[0]
    mats = kernel_derivative_blocks(kernel, X, X, ls, s)
    mats.append(np.eye(n))
    return mats


# ----------------------------------------------------------------------------
# (I) Plain definition through a dense Cholesky factorisation.
# ----------------------------------------------------------------------------
@dataclass
class ExactResult:
    u0: np.ndarray
    logdet: float
    yKinvy: float
    trace: np.ndarray       # Tr(K_hat^{-1} dK_hat/dtheta_h)
    quad: np.ndarray        # u0^T (dK_hat/dtheta_h) u0
    nlml: float
    grad: np.ndarray        # d nlml / d theta_h


def nlml_from_terms(yKinvy: float, logdet: float, n: int) -> float:
    return 0.5 * (yKinvy + logdet + n * np.log(2.0 * np.pi))


def exact_solve_logdet(Khat: np.ndarray, y: np.ndarray, overwrite: bool = False):
    """K_hat^{-1} y and log|K_hat| = 2 sum_i log G_ii from the dense Cholesky factor K_hat = G G^T
    (Sec. 3, "Required operations").  Returns (u0, logdet, factor) with `factor` in the form
    scipy.linalg.cho_solve takes.

    overwrite=True factorises in the memory of Khat (for matrices that fit only once): the
    transposed view of the symmetric row-major array is column-major, and its upper factor G^T
    lands where K_hat was."""
    if overwrite:
        factor = (sla.cholesky(Khat.T, lower=False, overwrite_a=True, check_finite=False), False)
    else:
        factor = (sla.cholesky(Khat, lower=True), True)
    u0 = sla.cho_solve(factor, y)
    logdet = 2.0 * np.sum(np.log(np.diag(factor[0])))
    return u0, float(logdet), factor


def exact_solve_logdet_blocked(Khat: np.ndarray, y: np.ndarray, block: int = 4096):
    """The same two quantities for matrices with more than 2^31 entries, which the LAPACK build
    behind scipy does not factorise in one call: textbook right-looking blocked Cholesky in the
    lower triangle of Khat (overwritten), then blocked forward and back substitution.
    Returns (u0, logdet)."""
    n = Khat.shape[0]
    for j0 in range(0, n, block):
        j1 = min(n, j0 + block)
        G11 = sla.cholesky(Khat[j0:j1, j0:j1], lower=True)
        Khat[j0:j1, j0:j1] = G11
        if j1 < n:
            # G21 = A21 G11^{-T}
            G21 = sla.solve_triangular(G11, Khat[j1:, j0:j1].T, lower=True, check_finite=False).T
            Khat[j1:, j0:j1] = G21
            # trailing matrix, lower part: A22 -= G21 G21^T
            for i0 in range(j1, n, block):
                i1 = min(n, i0 + block)
                Khat[i0:i1, j1:i1] -= G21[i0 - j1:i1 - j1] @ G21[:i1 - j1].T
    logdet = 2.0 * float(np.sum(np.log(np.diag(Khat))))
    w = np.array(y, dtype=np.float64)
    for j0 in range(0, n, block):                       # G w = y
        j1 = min(n, j0 + block)
        w[j0:j1] = sla.solve_triangular(Khat[j0:j1, j0:j1], w[j0:j1], lower=True, check_finite=False)
        if j1 < n:
            w[j1:] -= Khat[j1:, j0:j1] @ w[j0:j1]
    starts = list(range(0, n, block))
    for j0 in reversed(starts):                         # G^T u = w
        j1 = min(n, j0 + block)
        if j1 < n:
            w[j0:j1] -= Khat[j1:, j0:j1].T @ w[j1:]
        w[j0:j1] = sla.solve_triangular(Khat[j0:j1, j0:j1], w[j0:j1], lower=True, trans='T',
                                        check_finite=False)
    return w, logdet


def exact_inference(kernel: int, X, y, ls, s: float, noise: float,
                    with_traces: bool = True) -> ExactResult:
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n = X.shape[0]
    Khat = kernel_matrix(kernel, X, ls, s)
    Khat[np.diag_indices(n)] += noise
    u0, logdet, factor = exact_solve_logdet(Khat, y)
    G = factor[0]
    yKinvy = float(y @ u0)
    if with_traces:
        Kinv = sla.cho_solve((G, True), np.eye(n))
        mats = khat_derivatives(kernel, X, ls, s)
        trace = np.array([np.sum(Kinv * M) for M in mats])
        quad = np.array([u0 @ (M @ u0) for M in mats])
    else:
        trace = np.zeros(0)
        quad = np.zeros(0)
    return ExactResult(u0=u0, logdet=float(logdet), yKinvy=yKinvy, trace=trace, quad=quad,
                       nlml=nlml_from_terms(yKinvy, logdet, n), grad=0.5 * (trace - quad))


# ----------------------------------------------------------------------------
# (II) The paper's algorithm.
# ----------------------------------------------------------------------------
def pivoted_cholesky(diag: np.ndarray, get_row: Callable[[int], np.ndarray], k: int,
                     forced_pivots: Optional[Sequence[int]] = None, rel_stop: float = 1e-12):
    """Rank-k pivoted Cholesky of a PSD matrix (App. C).

    diag    -- the matrix diagonal
    get_row -- get_row(i) returns row i of the matrix
    Returns L (n x k, original row order), pivots, and the residual-diagonal
    maximum seen at each step (before the pivot is eliminated).
    Greedy rule: the pivot is the largest remaining residual diagonal, lowest
    index on ties; `forced_pivots` replays a given pivot order instead.
    """
    delta = np.array(diag, dtype=np.float64)
    n = delta.shape[0]
    L = np.zeros((n, k))
    picked = np.zeros(n, dtype=bool)
    pivots = []
    dmax_hist = []
    d0 = float(delta.max()) if n else 0.0
    for m in range(k):
        masked = np.where(picked, -np.inf, delta)
        best = int(np.argmax(masked))          # first occurrence == lowest index
        dmax_hist.append(float(masked[best]))
        piv = int(forced_pivots[m]) if forced_pivots is not None else best
        if delta[piv] <= rel_stop * d0:
            L = L[:, :m]
            break
        pivots.append(piv)
        root = np.sqrt(delta[piv])
        row = np.asarray(get_row(piv), dtype=np.float64)
        col = (row - L[:, :m] @ L[piv, :m]) / root
        col[picked] = 0.0
        col[piv] = root
        L[:, m] = col
        delta = delta - col * col
        picked[piv] = True
        delta[picked] = 0.0
    return L, np.array(pivots, dtype=np.int64), np.array(dmax_hist)


@dataclass
class Preconditioner:
    """P = L L^T + sigma^2 I through its k x k capacitance matrix (App. C)."""
    L: np.ndarray
    noise: float
    chol_C: Optional[np.ndarray]   # lower Cholesky factor of C = sigma^2 I + L^T L
    logdet: float                  # log|P| by the determinant lemma

    def solve(self, R: np.ndarray) -> np.ndarray:
        if self.L.shape[1] == 0:
            return R / self.noise
        q = sla.cho_solve((self.chol_C, True), self.L.T @ R)
        return (R - self.L @ q) / self.noise


def make_preconditioner(L: np.ndarray, noise: float) -> Preconditioner:
    n, k = L.shape
    if k == 0:
        return Preconditioner(L=L, noise=noise, chol_C=None, logdet=n * np.log(noise))
    C = noise * np.eye(k) + L.T @ L
    G = sla.cholesky(C, lower=True)
    # |L L^T + s2 I| = |I_k + L^T L / s2| * s2^n = |C| * s2^(n-k)
    logdet = 2.0 * np.sum(np.log(np.diag(G))) + (n - k) * np.log(noise)
    return Preconditioner(L=L, noise=noise, chol_C=G, logdet=float(logdet))


def make_probes(L: np.ndarray, noise: float, E1: np.ndarray, E2: np.ndarray) -> np.ndarray:
    """z_i = L e1_i + sigma e2_i, columns i = 1..t (covariance L L^T + sigma^2 I)."""
    E1 = np.asarray(E1, dtype=np.float64)
    E2 = np.asarray(E2, dtype=np.float64)
    Z = np.sqrt(noise) * E2
    if L.shape[1]:
        Z = Z + L @ E1
    return Z


@dataclass
class MbcgResult:
    U: np.ndarray            # n x c solves
    alpha: np.ndarray        # iters_run x c
    beta: np.ndarray         # iters_run x c
    resid: np.ndarray        # iters_run x c relative recurrence residuals |r_j|/|b|
    iters_run: int
    Z0: np.ndarray           # P^{-1} B (first preconditioned residual)
    rho0: np.ndarray         # b^T P^{-1} b per column
    m_valid: np.ndarray      # per column: number of iterations with valid coefficients


def mbcg(matmul: Callable[[np.ndarray], np.ndarray], B: np.ndarray,
         psolve: Callable[[np.ndarray], np.ndarray], p: int, tol: float = 0.0,
         U0: Optional[np.ndarray] = None) -> MbcgResult:
    """Modified batched preconditioned CG (Alg. 2) on the n x c block B.

    Every column runs its own PCG recurrence with its own alpha_j, beta_j; the
    coefficients are kept so that the Lanczos tridiagonals can be rebuilt.
    U0: the current solutions the algorithm takes as input (first line of Alg. 1/2:
    r_0 = b - A u_0); None = zero.  Residuals stay relative to |b|.
    """
    B = np.asarray(B, dtype=np.float64)
    n, c = B.shape
    if U0 is None:
        U = np.zeros((n, c))
        R = B.copy()
    else:
        U = np.array(U0, dtype=np.float64)
        R = B - matmul(U)
    Z = psolve(R)
    D = Z.copy()
    rho = np.sum(R * Z, axis=0)
    Z0 = Z.copy()
    rho0 = rho.copy()
    bnorm = np.sqrt(np.sum(B * B, axis=0))
    active = np.isfinite(rho) & (rho > 0)
    m_valid = np.zeros(c, dtype=np.int64)
    alphas, betas, resids = [], [], []
    iters_run = 0
    for _ in range(p):
        V = matmul(D)
        dv = np.sum(D * V, axis=0)
        ok = active & np.isfinite(dv) & (dv > 0)
        alpha = np.where(ok, rho / np.where(ok, dv, 1.0), 0.0)
        active = ok
        U = U + D * alpha
        R = R - V * alpha
        m_valid = m_valid + ok.astype(np.int64)
        iters_run += 1
        rnorm = np.sqrt(np.sum(R * R, axis=0))
        rel = rnorm / np.where(bnorm > 0, bnorm, 1.0)
        Z = psolve(R)
        rho_new = np.sum(R * Z, axis=0)
        ok2 = active & np.isfinite(rho_new) & (rho_new > 0)
        beta = np.where(ok2, rho_new / np.where(active, rho, 1.0), 0.0)
        active = ok2
        alphas.append(alpha)
        betas.append(beta)
        resids.append(rel)
        if tol > 0 and np.all(rel < tol):
            break
        D = Z + D * beta
        rho = np.where(ok2, rho_new, rho)
    return MbcgResult(U=U, alpha=np.array(alphas).reshape(iters_run, c),
                      beta=np.array(betas).reshape(iters_run, c),
                      resid=np.array(resids).reshape(iters_run, c), iters_run=iters_run,
                      Z0=Z0, rho0=rho0, m_valid=m_valid)


def tridiag_from_cg(alpha: np.ndarray, beta: np.ndarray, m: int):
    """Lanczos tridiagonal of size m from one column's CG coefficients.

    diag_j = 1/alpha_j + beta_{j-1}/alpha_{j-1},  off_{j-1} = sqrt(beta_{j-1})/alpha_{j-1}
    (Observation "Recovering Lanczos tridiagonal matrices from standard CG", App. A).
    Returns (diag[m], off[m-1]).
    """
    dg = np.zeros(m)
    off = np.zeros(max(m - 1, 0))
    for j in range(m):
        dg[j] = 1.0 / alpha[j]
        if j > 0:
            dg[j] += beta[j - 1] / alpha[j - 1]
            off[j - 1] = np.sqrt(beta[j - 1]) / alpha[j - 1]
    return dg, off


def e1_logT_e1(dg: np.ndarray, off: np.ndarray) -> float:
    """e_1^T log(T) e_1 = sum_m V[0,m]^2 log(lambda_m)  (App. B, log-det paragraph)."""
    if dg.shape[0] == 0:
        return 0.0
    # (LAPACK's QL/QR driver: the default MRRR driver gives up on Lanczos tridiagonals that hold
    # near-duplicate eigenvalues, which long CG runs produce)
    lam, vec = sla.eigh_tridiagonal(dg, off, lapack_driver="stev")
    return float(np.sum(vec[0, :] ** 2 * np.log(lam)))


@dataclass
class BbmmResult:
    u0: np.ndarray
    U: np.ndarray
    W: np.ndarray            # P^{-1} z_i, i = 1..t
    logdet: float
    logdet_precond: float
    slq_terms: np.ndarray    # rho0_i * e1^T log(T_i) e1
    yKinvy: float
    trace: np.ndarray
    quad: np.ndarray
    nlml: float
    grad: np.ndarray
    L: np.ndarray
    pivots: np.ndarray
    pivot_dmax: np.ndarray
    mbcg: MbcgResult
    B: np.ndarray


def bbmm_inference(kernel: int, X, y, ls, s: float, noise: float, E1, E2, k: int, p: int,
                   tol: float = 0.0, forced_pivots: Optional[Sequence[int]] = None,
                   Khat: Optional[np.ndarray] = None, trace_row_chunk: int = 2048,
                   progress: Optional[Callable[[str], None]] = None,
                   u0_init: Optional[np.ndarray] = None) -> BbmmResult:
    """One BBMM call: K_hat^{-1} y, log|K_hat| estimate, trace estimates, NLML and gradient.

    `progress`, if given, is called with a short text at stage boundaries (long runs only).
    `u0_init` warm-starts the y column (Alg. 2's input U_0); the probe columns start from zero,
    because their tridiagonals are those of the Lanczos process started at z_i.
    """
    say = progress if progress is not None else (lambda msg: None)
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    ls = np.atleast_1d(np.asarray(ls, dtype=np.float64))
    n = X.shape[0]
    t = np.asarray(E2).shape[1]
    if Khat is None:
        Khat = kernel_matrix(kernel, X, ls, s)
        Khat[np.diag_indices(n)] += noise

    # rank-k pivoted Cholesky of K_XX (not K_hat): rows come from K_hat minus the noise.
    def get_row(i):
        row = Khat[i].copy()
        row[i] -= noise
        return row

    diagK = np.diag(Khat) - noise
    L, pivots, dmax = pivoted_cholesky(diagK, get_row, k, forced_pivots)
    P = make_preconditioner(L, noise)
    Zp = make_probes(L, noise, np.asarray(E1)[:L.shape[1]], E2)
    B = np.concatenate([y[:, None], Zp], axis=1)

    say("preconditioner and probes ready")
    U0 = None
    if u0_init is not None:
        U0 = np.zeros_like(B)
        U0[:, 0] = np.asarray(u0_init, dtype=np.float64)
    res = mbcg(lambda M: Khat @ M, B, P.solve, p, tol, U0=U0)
    say("mBCG done: %d iterations" % res.iters_run)

    # stochastic Lanczos quadrature, probe columns only
    terms = np.zeros(t)
    for i in range(t):
        col = i + 1
        m = int(res.m_valid[col])
        dg, off = tridiag_from_cg(res.alpha[:, col], res.beta[:, col], m)
        terms[i] = res.rho0[col] * e1_logT_e1(dg, off)
    logdet = P.logdet + float(np.mean(terms))

    # trace estimates with preconditioned probes: (1/t) sum_i u_i^T M_h w_i, and u_0^T M_h u_0.
    # The derivative matrices are formed a block of rows at a time (memory only; each row
    # block contributes its rows of M_h W and M_h u_0 exactly as the full matrix would).
    U = res.U
    u0 = U[:, 0]
    W = res.Z0[:, 1:]
    H = ls.shape[0] + 1
    trace = [0.0] * H
    quad = [0.0] * H
    for a in range(0, n, trace_row_chunk):
        b = min(n, a + trace_row_chunk)
        mats = kernel_derivative_blocks(kernel, X[a:b], X, ls, s)
        for h, M in enumerate(mats):
            trace[h] += float(np.sum(U[a:b, 1:] * (M @ W)) / t)
            quad[h] += float(u0[a:b] @ (M @ u0))
        say("derivative rows %d / %d" % (b, n))
    trace.append(float(np.sum(U[:, 1:] * W) / t))     # dK_hat/dsigma^2 = I
    quad.append(float(u0 @ u0))
    trace = np.array(trace)
    quad = np.array(quad)
    yKinvy = float(y @ u0)
    return BbmmResult(u0=u0, U=U, W=W, logdet=logdet, logdet_precond=P.logdet, slq_terms=terms,
                      yKinvy=yKinvy, trace=trace, quad=quad,
                      nlml=nlml_from_terms(yKinvy, logdet, n), grad=0.5 * (trace - quad),
                      L=L, pivots=pivots, pivot_dmax=dmax, mbcg=res, B=B)


# ----------------------------------------------------------------------------
# Predictive distribution at test inputs (Sec. 2, Eq. (1), zero prior mean):
#   mean(x*)       = k_{X x*}^T K_hat^{-1} y
#   cov(x*, x*')   = k(x*, x*') - k_{X x*}^T K_hat^{-1} k_{X x*'}      (latent f; add sigma^2 for y)
# ----------------------------------------------------------------------------
def exact_predict(kernel: int, X, y, ls, s: float, noise: float, Xs):
    """The plain definition through the dense Cholesky factor.  Returns (mean, cov), cov ns x ns."""
    X = np.asarray(X, dtype=np.float64)
    Xs = np.asarray(Xs, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n = X.shape[0]
    Khat = kernel_matrix(kernel, X, ls, s)
    Khat[np.diag_indices(n)] += noise
    KXs = kernel_block(kernel, X, Xs, ls, s)                  # n x ns, columns k_{X x*}
    u0, _, factor = exact_solve_logdet(Khat, y)
    mean = KXs.T @ u0
    cov = kernel_block(kernel, Xs, Xs, ls, s) - KXs.T @ sla.cho_solve(factor, KXs)
    return mean, cov


def bbmm_predict(kernel: int, X, ls, s: float, noise: float, Xs, u0: np.ndarray,
                 P: "Preconditioner", p: int, tol: float = 0.0, Khat: Optional[np.ndarray] = None):
    """The same two quantities the way the method obtains them: the mean from a solve u0 that is
    already there, the variances from one more preconditioned mBCG run (Alg. 2) whose right-hand
    sides are the columns k_{X x*}.  Returns (mean, var, MbcgResult)."""
    X = np.asarray(X, dtype=np.float64)
    Xs = np.asarray(Xs, dtype=np.float64)
    n = X.shape[0]
    if Khat is None:
        Khat = kernel_matrix(kernel, X, ls, s)
        Khat[np.diag_indices(n)] += noise
    KXs = kernel_block(kernel, X, Xs, ls, s)
    mean = KXs.T @ np.asarray(u0, dtype=np.float64)
    res = mbcg(lambda M: Khat @ M, KXs, P.solve, p, tol)
    prior = np.array([kernel_block(kernel, Xs[a:a + 1], Xs[a:a + 1], ls, s)[0, 0] for a in range(Xs.shape[0])])
    var = prior - np.sum(KXs * res.U, axis=0)
    return mean, var, res
