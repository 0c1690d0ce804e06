"""GPU parity tests: every stage of the HIP path, called through the C ABI, against the fp64
oracle on the same seeded inputs.  Sizes span several 16-row tiles, several 256-row padding
groups and ragged tails.

Tolerances (fp32 GPU vs fp64 oracle): relative 1e-3 norm-wise on each solve column, on the
log-determinant and on each trace / quadratic term; 1e-2 on the log-determinant against the
dense-Cholesky value.  Stage outputs that involve no iteration are held to tighter bounds
derived from fp32 rounding (stated at each test)."""
import numpy as np
import pytest

from oracle import bbmm_oracle as O
from paper_1809_11165_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ctx():
    from paper_1809_11165_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def _problem(w, mode):
    from paper_1809_11165_amd import binding
    return binding.problem_from_workload(w, mode)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")


def _host(tn):
    return tn.detach().cpu().numpy().astype(np.float64)


def _colrel(a, b):
    """max over columns of |a - b|_2 / |b|_2"""
    a = np.atleast_2d(a.T).T
    b = np.atleast_2d(b.T).T
    num = np.linalg.norm(a - b, axis=0)
    den = np.linalg.norm(b, axis=0)
    return float(np.max(num / np.where(den > 0, den, 1.0)))


def _khat(w):
    K = O.kernel_matrix(w.kernel, w.X, w.lengthscale, w.outputscale)
    return K + w.noise * np.eye(w.n)


CASES = [
    # (kernel, ard, n, d) -- ragged n, d not a multiple of 4, d > 16
    (inputs.RBF, False, 700, 5),
    (inputs.MATERN52, True, 523, 16),
    (inputs.RBF, True, 300, 3),
    (inputs.MATERN52, False, 1030, 20),
]


def _case(kernel, ard, n, d, t=6, k=7, iters=12, noise=0.2, seed=0):
    return inputs.tiny(n, d, kernel=kernel, ard=ard, t=t, k=k, iters=iters, noise=noise, seed=seed)


# ------------------------------------------------------------- K_hat builder ---
@pytest.mark.parametrize("kernel,ard,n,d", CASES)
def test_build_khat_matches_oracle_kernel_matrix(ctx, kernel, ard, n, d):
    w = _case(kernel, ard, n, d)
    ctx.bbmm_setup(_problem(w, inputs.MATERIALISED))
    ctx.bbmm_build_khat()
    got = _host(ctx.bbmm_khat_block(0, n, 0, n))
    ref = _khat(w)
    # distance by the |x|^2+|x'|^2-2x.x' expansion in fp32: absolute error ~ 1e-6 |x|^2 in the
    # exponent, i.e. a few 1e-6 relative to the outputscale
    assert np.max(np.abs(got - ref)) < 2e-5 * w.outputscale
    assert np.allclose(np.diag(got), w.outputscale + w.noise, rtol=1e-6)
    # sub-block access
    blk = _host(ctx.bbmm_khat_block(17, 40, n - 33, 33))
    assert np.array_equal(blk, got[17:57, n - 33:].astype(np.float32).astype(np.float64))


# ---------------------------------------------------------------- K_hat . M ----
@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
@pytest.mark.parametrize("kernel,ard,n,d", CASES)
@pytest.mark.parametrize("c", [11, 17])
def test_kernel_mm_matches_oracle_product(ctx, mode, kernel, ard, n, d, c):
    w = _case(kernel, ard, n, d)
    ctx.bbmm_setup(_problem(w, mode))
    if mode == inputs.MATERIALISED:
        ctx.bbmm_build_khat()
    rng = np.random.default_rng(5)
    M = rng.standard_normal((n, c)).astype(np.float32)
    V = _host(ctx.bbmm_kernel_mm(mode, _dev(M)))
    ref = _khat(w) @ M.astype(np.float64)
    # fp32 kernel entries, fp64 sums
    assert _colrel(V, ref) < 1e-4


@pytest.mark.parametrize("c", [1, 16, 18, 19, 20, 21, 32])
def test_kernel_mm_block_widths(ctx, c):
    # every width class of the right-hand side: one MFMA group, one group plus 1/2/4 columns on
    # the vector unit (17..20), two groups; each column must come out in its own place
    w = _case(inputs.MATERN52, True, 777, 5)
    rng = np.random.default_rng(50 + c)
    M = rng.standard_normal((w.n, c)).astype(np.float32)
    ref = _khat(w) @ M.astype(np.float64)
    for mode in (inputs.MATERIALISED, inputs.ONTHEFLY):
        ctx.bbmm_setup(_problem(w, mode))
        if mode == inputs.MATERIALISED:
            ctx.bbmm_build_khat()
        V = _host(ctx.bbmm_kernel_mm(mode, _dev(M)))
        assert V.shape == ref.shape
        assert _colrel(V, ref) < 1e-4, mode


@pytest.mark.parametrize("c", [11, 20])
def test_kernel_mm_work_decompositions_agree(ctx, c):
    # the way the product is dealt out to workgroups (and the number of partial results summed
    # per row) must not change the result beyond rounding order
    w = _case(inputs.RBF, False, 2100, 8)
    rng = np.random.default_rng(6)
    M = _dev(rng.standard_normal((w.n, c)))
    ref = _khat(w) @ _host(M)
    for mode in (inputs.MATERIALISED, inputs.ONTHEFLY):
        ctx.bbmm_setup(_problem(w, mode))
        if mode == inputs.MATERIALISED:
            ctx.bbmm_build_khat()
        for split in (1, 3, 8, 64, 177):
            ctx.bbmm_tune("mat_wgs", split)
            ctx.bbmm_tune("otf_split", split)
            V = _host(ctx.bbmm_kernel_mm(mode, M))
            assert _colrel(V, ref) < 1e-4, (mode, split)
    ctx.bbmm_tune("mat_wgs", 0)
    ctx.bbmm_tune("otf_split", 0)


# ------------------------------------------------------- pivoted Cholesky ------
def _oracle_pc(w, k, forced=None):
    K = O.kernel_matrix(w.kernel, w.X, w.lengthscale, w.outputscale)
    return O.pivoted_cholesky(np.diag(K).copy(), lambda i: K[i], k, forced), K


@pytest.mark.parametrize("kernel,ard,n,d", CASES)
def test_pivoted_cholesky_matches_oracle(ctx, kernel, ard, n, d):
    w = _case(kernel, ard, n, d, k=9)
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    assert rank == 9
    assert len(set(piv.tolist())) == 9
    assert piv[0] == 0          # constant diagonal: the tie goes to the lowest index
    # each GPU pivot attains (within fp32 rounding of L) the oracle's maximal residual diagonal
    (Lf, pf, dmax_forced), K = _oracle_pc(w, 9, piv)
    delta = np.diag(K).copy()
    for m in range(9):
        masked = delta.copy()
        masked[piv[:m]] = -np.inf
        assert delta[piv[m]] >= masked.max() * (1 - 1e-4)
        delta = delta - Lf[:, m] ** 2
    # factor replayed with the same pivot order
    got = _host(L)
    assert np.max(np.abs(got - Lf)) < 5e-6 * np.sqrt(w.outputscale) * 10


def test_pivoted_cholesky_replays_a_given_pivot_order(ctx):
    # pivots_in: the factor of App. C along a caller-given order (here not the greedy one)
    w = _case(inputs.MATERN52, True, 523, 16, k=6)
    order = np.array([400, 3, 77, 522, 250, 9], dtype=np.int64)
    prob = _problem(w, inputs.ONTHEFLY)
    prob.pivots_in = order
    ctx.bbmm_setup(prob)
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    assert rank == 6 and piv.tolist() == order.tolist()
    (Lf, pf, dmax), K = _oracle_pc(w, 6, order)
    assert np.max(np.abs(_host(L) - Lf)) < 5e-6 * np.sqrt(w.outputscale) * 10
    # and the whole call runs on that preconditioner
    res = ctx.bbmm_solve_logdet_grad(prob)
    assert res.pivots.tolist() == order.tolist()
    ref = O.bbmm_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise, w.E1, w.E2,
                           6, res.iters_run, forced_pivots=order)
    assert res.logdet_precond == pytest.approx(ref.logdet_precond, rel=1e-6)
    assert _colrel(_host(res.u0), ref.u0) < 1e-3
    # invalid orders are rejected
    from paper_1809_11165_amd import binding
    for bad in ([1, 1, 2, 3, 4, 5], [0, 1, 2, 3, 4, 523]):
        prob.pivots_in = np.array(bad, dtype=np.int64)
        with pytest.raises(binding.BbmmError) as ei:
            ctx.bbmm_setup(prob)
        assert ei.value.code == binding.EINVAL


def test_pivoted_cholesky_rank_zero_and_full_small(ctx):
    w = _case(inputs.RBF, False, 40, 2, k=0, t=2)
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    assert rank == 0 and len(piv) == 0
    assert ctx.bbmm_precond_setup() == pytest.approx(40 * np.log(w.noise), rel=1e-12)
    w = inputs.tiny(24, 2, kernel=inputs.RBF, t=2, k=24, noise=0.3)
    w.lengthscale[:] = 0.5
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    assert rank == 24 and sorted(piv.tolist()) == list(range(24))
    K = O.kernel_matrix(w.kernel, w.X, w.lengthscale, w.outputscale)
    Lh = _host(L)
    assert np.max(np.abs(Lh @ Lh.T - K)) < 1e-4


# --------------------------------------- Woodbury solve, log|P|, probes --------
@pytest.mark.parametrize("kernel,ard,n,d", CASES[:2])
def test_preconditioner_and_probes_match_oracle(ctx, kernel, ard, n, d):
    w = _case(kernel, ard, n, d, k=8)
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    logdetP = ctx.bbmm_precond_setup()
    Lh = _host(L)                                  # the fp64 factor the GPU really uses
    P = O.make_preconditioner(Lh, w.noise)
    assert logdetP == pytest.approx(P.logdet, rel=1e-10)
    rng = np.random.default_rng(2)
    R = rng.standard_normal((n, 7)).astype(np.float32)
    Z = _host(ctx.bbmm_precond_solve(_dev(R)))
    assert _colrel(Z, P.solve(R.astype(np.float64))) < 1e-5
    B = _host(ctx.bbmm_make_probes())
    ref = np.concatenate([w.y[:, None].astype(np.float64),
                          O.make_probes(Lh, w.noise, w.E1, w.E2)], axis=1)
    assert np.max(np.abs(B - ref)) < 1e-6 * np.max(np.abs(ref))


# ---------------------------------------------------------------- mBCG ---------
@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
@pytest.mark.parametrize("kernel,ard,n,d", CASES[:3])
def test_mbcg_matches_oracle_at_fixed_iterations(ctx, mode, kernel, ard, n, d):
    w = _case(kernel, ard, n, d, k=6, iters=10)
    ctx.bbmm_setup(_problem(w, mode))
    if mode == inputs.MATERIALISED:
        ctx.bbmm_build_khat()
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    ctx.bbmm_precond_setup()
    B = ctx.bbmm_make_probes()
    U, alpha, beta, resid, iters = ctx.bbmm_mbcg(mode, B)
    assert iters == 10
    Kh = _khat(w)
    P = O.make_preconditioner(_host(L), w.noise)
    ref = O.mbcg(lambda M: Kh @ M, _host(B), P.solve, 10)
    assert _colrel(_host(U), ref.U) < 1e-3
    assert np.allclose(alpha[:5], ref.alpha[:5], rtol=1e-3)
    assert np.allclose(beta[:5], ref.beta[:5], rtol=2e-3)
    assert np.allclose(resid, ref.resid, rtol=5e-2, atol=1e-6)
    logdet, terms = ctx.bbmm_slq_logdet()
    ref_terms = []
    for i in range(w.t):
        dg, off = O.tridiag_from_cg(ref.alpha[:, i + 1], ref.beta[:, i + 1], 10)
        ref_terms.append(ref.rho0[i + 1] * O.e1_logT_e1(dg, off))
    ref_logdet = P.logdet + np.mean(ref_terms)
    assert logdet == pytest.approx(ref_logdet, rel=1e-3)
    assert np.allclose(terms, ref_terms, rtol=1e-3, atol=1e-3 * np.max(np.abs(ref_terms)))


def test_mbcg_tolerance_stop_and_wide_block(ctx):
    w = _case(inputs.RBF, False, 900, 4, t=20, k=10, iters=80, noise=0.3)
    w.tol = 0.01
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    ctx.bbmm_precond_setup()
    B = ctx.bbmm_make_probes()                       # 21 columns -> 32-wide path
    U, alpha, beta, resid, iters = ctx.bbmm_mbcg(inputs.ONTHEFLY, B)
    assert 1 <= iters < 80
    assert resid[iters - 1].max() < 0.01
    if iters > 1:
        assert resid[iters - 2].max() >= 0.01
    assert np.all(alpha[iters:] == 0.0)
    Kh = _khat(w)
    P = O.make_preconditioner(_host(L), w.noise)
    ref = O.mbcg(lambda M: Kh @ M, _host(B), P.solve, iters)
    # the residual hovers near the threshold for several iterations, so the exact stopping
    # iteration is not unique across precisions: the oracle, run for the same number of
    # iterations, must itself be at the threshold (within a factor 2)
    assert ref.resid[-1].max() < 0.02
    assert _colrel(_host(U), ref.U) < 1e-3
    true_rel = np.linalg.norm(_host(B) - Kh @ _host(U), axis=0) / np.linalg.norm(_host(B), axis=0)
    assert true_rel.max() < 0.011


def test_warm_start_of_the_y_column(ctx):
    # Alg. 1/2 take the current solution as input (r_0 = b - K_hat u_0): u0_init
    w = _case(inputs.RBF, False, 900, 4, t=5, k=6, iters=12, noise=0.05)
    Kh = _khat(w)
    exact = np.linalg.solve(Kh, w.y.astype(np.float64))
    rng = np.random.default_rng(4)
    u_init = (exact + 0.02 * np.abs(exact).max() * rng.standard_normal(w.n)).astype(np.float32)
    for mode in (inputs.MATERIALISED, inputs.ONTHEFLY):
        prob = _problem(w, mode)
        cold = ctx.bbmm_solve_logdet_grad(prob)
        prob.u0_init = _dev(u_init)
        warm = ctx.bbmm_solve_logdet_grad(prob)
        ref = O.bbmm_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise, w.E1, w.E2,
                               w.k, warm.iters_run, forced_pivots=warm.pivots, u0_init=u_init)
        assert _colrel(_host(warm.U), ref.U) < 1e-3
        assert np.allclose(warm.resid[:, 0], ref.mbcg.resid[:, 0], rtol=5e-2, atol=1e-7)
        assert np.allclose(warm.alpha[:5], ref.mbcg.alpha[:5], rtol=1e-3)
        # the probe columns, and with them the log-det estimate, do not depend on the start
        assert np.array_equal(warm.alpha[:, 1:], cold.alpha[:, 1:])
        assert warm.logdet == cold.logdet
        assert torch.equal(warm.U[:, 1:], cold.U[:, 1:])
        # and the y column is ahead of the cold start
        assert np.all(warm.resid[:6, 0] < cold.resid[:6, 0])
    # with a tolerance the warm start stops earlier (one column: the stop test is over all columns)
    w1 = _case(inputs.RBF, False, 900, 4, t=1, k=6, iters=200, noise=0.05)
    w1.tol = 1e-4
    ctx.bbmm_setup(_problem(w1, inputs.ONTHEFLY))
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    ctx.bbmm_precond_setup()
    B = _dev(w1.y[:, None])
    U, a, b, r, it_cold = ctx.bbmm_mbcg(inputs.ONTHEFLY, B)
    prob = _problem(w1, inputs.ONTHEFLY)
    prob.u0_init = _dev(u_init)
    ctx.bbmm_setup(prob)
    ctx.bbmm_pivoted_cholesky()
    ctx.bbmm_precond_setup()
    Uw, a, b, rw, it_warm = ctx.bbmm_mbcg(inputs.ONTHEFLY, B)
    assert it_warm < it_cold
    assert rw[it_warm - 1, 0] < 1e-4
    assert _colrel(_host(Uw), exact[:, None]) < 1e-3


def test_iterations_to_tolerance_fall_with_the_preconditioner_rank(ctx):
    # Sec. 4, Theorem 1 and the residual-against-iteration experiment: on a univariate RBF kernel
    # the rank-k pivoted-Cholesky preconditioner cuts the iterations CG needs; the GPU's counts
    # follow the oracle's within three iterations
    from paper_1809_11165_amd import binding
    rng = np.random.default_rng(0)
    n = 3000
    X = np.sort(rng.uniform(0, 1, (n, 1)), axis=0).astype(np.float32)
    y = np.sin(6 * X[:, 0]).astype(np.float32)
    E2 = inputs.rademacher(rng, (n, 1))
    Kh = O.kernel_matrix(O.RBF, X, [0.2], 1.0) + 0.01 * np.eye(n)
    its_gpu, its_ref, curves = [], [], []
    for k in (0, 2, 5, 9):
        E1 = inputs.rademacher(rng, (max(k, 1), 1))[:k]
        prob = binding.Problem(kernel=inputs.RBF, mode=inputs.ONTHEFLY, X=_dev(X), y=_dev(y),
                               lengthscale=np.array([0.2]), outputscale=1.0, noise=0.01,
                               E1=_dev(E1) if k else None, E2=_dev(E2), k=k, max_iters=200, tol=1e-6)
        ctx.bbmm_setup(prob)
        L, piv, rank = ctx.bbmm_pivoted_cholesky()
        ctx.bbmm_precond_setup()
        U, alpha, beta, resid, iters = ctx.bbmm_mbcg(inputs.ONTHEFLY, _dev(y[:, None]))
        P = O.make_preconditioner(_host(L) if k else np.zeros((n, 0)), 0.01)
        ref = O.mbcg(lambda M: Kh @ M, y[:, None].astype(np.float64), P.solve, 200, tol=1e-6)
        its_gpu.append(iters)
        its_ref.append(ref.iters_run)
        curves.append(resid[:iters, 0])
        # the first iterations of the curves agree; later the residual (not monotone in CG) jumps
        # about in a way that the fp32 rounding of the kernel entries already changes
        assert np.allclose(resid[:3, 0], ref.resid[:3, 0], rtol=0.05)
    assert all(abs(a - b) <= 3 for a, b in zip(its_gpu, its_ref)), (its_gpu, its_ref)
    assert all(a >= b for a, b in zip(its_gpu, its_gpu[1:])), its_gpu
    assert its_gpu[-1] < its_gpu[0]
    # at a fixed iteration the residual falls with the rank (the figure's curves do not cross here)
    j = min(len(c) for c in curves) - 1
    assert curves[3][j] < curves[0][j]


# ------------------------------------------- tridiagonal eigen-solver, SLQ -----
@pytest.mark.parametrize("m", [1, 2, 3, 17, 50, 100, 256])
def test_tridiag_eig_batched_against_lapack(ctx, m):
    import scipy.linalg as sla
    rng = np.random.default_rng(m)
    batch = 5
    diag = rng.uniform(0.5, 3.0, (batch, m))
    off = rng.uniform(-1.0, 1.0, (batch, max(m - 1, 0))) * 0.4
    if m > 4:
        off[1, 2] = 0.0                      # an exactly split matrix
        diag[2, :] = 1.0                     # constant diagonal
    vals, first = ctx.bbmm_tridiag_eig_batched(diag, off)
    for b in range(batch):
        if m == 1:
            lam, vec = diag[b], np.ones((1, 1))
        else:
            lam, vec = sla.eigh_tridiagonal(diag[b], off[b])
        order = np.argsort(vals[b])
        assert np.allclose(vals[b][order], lam, rtol=1e-11, atol=1e-12)
        assert np.sum(first[b] ** 2) == pytest.approx(1.0, rel=1e-10)
        # compare the quadrature functional, which is what the weights are for
        got = np.sum(first[b] ** 2 * np.log(vals[b]))
        ref = np.sum(vec[0] ** 2 * np.log(lam))
        assert got == pytest.approx(ref, rel=1e-9, abs=1e-11)


def test_tridiag_eig_on_hard_matrices(ctx):
    # the cases the QR iteration's bookkeeping has to get right: several exact and near splits (also
    # adjacent ones and one at the bottom), a graded matrix, and a Lanczos tridiagonal run long enough
    # without reorthogonalisation to hold near-duplicate ("ghost") eigenvalues
    import scipy.linalg as sla
    rng = np.random.default_rng(12)
    m = 96
    mats = []
    d0 = rng.uniform(0.5, 3.0, m)
    o0 = rng.uniform(0.05, 0.4, m - 1)
    o1 = o0.copy()
    o1[[4, 5, 30, 31, 32, 70, m - 2]] = 0.0
    mats.append((d0, o1))
    o2 = o0.copy()
    o2[[10, 11, 50]] = 1e-18                         # below eps * (|a_i| + |a_i+1|): treated as a split
    o2[[20, 60]] = 1e-9                              # small but not negligible
    mats.append((d0, o2))
    g = np.logspace(-8, 4, m)                        # graded: entries over twelve orders of magnitude
    mats.append((g * rng.uniform(1.0, 2.0, m), 0.3 * np.sqrt(g[:-1] * g[1:])))
    lam = np.concatenate([np.linspace(0.1, 1.0, 380), [50.0, 80.0, 120.0, 200.0]])
    q = rng.standard_normal(lam.size)
    q /= np.linalg.norm(q)
    qp, beta = np.zeros_like(q), 0.0
    al, be = [], []
    for _ in range(m):                               # plain Lanczos on diag(lam)
        v = lam * q - beta * qp
        alpha = v @ q
        v -= alpha * q
        beta = np.linalg.norm(v)
        al.append(alpha)
        be.append(beta)
        qp, q = q, v / beta
    mats.append((np.array(al), np.array(be[:-1])))
    lam_l = sla.eigh_tridiagonal(mats[-1][0], mats[-1][1], eigvals_only=True)
    assert np.min(np.diff(lam_l)) < 1e-8 * lam_l[-1]    # the case does contain ghosts
    diag = np.stack([a for a, _ in mats])
    off = np.stack([b for _, b in mats])
    vals, first = ctx.bbmm_tridiag_eig_batched(diag, off)
    for b in range(len(mats)):
        lam_ref, vec = sla.eigh_tridiagonal(diag[b], off[b])
        order = np.argsort(vals[b])
        scale = np.max(np.abs(lam_ref))
        assert np.max(np.abs(vals[b][order] - lam_ref)) < 1e-12 * scale, b
        assert np.sum(first[b] ** 2) == pytest.approx(1.0, rel=1e-10)
        # quadrature functionals, which sum the weights of a cluster: e_1^T f(T) e_1 for f = log, 1/x
        pos = lam_ref > 0
        assert np.all(pos)
        for f in (np.log, lambda x: 1.0 / x):
            got = np.sum(first[b] ** 2 * f(vals[b]))
            ref = np.sum(vec[0] ** 2 * f(lam_ref))
            assert got == pytest.approx(ref, rel=1e-8, abs=1e-10), b


def test_tridiag_eig_reports_an_exhausted_sweep_budget(ctx):
    # forced from the host: with one trip per row a 50 x 50 matrix cannot be reduced; the kernel
    # still runs to its normal end and the call reports BBMM_ENOCONV instead of unfinished values
    from paper_1809_11165_amd import binding
    rng = np.random.default_rng(5)
    m = 50
    diag = rng.uniform(0.5, 3.0, (3, m))
    off = rng.uniform(0.1, 0.4, (3, m - 1))
    ctx.bbmm_tune("eig_sweeps", 1)
    ctx.bbmm_tune("slq_eig", 1)
    try:
        with pytest.raises(binding.BbmmError) as e:
            ctx.bbmm_tridiag_eig_batched(diag, off)
        assert e.value.code == binding.ENOCONV
        with pytest.raises(binding.BbmmError) as e:
            ctx.bbmm_slq_from_coeffs(np.full((m, 2), 0.5), np.full((m, 2), 0.3), np.ones(2))
        assert e.value.code == binding.ENOCONV
    finally:
        ctx.bbmm_tune("eig_sweeps", 0)
        ctx.bbmm_tune("slq_eig", 0)
    vals, first = ctx.bbmm_tridiag_eig_batched(diag, off)          # default budget: fine again
    assert np.all(np.isfinite(vals)) and np.allclose(np.sum(first ** 2, axis=1), 1.0)


def test_whole_call_reports_an_exhausted_sweep_budget(ctx):
    from paper_1809_11165_amd import binding
    w = inputs.tiny(400, 3, t=3, k=2, iters=30)
    ctx.bbmm_tune("eig_sweeps", 1)
    ctx.bbmm_tune("slq_eig", 1)                     # the eigen-decomposition route of the SLQ terms
    try:
        with pytest.raises(binding.BbmmError) as e:
            ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
        assert e.value.code == binding.ENOCONV
    finally:
        ctx.bbmm_tune("eig_sweeps", 0)
        ctx.bbmm_tune("slq_eig", 0)
    res = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
    assert np.isfinite(res.logdet)


def test_slq_from_coeffs_on_the_oracles_coefficients(ctx):
    """The SLQ stage in isolation (App. A Observation, App. B): the ORACLE's alpha, beta, rho0 and
    m_valid go in, its terms and log-det must come out -- including a column that the breakdown
    guard froze early (a zero right-hand side never starts: m_valid = 0, term 0) and columns whose
    tridiagonals are truncated below the iteration count."""
    w = _case(inputs.MATERN52, True, 600, 6, t=6, k=5, iters=40, noise=0.05)
    Kh = _khat(w)
    Kxx = Kh - w.noise * np.eye(w.n)
    L, piv, _ = O.pivoted_cholesky(np.diag(Kxx).copy(), lambda i: Kxx[i], w.k)
    P = O.make_preconditioner(L, w.noise)
    Z = O.make_probes(L, w.noise, w.E1, w.E2)
    Z[:, 2] = 0.0                                    # frozen from the start
    ref = O.mbcg(lambda M: Kh @ M, Z, P.solve, 40)
    mv = ref.m_valid.copy()
    assert mv[2] == 0
    mv[4] = 17                                       # a tridiagonal cut short on purpose
    mv[5] = 1                                        # 1 x 1
    terms_ref = np.array([ref.rho0[i] * O.e1_logT_e1(*O.tridiag_from_cg(ref.alpha[:, i], ref.beta[:, i], int(mv[i])))
                          for i in range(w.t)])
    logdet, terms = ctx.bbmm_slq_from_coeffs(ref.alpha, ref.beta, ref.rho0, mv, logdet_precond=P.logdet)
    assert terms[2] == 0.0
    assert np.allclose(terms, terms_ref, rtol=1e-10, atol=1e-10 * np.abs(terms_ref).max())
    assert logdet == pytest.approx(P.logdet + terms_ref.mean(), rel=1e-11)
    # m_valid = NULL means p for every column
    ld2, t2 = ctx.bbmm_slq_from_coeffs(ref.alpha[:, [0, 1, 3]], ref.beta[:, [0, 1, 3]], ref.rho0[[0, 1, 3]])
    full = [ref.rho0[i] * O.e1_logT_e1(*O.tridiag_from_cg(ref.alpha[:, i], ref.beta[:, i], 40)) for i in (0, 1, 3)]
    assert np.allclose(t2, full, rtol=1e-10)
    assert ld2 == pytest.approx(np.mean(full), rel=1e-10)


@pytest.mark.parametrize("route", [0, 1])
def test_slq_terms_by_quadrature_and_by_eigen_decomposition(ctx, route):
    """Both routes to e_1^T log(T) e_1 -- the quadrature of the resolvent (default) and the
    eigen-decomposition of App. B -- on the ORACLE's coefficients of long, ill-conditioned CG runs
    (Ritz values converged and re-found many times over: clusters of near-duplicate eigenvalues),
    against the oracle's eigen-decomposition."""
    rng = np.random.default_rng(3)
    lam = np.concatenate([np.logspace(-6, 0, 380), [50.0, 80.0, 120.0, 200.0]])
    B = rng.standard_normal((lam.size, 4))
    alpha, beta, rho0, mv, ref = [], [], [], [], []
    for p in (1, 2, 20, 60, 150, 250):
        r = O.mbcg(lambda M: lam[:, None] * M, B, lambda R: R, p)
        pad = np.zeros((250 - p, 4))
        alpha.append(np.vstack([r.alpha, pad]))
        beta.append(np.vstack([r.beta, pad]))
        rho0.append(r.rho0)
        mv.append(r.m_valid)
        ref.append([r.rho0[i] * O.e1_logT_e1(*O.tridiag_from_cg(r.alpha[:, i], r.beta[:, i], int(r.m_valid[i])))
                    for i in range(4)])
    alpha, beta = np.hstack(alpha), np.hstack(beta)
    rho0, mv, ref = np.concatenate(rho0), np.concatenate(mv), np.concatenate(ref)
    ctx.bbmm_tune("slq_eig", route)
    try:
        logdet, terms = ctx.bbmm_slq_from_coeffs(alpha, beta, rho0, mv, logdet_precond=1.5)
    finally:
        ctx.bbmm_tune("slq_eig", 0)
    assert np.allclose(terms, ref, rtol=2e-9)
    assert logdet == pytest.approx(1.5 + ref.mean(), rel=1e-9)


def test_slq_refuses_a_tridiagonal_that_is_not_positive_definite(ctx):
    from paper_1809_11165_amd import binding
    alpha = np.full((6, 2), 0.5)
    beta = np.full((6, 2), 0.3)
    alpha[3, 1] = -0.5                                 # 1 / alpha < 0 on the diagonal of T_2
    with pytest.raises(binding.BbmmError) as e:
        ctx.bbmm_slq_from_coeffs(alpha, beta, np.ones(2))
    assert e.value.code == binding.ENONFINITE
    ctx.bbmm_slq_from_coeffs(alpha[:, :1], beta[:, :1], np.ones(1))      # the other column alone is fine


def test_slq_from_coeffs_equals_the_in_context_stage(ctx):
    # the coefficients of a GPU run handed back in: same kernel arithmetic, so bit-identical terms
    w = _case(inputs.RBF, False, 700, 5, t=6, k=7, iters=25)
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    ctx.bbmm_pivoted_cholesky()
    logdetP = ctx.bbmm_precond_setup()
    B = ctx.bbmm_make_probes()
    U, alpha, beta, resid, iters = ctx.bbmm_mbcg(inputs.ONTHEFLY, B)
    logdet, terms = ctx.bbmm_slq_logdet()
    Bh = _host(B)
    # rho0 = z^T P^-1 z from the preconditioner stage
    Zp = _host(ctx.bbmm_precond_solve(B))
    rho0 = np.sum(Bh[:, 1:] * Zp[:, 1:], axis=0)
    ld2, t2 = ctx.bbmm_slq_from_coeffs(alpha[:iters, 1:], beta[:iters, 1:], rho0, logdet_precond=logdetP)
    # rho0 here went through fp32 blocks, the context keeps it in fp64: 1e-6
    assert np.allclose(t2, terms, rtol=1e-5)
    assert ld2 == pytest.approx(logdet, rel=1e-5)


# ------------------------------------------------------- derivative pass -------
@pytest.mark.parametrize("kernel,ard,n,d", CASES)
def test_dk_traces_match_oracle_formulas(ctx, kernel, ard, n, d):
    w = _case(kernel, ard, n, d, t=5)
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    rng = np.random.default_rng(9)
    U = rng.standard_normal((n, w.t + 1)).astype(np.float32)
    W = rng.standard_normal((n, w.t)).astype(np.float32)
    trace, quad = ctx.bbmm_dk_traces(_dev(U), _dev(W))
    mats = O.kernel_derivative_blocks(w.kernel, w.X, w.X, w.lengthscale, w.outputscale)
    Ud, Wd = U.astype(np.float64), W.astype(np.float64)
    ref_tr = [np.sum(Ud[:, 1:] * (M @ Wd)) / w.t for M in mats] + [np.sum(Ud[:, 1:] * Wd) / w.t]
    ref_q = [Ud[:, 0] @ M @ Ud[:, 0] for M in mats] + [Ud[:, 0] @ Ud[:, 0]]
    # random-sign sums cancel heavily: scale the tolerance by the sum of absolute terms
    scale_tr = [np.sum(np.abs(Ud[:, 1:]) * (np.abs(M) @ np.abs(Wd))) / w.t for M in mats] + [1.0]
    scale_q = [np.abs(Ud[:, 0]) @ np.abs(M) @ np.abs(Ud[:, 0]) for M in mats] + [1.0]
    for h in range(len(ref_tr)):
        assert abs(trace[h] - ref_tr[h]) < 2e-5 * scale_tr[h] + 1e-3 * abs(ref_tr[h]), h
        assert abs(quad[h] - ref_q[h]) < 2e-5 * scale_q[h] + 1e-3 * abs(ref_q[h]), h


# ------------------------------------------------------------ whole path -------
def _full_parity(ctx, w, mode, check_exact=True, tol_solve=1e-3):
    res = ctx.bbmm_solve_logdet_grad(_problem(w, mode))
    ref = O.bbmm_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise, w.E1, w.E2,
                           w.k, res.iters_run, forced_pivots=res.pivots)
    assert res.rank == w.k
    assert _colrel(_host(res.U), ref.U) < tol_solve
    assert _colrel(_host(res.u0), ref.u0) < tol_solve
    assert res.logdet_precond == pytest.approx(ref.logdet_precond, rel=1e-5)
    assert res.logdet == pytest.approx(ref.logdet, rel=1e-3)
    assert res.yKinvy == pytest.approx(ref.yKinvy, rel=1e-3)
    assert res.nlml == pytest.approx(ref.nlml, rel=1e-3)
    for h in range(len(ref.trace)):
        assert res.trace[h] == pytest.approx(ref.trace[h], rel=1e-3, abs=1e-3 * np.max(np.abs(ref.trace))), h
        assert res.quad[h] == pytest.approx(ref.quad[h], rel=1e-3, abs=1e-3 * np.max(np.abs(ref.quad))), h
        denom = max(abs(ref.trace[h]), abs(ref.quad[h])) / 2
        assert abs(res.grad_nlml[h] - ref.grad[h]) < 1e-3 * denom + 1e-9, h
    if check_exact:
        # against the dense-Cholesky value: 1e-2, unless the estimator itself (t probes, p
        # iterations, evaluated by the fp64 oracle) is further away than that -- then the GPU
        # must reproduce the oracle's estimate, which the 1e-3 check above already enforces,
        # and may not be further from the exact value than the oracle is (plus 1e-3).
        ex = O.exact_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise,
                               with_traces=False)
        est_err = abs(ref.logdet - ex.logdet)
        assert abs(res.logdet - ex.logdet) <= max(1e-2 * abs(ex.logdet),
                                                  est_err + 1e-3 * abs(ex.logdet))
        res.estimator_rel_err = est_err / abs(ex.logdet)
    return res, ref


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_full_path_config1(ctx, mode):
    w = inputs.make(1)                      # n = 1000, d = 4, t = 10, k = 5, p = 20
    res, ref = _full_parity(ctx, w, mode)
    assert res.iters_run == 20


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_full_path_config2_shape_with_tolerance(ctx, mode):
    w = inputs.make(2, n=3000)              # RBF d = 8, k = 10, tol 1e-2 or 50 iterations
    res, ref = _full_parity(ctx, w, mode)
    assert res.iters_run <= 50
    assert ref.mbcg.resid[res.iters_run - 1].max() < 2e-2     # oracle is at the threshold too


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_full_path_config3_shape(ctx, mode):
    w = inputs.make(3, n=2500)              # Matern-5/2 ARD d = 16, k = 20, p = 50
    res, ref = _full_parity(ctx, w, mode)
    ex = O.exact_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise,
                           with_traces=False)
    assert res.logdet == pytest.approx(ex.logdet, rel=1e-2)     # converged: plain 1e-2 bound holds
    assert _colrel(_host(res.u0), ex.u0) < 1e-3


def test_full_path_config4_shape(ctx):
    w = inputs.make(4, n=3000, iters=40)    # clustered RBF d = 8, t = 16 (17 columns), k = 20
    _full_parity(ctx, w, inputs.ONTHEFLY)


def test_full_path_at_the_interface_limits(ctx):
    """Everything at its documented maximum at once: t = 31 probes (32 columns), rank k = 32, d = 64 ARD
    input dimensions, 256 iterations without a tolerance stop, n ragged (1237 = 77 * 16 + 5).  The
    iteration converges to rounding level after about 50 steps and runs on for 200 more (recurrence
    residual 1e-93 at the end): the coefficients of those steps are rounding noise, different on the
    two sides, and must not disturb the solves or the quadrature of the first row (App. A, B)."""
    w = inputs.tiny(1237, 64, kernel=O.MATERN52, ard=True, t=31, k=32, iters=256, noise=0.05, seed=3)
    w.X *= 0.25                               # distances of a few lengthscales, not of dozens
    runs = {}
    for name, mode, sym in (("mat", inputs.MATERIALISED, 0), ("sym", inputs.MATERIALISED, 1),
                            ("otf", inputs.ONTHEFLY, 0)):
        ctx.bbmm_tune("khat_sym", sym)
        runs[name] = ctx.bbmm_solve_logdet_grad(_problem(w, mode))
    ctx.bbmm_tune("khat_sym", 0)
    first = runs["mat"]
    ref = O.bbmm_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise, w.E1, w.E2,
                           w.k, 256, forced_pivots=first.pivots)
    ex = O.exact_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise, with_traces=False)
    assert np.linalg.norm(ref.u0 - ex.u0) < 1e-12 * np.linalg.norm(ex.u0)       # the oracle has converged
    for name, res in runs.items():
        assert res.iters_run == 256 and res.rank == 32, name
        assert np.array_equal(res.pivots, first.pivots), name
        assert _colrel(_host(res.U), ref.U) < 1e-3, name
        assert _colrel(_host(res.u0), ex.u0) < 1e-3, name
        assert np.all(np.isfinite(res.alpha)) and np.all(np.isfinite(res.beta)), name
        assert res.logdet_precond == pytest.approx(ref.logdet_precond, rel=1e-5), name
        assert np.allclose(res.slq_terms, ref.slq_terms, rtol=1e-3, atol=1e-3 * np.abs(ref.slq_terms).max()), name
        for key in ("logdet", "yKinvy", "nlml"):
            assert getattr(res, key) == pytest.approx(getattr(ref, key), rel=1e-3), (name, key)
        assert res.logdet == pytest.approx(ex.logdet, rel=1e-2), name
        for h in range(len(ref.trace)):
            assert res.trace[h] == pytest.approx(ref.trace[h], rel=1e-3, abs=1e-3 * np.max(np.abs(ref.trace))), (name, h)
            assert res.quad[h] == pytest.approx(ref.quad[h], rel=1e-3, abs=1e-3 * np.max(np.abs(ref.quad))), (name, h)


def test_full_path_is_deterministic(ctx):
    w = inputs.make(1, n=777)
    a = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
    b = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
    assert torch.equal(a.U, b.U)
    assert a.logdet == b.logdet and np.array_equal(a.trace, b.trace)
    assert np.array_equal(a.alpha, b.alpha)


@pytest.mark.parametrize("mode,tri", [(inputs.ONTHEFLY, 0), (inputs.MATERIALISED, 0), (inputs.MATERIALISED, 1),
                                      (inputs.SGPR, 0)])
def test_loop_graph_replays_equal_kernel_by_kernel_launches(ctx, mode, tri):
    """The mBCG loop replayed as a HIP graph against the same loop launched kernel by kernel: bit
    for bit, over several replays with other work and synchronisations of the program in between,
    with the hyperparameters (which the loop's kernels read from the device state, not from their
    arguments) changing from call to call, and with a tolerance stop that ends one run early."""
    w = inputs.make(2, n=2100, iters=40)
    if mode == inputs.SGPR:
        w = inputs.with_inducing(w, 300, np.random.Generator(np.random.Philox(7)))
    variants = [(0.05, 1.0, 0.0), (0.2, 1.7, 0.0), (0.05, 1.0, 0.15), (0.4, 0.6, 0.3)]   # (noise, outputscale, tol)

    def run(noise, s, tol):
        w.noise, w.outputscale, w.tol = noise, s, tol
        return ctx.bbmm_solve_logdet_grad(_problem(w, mode))

    ctx.bbmm_tune("khat_sym", tri)
    try:
        ctx.bbmm_tune("loop_graph", 0)
        ref = [run(*v) for v in variants]
        assert ref[2].iters_run < 40 and ref[0].iters_run == 40       # the stop rule does end a run early
        ctx.bbmm_tune("loop_graph", 1)
        cap0, rep0 = ctx.bbmm_loop_graph_stats()
        for rep in range(4):                  # run 1 kernel by kernel, run 2 records, later runs replay
            for v, r in zip(variants, ref):
                res = run(*v)
                # the program's own eager work and a synchronisation between the replays
                junk = torch.randn(512, 512, device="cuda:0") @ torch.randn(512, 512, device="cuda:0")
                torch.cuda.synchronize()
                assert torch.equal(res.U, r.U), (rep, v)
                assert res.iters_run == r.iters_run and res.logdet == r.logdet
                assert np.array_equal(res.alpha, r.alpha) and np.array_equal(res.beta, r.beta)
                assert np.array_equal(res.trace, r.trace) and np.array_equal(res.resid, r.resid)
                del junk
        cap1, rep1 = ctx.bbmm_loop_graph_stats()
        # one launch sequence for all four hyperparameter settings: recorded once, replayed 15 times
        assert (cap1 - cap0, rep1 - rep0) == (1, 15)
    finally:
        ctx.bbmm_tune("loop_graph", 0)
        ctx.bbmm_tune("khat_sym", 0)


# -------------------------------------------------------------- edge cases -----
def test_edge_small_n_rank0_single_probe(ctx):
    w = inputs.tiny(13, 2, kernel=inputs.RBF, t=1, k=0, iters=13, noise=0.3)
    res = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
    ref = O.bbmm_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise, w.E1, w.E2,
                           0, 13)
    ex = O.exact_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise)
    assert _colrel(_host(res.u0), ex.u0) < 1e-3      # p = n: CG has converged
    assert res.logdet == pytest.approx(ref.logdet, rel=2e-3)


def test_edge_n_equals_one(ctx):
    w = inputs.tiny(1, 1, kernel=inputs.MATERN52, t=2, k=1, iters=2, noise=0.5)
    res = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.MATERIALISED))
    a = w.outputscale + w.noise
    assert float(res.u0[0]) == pytest.approx(float(w.y[0]) / a, rel=1e-5)
    assert res.logdet == pytest.approx(np.log(a), rel=1e-5)


def test_invalid_arguments_are_rejected(ctx):
    from paper_1809_11165_amd import binding
    w = inputs.tiny(50, 3, t=3, k=2)
    p = _problem(w, inputs.ONTHEFLY)
    for field, value in [("max_iters", 0), ("max_iters", 257), ("noise", 0.0), ("outputscale", -1.0),
                         ("k", 33), ("kernel", 7), ("mode", 3)]:
        q = binding.Problem(**{**{f: getattr(p, f) for f in
                                  ("kernel", "mode", "X", "y", "lengthscale", "outputscale", "noise",
                                   "E1", "E2", "k", "max_iters", "tol")}, field: value})
        if field == "k":
            q.E1 = _dev(np.ones((33, 3)))
        with pytest.raises(binding.BbmmError) as ei:
            ctx.bbmm_solve_logdet_grad(q)
        assert ei.value.code == binding.EINVAL
    q = binding.Problem(kernel=p.kernel, mode=p.mode, X=p.X, y=p.y, lengthscale=np.array([1.0, 2.0]),
                        outputscale=1.0, noise=0.1, E1=p.E1, E2=p.E2, k=2, max_iters=5)
    with pytest.raises(binding.BbmmError):
        ctx.bbmm_solve_logdet_grad(q)            # 2 lengthscales for d = 3
    # call order: the materialised product needs K_hat
    ctx.bbmm_setup(_problem(w, inputs.MATERIALISED))
    with pytest.raises(binding.BbmmError):
        ctx.bbmm_kernel_mm(inputs.MATERIALISED, _dev(np.ones((50, 3))))


def test_nan_in_targets_is_reported_not_propagated_silently(ctx):
    from paper_1809_11165_amd import binding
    w = inputs.tiny(64, 3, t=3, k=2, iters=4)
    w.y[5] = np.nan
    with pytest.raises(binding.BbmmError) as ei:
        ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
    assert ei.value.code == binding.ENONFINITE


# ------------------------------ default work plans of the products over sizes -----
@pytest.mark.parametrize("n", [1000, 2500, 4100, 5000, 10000, 17000, 20000, 30000])
def test_products_with_their_default_plans_on_sampled_rows(ctx, n):
    # the default number of workgroups depends on how the column strips divide the compute units
    # (a whole number per strip, fewer for short matrices): every branch of that choice, in all three
    # storages, against rows of the oracle's kernel matrix picked at random
    w = _case(inputs.RBF, True, n, 7)
    rng = np.random.default_rng(n + 1)
    rows = np.sort(rng.choice(n, size=40, replace=False))
    rows[0], rows[-1] = 0, n - 1
    Krows = O.kernel_block(w.kernel, w.X[rows], w.X, w.lengthscale, w.outputscale)
    for c in (11, 17):
        M = _dev(rng.standard_normal((n, c)))
        ref = Krows @ _host(M) + w.noise * _host(M)[rows]
        scale = np.max(np.abs(ref))
        ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
        got = _host(ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M))[rows]
        assert np.max(np.abs(got - ref)) < 1e-4 * scale, ("on the fly", c)
        for tri in (0, 1):
            try:
                ctx.bbmm_tune("khat_sym", tri)
                ctx.bbmm_setup(_problem(w, inputs.MATERIALISED))
                ctx.bbmm_build_khat()
                got = _host(ctx.bbmm_kernel_mm(inputs.MATERIALISED, M))[rows]
            finally:
                ctx.bbmm_tune("khat_sym", 0)
            assert np.max(np.abs(got - ref)) < 1e-4 * scale, ("triangle" if tri else "whole matrix", c)


# ------------------------------------- on-the-fly product, tile pairs once -----
@pytest.mark.parametrize("n", [300, 512, 523, 1030, 1600, 2100, 4200])
@pytest.mark.parametrize("c", [1, 11, 12, 13, 16])
def test_onthefly_product_with_each_tile_pair_once(ctx, n, c):
    # tiles on and above the diagonal only, each used for both of its contributions (the default from
    # 12288 rows on, forced here with the value 2); against the plain form (every tile evaluated) and
    # the oracle
    w = _case(inputs.MATERN52, True, n, 5)
    rng = np.random.default_rng(70 + c)
    M = _dev(rng.standard_normal((n, c)))
    ref = _khat(w) @ _host(M)
    ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
    try:
        ctx.bbmm_tune("otf_sym", 0)
        V0 = _host(ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M))
        ctx.bbmm_tune("otf_sym", 2)
        for wgs in (0, 1, 7, 300):
            ctx.bbmm_tune("otf_split", wgs)
            V1 = _host(ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M))
            assert _colrel(V1, V0) < 2e-7, wgs
            assert _colrel(V1, ref) < 1e-4, wgs
    finally:
        ctx.bbmm_tune("otf_sym", 1)
        ctx.bbmm_tune("otf_split", 0)


@pytest.mark.parametrize("kernel", [inputs.RBF, inputs.MATERN52])
@pytest.mark.parametrize("d", [1, 3, 4, 9, 16, 20, 32, 33, 64])
def test_onthefly_tile_pairs_once_over_input_dimensions(ctx, kernel, d):
    # d is padded to 4, 8, 16, 32 or 64 coordinates per point; up to 32 the paired form is available
    # (forced here), beyond it the plain one runs: either way the product must match the oracle
    n = 1600
    w = _case(kernel, True, n, d)
    rng = np.random.default_rng(170 + d)
    for c in (11, 16):
        M = _dev(rng.standard_normal((n, c)))
        ref = _khat(w) @ _host(M)
        ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
        try:
            ctx.bbmm_tune("otf_sym", 0)
            V0 = _host(ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M))
            ctx.bbmm_tune("otf_sym", 2)
            V1 = _host(ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M))
        finally:
            ctx.bbmm_tune("otf_sym", 1)
        assert _colrel(V1, V0) < 2e-7, c
        assert _colrel(V1, ref) < 1e-4, c
        assert _colrel(V0, ref) < 1e-4, c


def test_onthefly_default_form_depends_on_the_size(ctx):
    # by default the paired form runs from 12288 (padded) rows on: there the default must be the forced
    # paired product bit for bit, below it the plain one; sampled rows against the oracle's kernel rows
    for n, paired in ((4000, False), (12500, True)):
        w = _case(inputs.MATERN52, True, n, 6)
        rng = np.random.default_rng(n)
        M = _dev(rng.standard_normal((n, 11)))
        ctx.bbmm_setup(_problem(w, inputs.ONTHEFLY))
        try:
            Vd = ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M)
            ctx.bbmm_tune("otf_sym", 0)
            V0 = ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M)
            ctx.bbmm_tune("otf_sym", 2)
            V2 = ctx.bbmm_kernel_mm(inputs.ONTHEFLY, M)
        finally:
            ctx.bbmm_tune("otf_sym", 1)
        assert torch.equal(Vd, V2 if paired else V0), n
        rows = rng.choice(n, size=48, replace=False)
        Krows = O.kernel_block(w.kernel, w.X[rows], w.X, w.lengthscale, w.outputscale)
        ref = Krows @ _host(M) + w.noise * _host(M)[rows]
        for V in (V0, V2):
            got = _host(V)[rows]
            assert np.max(np.abs(got - ref)) < 1e-4 * np.max(np.abs(ref)), n


def test_onthefly_forms_agree_on_the_whole_call(ctx):
    w = inputs.make(3, n=2300)
    try:
        ctx.bbmm_tune("otf_sym", 0)
        a = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
        ctx.bbmm_tune("otf_sym", 2)
        b = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.ONTHEFLY))
    finally:
        ctx.bbmm_tune("otf_sym", 1)
    assert a.pivots.tolist() == b.pivots.tolist()
    assert _colrel(_host(a.U), _host(b.U)) < 1e-5
    assert a.logdet == pytest.approx(b.logdet, rel=1e-8)
    assert np.allclose(a.trace, b.trace, rtol=1e-6)
