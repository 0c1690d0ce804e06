"""Full-size GPU parity: the benchmark configurations at (or near) their stated sizes, in the
launch configuration bench.py times.

Where the fp64 oracle needs minutes, its results are stored under tests/golden/ by
tests/golden/make_golden.py (which calls only the oracle); the comparison is then on the stored
scalars and on EVERY row of the solves (<case>_U.npy; at n = 500,000 every row of u_0 and every
8th row of the probe solves).  Each configuration is compared twice: at a "converged cap"
(`*_capN`: the iteration count raised until the oracle's last update is ~1e-5 of the iterate),
where every solve column, the log-det, y^T K^-1 y and every trace / quadratic term are held to the
plain 1e-3; and at the cap the configuration states, where the iterate is only defined up to the
distance between fp64 runs of the oracle itself (see _iterate_tolerance).  Where even the stored
route is out of reach (n = 200,000) the checks are on sampled outputs the oracle computes one by
one in fp64 and on properties that hold at any size."""
import json
import os

import numpy as np
import pytest

from oracle import bbmm_oracle as O
from paper_1809_11165_amd import inputs

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def ctx():
    from paper_1809_11165_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def _problem(w, mode):
    from paper_1809_11165_amd import binding
    return binding.problem_from_workload(w, mode)


def _load(name):
    path = os.path.join(GOLDEN, name + ".json")
    if not os.path.exists(path):
        pytest.skip("stored oracle result %s.json has not been generated" % name)
    with open(path) as f:
        return json.load(f)


TOL = 1e-3          # the parity bound on solves, log-det and traces

# Every full-size comparison also writes what it measured (one JSON line per case) so that the
# margin to the bound is on record, not only pass / fail: to the file named by BBMM_PARITY_LOG,
# else to a file in the temporary directory.
import tempfile  # noqa: E402

MEASURED = os.environ.get("BBMM_PARITY_LOG", os.path.join(tempfile.gettempdir(), "bbmm_parity_measured.jsonl"))


def _record(case, **values):
    try:
        os.makedirs(os.path.dirname(os.path.abspath(MEASURED)), exist_ok=True)
        with open(MEASURED, "a") as f:
            f.write(json.dumps(dict(case=case, **{k: (v.tolist() if hasattr(v, "tolist") else v)
                                                  for k, v in values.items()})) + "\n")
    except OSError:
        pass


def _iterate_tolerance(g):
    """Bound for comparing the iterate U_p itself.

    The scalars (log-det, y^T K^-1 y, NLML, traces) are held to TOL everywhere.  The iterate is
    held to TOL wherever it is defined that sharply -- every converged-cap case.  At an
    unconverged cap CG amplifies any perturbation by ~100x per iteration once the leading Ritz
    values have converged (iteration ~15 on these problems), until two runs that are each correct
    sit a fraction of an iteration apart.  The oracle measures this on itself, with no GPU
    involved: "U_last_step" is the size of its final update |U_p - U_(p-1)| / |U_p|,
    "U_reorder_dev" the distance between two fp64 runs that differ only in the order their
    K_hat.M products are summed, "U_fp32_dev" the distance to a third fp64 run whose matrix
    entries were rounded once to float32 (the precision the paper runs in and the HIP path stores
    the matrix in).  Those distances are single samples of a chaotic amplification, not constants:
    over the configurations the HIP path lands between 1.2 and 4.5 times the larger of them
    (the three product modes, which differ among themselves in nothing but the order of the sums,
    spread over 2.1e-3 .. 2.8e-3 on configuration 3), so no fixed multiple of one sample is a
    bound.  What does bound the distance of two correct runs is one update of the iteration: the
    GPU iterate must lie within the oracle's last update (largest column) of the oracle's; where
    the run has converged that is below TOL and TOL applies.  The measured distance and the three
    oracle-only measures are recorded for every case (see _record)."""
    return max(TOL, float(np.max(g["U_last_step"])))


def _solve_errors(res, name, g):
    """Column-wise |U_gpu - U_oracle| / |U_oracle| over every stored row of the oracle's solves."""
    Uref = np.load(os.path.join(GOLDEN, name + "_U.npy")).astype(np.float64)
    every = int(g.get("U_rows_every", 1))
    U = res.U[::every].cpu().numpy().astype(np.float64)
    assert U.shape == Uref.shape
    err = np.linalg.norm(U - Uref, axis=0) / np.linalg.norm(Uref, axis=0)
    # the worst single row (relative to the column's root-mean-square entry): a wrong row shows here
    rms = np.linalg.norm(Uref, axis=0) / np.sqrt(Uref.shape[0])
    worst_row = float(np.max(np.abs(U - Uref) / rms))
    if every > 1:
        u0ref = np.load(os.path.join(GOLDEN, name + "_u0.npy")).astype(np.float64)
        u0 = res.u0.cpu().numpy().astype(np.float64)
        err[0] = np.linalg.norm(u0 - u0ref) / np.linalg.norm(u0ref)
        worst_row = max(worst_row, float(np.max(np.abs(u0 - u0ref)) / (np.linalg.norm(u0ref) / np.sqrt(u0ref.size))))
    return err, worst_row


def _compare_with_golden(res, g, w, name, case=""):
    tol_u = _iterate_tolerance(g)
    err, worst_row = _solve_errors(res, name, g)
    rel = lambda a, b: float(abs(a - b) / abs(b))
    tr, qd, gr = np.array(g["trace"]), np.array(g["quad"]), np.array(g["grad"])
    _record(case, n=g["n"], iters=g["iters_run"], solve_err_max=float(err.max()), solve_err_y=float(err[0]),
            worst_row=worst_row, bound=tol_u, U_last_step=float(np.max(g["U_last_step"])),
            U_reorder_dev=float(np.max(g["U_reorder_dev"])), U_fp32_dev=float(np.max(g["U_fp32_dev"])),
            logdet_err=rel(res.logdet, g["logdet"]), yKinvy_err=rel(res.yKinvy, g["yKinvy"]),
            trace_err=float(np.max(np.abs(res.trace - tr) / np.abs(tr))),
            quad_err=float(np.max(np.abs(res.quad - qd) / np.abs(qd))),
            logdet_vs_exact=rel(res.logdet, g["exact_logdet"]), oracle_logdet_vs_exact=rel(g["logdet"], g["exact_logdet"]))
    assert err.max() < tol_u, (err, tol_u)
    # no single row off by more than 30 bounds' worth of the column's typical entry
    assert worst_row < 30 * tol_u, worst_row
    coln = torch.linalg.vector_norm(res.U.double(), dim=0).cpu().numpy()
    assert np.allclose(coln, g["U_colnorm"], rtol=tol_u)
    assert res.logdet_precond == pytest.approx(g["logdet_precond"], rel=1e-5)
    assert res.logdet == pytest.approx(g["logdet"], rel=TOL)
    assert res.yKinvy == pytest.approx(g["yKinvy"], rel=TOL)
    assert res.nlml == pytest.approx(g["nlml"], rel=TOL)
    # u0^T (dK/dtheta) u0 is quadratic in the iterate u0: twice its bound
    tol_q = max(TOL, 2.0 * tol_u) if tol_u > TOL else TOL
    for h in range(len(tr)):
        assert abs(res.trace[h] - tr[h]) <= TOL * max(abs(tr[h]), 1e-3 * np.abs(tr).max()), h
        assert abs(res.quad[h] - qd[h]) <= tol_q * max(abs(qd[h]), 1e-3 * np.abs(qd).max()), h
        assert abs(res.grad_nlml[h] - gr[h]) <= (TOL * abs(tr[h]) + tol_q * abs(qd[h])) / 2 + 1e-9, h
    it = res.iters_run
    assert np.allclose(res.alpha[:min(it, 5)], np.array(g["alpha"])[:min(it, 5)], rtol=1e-4)
    # against the plain definition (dense Cholesky of K_hat, stored with the oracle's results).
    # The SLQ estimate with these t, p, k is itself 0.06-2 % from the exact log-determinant in
    # fp64 (estimator error; 2.1 % on configuration 3, whose log|K_hat| = -0.064 n nearly
    # cancels), so the GPU is required to be within 1e-2 where the oracle is, and nowhere
    # further from the exact value than the oracle plus the parity bound.
    exact = g["exact_logdet"]
    assert abs(res.logdet - exact) <= max(1e-2 * abs(exact), abs(g["logdet"] - exact) + TOL * abs(exact))
    if abs(g["logdet"] - exact) <= 0.9e-2 * abs(exact):
        assert res.logdet == pytest.approx(exact, rel=1e-2)
    oracle_gap = abs(g["yKinvy"] - g["exact_yKinvy"])
    assert abs(res.yKinvy - g["exact_yKinvy"]) <= oracle_gap + TOL * abs(g["exact_yKinvy"])


def _run_case(ctx, name, mode):
    from paper_1809_11165_amd import binding
    g = _load(name)
    w = inputs.make(g["config"], n=g["n"], iters=g["iters_cap"])
    w.tol = float(g["tol"])
    prob = _problem(w, mode)
    if g["tol"] > 0:
        # stop rule: the GPU must stop within a few iterations of the oracle, below the tolerance
        free = ctx.bbmm_solve_logdet_grad(prob, want_U=False)
        assert abs(free.iters_run - g["iters_run"]) <= 3
        if free.iters_run < g["iters_cap"]:
            assert free.resid[free.iters_run - 1].max() < g["tol"]
        else:                                   # cap reached: the oracle did not converge either
            assert g["iters_run"] == g["iters_cap"]
        # parity at the oracle's iteration count
        prob = binding.Problem(kernel=prob.kernel, mode=mode, X=prob.X, y=prob.y,
                               lengthscale=prob.lengthscale, outputscale=prob.outputscale,
                               noise=prob.noise, E1=prob.E1, E2=prob.E2, k=prob.k,
                               max_iters=g["iters_run"], tol=0.0)
    res = ctx.bbmm_solve_logdet_grad(prob)
    assert res.iters_run == g["iters_run"]
    assert res.pivots.tolist() == g["pivots"]
    _compare_with_golden(res, g, w, name, case="%s mode=%d tri=%d" % (name, mode, int(getattr(ctx, "_tri", 0))))
    return res, w, g


def _run_converged_case(ctx, name, mode):
    """A converged-cap case: the bound on every solve column is the plain TOL, and so is the bound
    on u_0^T (dK/dtheta) u_0."""
    res, w, g = _run_case(ctx, name, mode)
    assert _iterate_tolerance(g) == TOL and float(np.max(g["U_last_step"])) < 1e-4
    return res, w, g


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_config2_full_size_converged_cap(ctx, mode):
    # 160 fixed iterations: the oracle's last update is 5e-6 of the iterate
    _run_converged_case(ctx, "cfg2_n10000_cap160", mode)


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_config3_full_size_converged_cap(ctx, mode):
    # the benchmark problem (n = 50,000) at 100 iterations: last update 2e-6 of the iterate
    _run_converged_case(ctx, "cfg3_n50000_cap100", mode)


def test_converged_caps_triangle_storage(ctx):
    ctx.bbmm_tune("khat_sym", 1)
    ctx._tri = 1
    try:
        _run_converged_case(ctx, "cfg3_n50000_cap100", inputs.MATERIALISED)
        _run_converged_case(ctx, "cfg2_n10000_cap160", inputs.MATERIALISED)
    finally:
        ctx._tri = 0
        ctx.bbmm_tune("khat_sym", 0)


def test_config4_subsample_20000_converged_cap(ctx):
    _run_converged_case(ctx, "cfg4_sub_n20000_cap200", inputs.ONTHEFLY)


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_config2_full_size_tolerance_reached(ctx, mode):
    # cap raised from 50 to 128 so that the configured tolerance 1e-2 is reached (~95 iterations)
    _run_case(ctx, "cfg2_n10000_cap128", mode)


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_config2_full_size_as_configured(ctx, mode):
    # As configured the cap of 50 iterations ends the run at a relative residual of 0.2; the
    # iterate is compared within the bound of _iterate_tolerance, the scalars within TOL.
    _run_case(ctx, "cfg2_n10000", mode)


def test_config2_full_size_same_operator(ctx):
    """Oracle mBCG run on the very operands the GPU used -- its fp32 K_hat, its fp64 factor L and
    its right-hand-side block -- so that only the rounding order of the iteration differs.  The
    coefficients agree to 1e-6 while the recurrences are still well determined (the first 10
    iterations); at the unconverged 50-iteration cap the iterates agree within one update of the
    oracle's, and the log-det within 1e-3."""
    w = inputs.make(2)
    w.tol = 0.0
    ctx.bbmm_setup(_problem(w, inputs.MATERIALISED))
    ctx.bbmm_build_khat()
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    logdetP = ctx.bbmm_precond_setup()
    B = ctx.bbmm_make_probes()
    U, alpha, beta, resid, iters = ctx.bbmm_mbcg(inputs.MATERIALISED, B)
    logdet, terms = ctx.bbmm_slq_logdet()
    assert iters == 50
    Kh = ctx.bbmm_khat_block(0, w.n, 0, w.n).cpu().numpy().astype(np.float64)
    P = O.make_preconditioner(L.cpu().numpy().astype(np.float64), w.noise)
    Bh = B.cpu().numpy().astype(np.float64)
    ref = O.mbcg(lambda M: Kh @ M, Bh, P.solve, 50)
    prev = O.mbcg(lambda M: Kh @ M, Bh, P.solve, 49)
    norm = lambda A: np.linalg.norm(A, axis=0)
    last_step = (norm(ref.U - prev.U) / norm(ref.U)).max()
    Ug = U.cpu().numpy().astype(np.float64)
    err = norm(Ug - ref.U) / norm(ref.U)
    assert err.max() < max(1e-3, last_step), (err, last_step)
    assert np.allclose(alpha[:10], ref.alpha[:10], rtol=1e-6)
    assert np.allclose(beta[:10], ref.beta[:10], rtol=1e-6)
    ref_terms = [ref.rho0[i + 1] * O.e1_logT_e1(*O.tridiag_from_cg(ref.alpha[:, i + 1], ref.beta[:, i + 1], 50))
                 for i in range(w.t)]
    assert logdet == pytest.approx(P.logdet + np.mean(ref_terms), rel=1e-3)


@pytest.mark.parametrize("mode", [inputs.MATERIALISED, inputs.ONTHEFLY])
def test_config3_full_size(ctx, mode):
    _run_case(ctx, "cfg3_n50000", mode)


def test_config3_full_size_triangle_storage(ctx):
    # the reduced-traffic materialised mode: upper triangle of K_hat only, every tile used twice
    ctx.bbmm_tune("khat_sym", 1)
    ctx._tri = 1
    try:
        _run_case(ctx, "cfg3_n50000", inputs.MATERIALISED)
    finally:
        ctx._tri = 0
        ctx.bbmm_tune("khat_sym", 0)


def test_config2_full_size_triangle_storage(ctx):
    ctx.bbmm_tune("khat_sym", 1)
    ctx._tri = 1
    try:
        _run_case(ctx, "cfg2_n10000_cap128", inputs.MATERIALISED)
        _run_case(ctx, "cfg2_n10000", inputs.MATERIALISED)
    finally:
        ctx._tri = 0
        ctx.bbmm_tune("khat_sym", 0)


def test_config4_subsample_20000(ctx):
    _run_case(ctx, "cfg4_sub_n20000", inputs.ONTHEFLY)


def test_config4_full_size_first_iterations(ctx):
    """n = 200,000 (on-the-fly only): three mBCG iterations against the oracle run matrix-free at
    the same size.  No Ritz value has converged yet, so coefficients and iterates are sharply
    defined and are held far tighter than the 1e-3 bound."""
    from paper_1809_11165_amd import binding
    g = _load("cfg4_n200000_p3")
    w = inputs.make(4, iters=g["iters_run"])
    prob = _problem(w, inputs.ONTHEFLY)
    res = ctx.bbmm_solve_logdet_grad(prob)
    assert res.iters_run == g["iters_run"] == 3
    assert res.pivots.tolist() == g["pivots"]
    assert res.logdet_precond == pytest.approx(g["logdet_precond"], rel=1e-6)
    assert np.allclose(res.alpha, g["alpha"], rtol=1e-5)
    assert np.allclose(res.beta, g["beta"], rtol=1e-5)
    assert np.allclose(res.resid, g["resid"], rtol=1e-5)
    rows = np.array(g["sample_rows"])
    Ug = np.array(g["U_sample"])
    U = res.U[torch.from_numpy(rows).to(res.U.device)].cpu().numpy().astype(np.float64)
    err = np.linalg.norm(U - Ug, axis=0) / np.linalg.norm(Ug, axis=0)
    assert err.max() < 1e-5, err
    coln = torch.linalg.vector_norm(res.U.double(), dim=0).cpu().numpy()
    assert np.allclose(coln, g["U_colnorm"], rtol=1e-5)


# ------------------------------------------------------------ SGPR, configuration 5 -----
def _run_sgpr_case(ctx, name):
    """Configuration 5 against the stored results of oracle/sgpr_oracle.py.

    The inducing rows of an SoR matrix have residual diagonals that agree to ~1e-10 (1 - Q_ii =
    jitter-sized), so the greedy pivot order is decided by rounding and differs between the fp64
    oracle and a root stored in fp32; both orders are valid.  The stored results belong to the
    oracle's order, so the GPU replays that order (pivots_in) and is then compared like the
    exact-GP configurations.  With sigma^2 = 0.01 the run is far from converged after 50
    iterations (relative residual ~2), which is where the stored measures of how sharply the
    iterate and the heavily cancelling derivative terms are defined come in: "U_last_step",
    the second fp64 run with another rounding order ("U_reorder_dev", "trace_alt", "quad_alt") and
    the first-order sensitivities "trace_sens", "quad_sens"."""
    from paper_1809_11165_amd import binding
    g = _load(name)
    w = inputs.make(g["config"], n=g["n"], m=g["m"])
    prob = _problem(w, inputs.SGPR)
    prob.pivots_in = np.array(g["pivots"], dtype=np.int64)
    res = ctx.bbmm_solve_logdet_grad(prob)
    assert res.iters_run == g["iters_run"]
    assert res.pivots.tolist() == g["pivots"]
    assert res.logdet_precond == pytest.approx(g["logdet_precond"], rel=1e-6)
    # early coefficients: no Ritz value has converged yet, so they are sharply defined
    assert np.allclose(res.alpha[:5], np.array(g["alpha"])[:5], rtol=1e-4)
    assert np.allclose(res.beta[:5], np.array(g["beta"])[:5], rtol=1e-4)
    tol_u = _iterate_tolerance(g)
    rows = np.array(g["sample_rows"])
    Ug = np.array(g["U_sample"])
    U = res.U[torch.from_numpy(rows).to(res.U.device)].cpu().numpy().astype(np.float64)
    err, worst_row = _solve_errors(res, name, g)
    assert worst_row < 30 * tol_u, worst_row
    _record(name, worst_row=worst_row, U_fp32_dev=float(np.max(g["U_fp32_dev"])), n=g["n"], iters=g["iters_run"], solve_err_max=float(err.max()), solve_err_y=float(err[0]),
            bound=tol_u, U_last_step=float(np.max(g["U_last_step"])), U_reorder_dev=float(np.max(g["U_reorder_dev"])),
            logdet_err=float(abs(res.logdet - g["logdet"]) / abs(g["logdet"])),
            yKinvy_err=float(abs(res.yKinvy - g["yKinvy"]) / abs(g["yKinvy"])),
            trace_err=(np.abs(res.trace - np.array(g["trace"])) / np.abs(np.array(g["trace"]))),
            quad_err=(np.abs(res.quad - np.array(g["quad"])) / np.abs(np.array(g["quad"]))))
    assert err.max() < tol_u, (err, tol_u)
    coln = torch.linalg.vector_norm(res.U.double(), dim=0).cpu().numpy()
    assert np.allclose(coln, g["U_colnorm"], rtol=tol_u)
    # y^T u_p grows monotonically with p (CG minimises the energy norm of the error), so two runs
    # a fraction of an iteration apart differ by at most the last increment, which the oracle
    # stores ("yKinvy_prev"); the same for the quadrature estimate of the log-determinant.  Both
    # increments vanish when the run has converged, leaving the plain 1e-3.
    b_ld = TOL * abs(g["logdet"]) + abs(g["logdet"] - g["logdet_prev"])
    b_yk = TOL * abs(g["yKinvy"]) + abs(g["yKinvy"] - g["yKinvy_prev"])
    assert abs(res.logdet - g["logdet"]) <= b_ld
    assert abs(res.yKinvy - g["yKinvy"]) <= b_yk, (res.yKinvy, g["yKinvy"], g["yKinvy_prev"], g["yKinvy_alt"])
    assert abs(res.nlml - g["nlml"]) <= (b_ld + b_yk) / 2
    assert abs(g["yKinvy_alt"] - g["yKinvy"]) <= b_yk          # the second fp64 run is inside the bound
    tr, qd = np.array(g["trace"]), np.array(g["quad"])
    nl = len(w.lengthscale)
    # Derivative terms.  u^T dQ w is a small difference of terms as large as |u| |dQ w| (e.g.
    # u_0^T Q u_0 = y^T u_0 - sigma^2 |u_0|^2 up to the residual), so a bound relative to its own
    # value would ask for more than the iterate is defined to.  Two measures from the oracle alone
    # of how sharply a term is defined at this iteration count:
    #   * its last increment |term_p - term_(p-1)| ("trace_prev", "quad_prev"): two runs a
    #     fraction of an iteration apart differ by a fraction of it -- this is what moves the
    #     y-column terms, whose error lies in the Krylov space of y itself;
    #   * its Cauchy-Schwarz sensitivity "sens" to a change of the solves by eps of their norm:
    #     a change uncorrelated with dQ w moves the term by eps sens / sqrt(n); the GPU solves may
    #     differ by tol_u, and a factor 4 allows for correlation.
    # Hence  |term_gpu - term_oracle| <= 1e-3 |term| + increment + 4 tol_u sens / sqrt(n)
    #                                    + 1e-6 (noise term),
    # the last being what fp32 storage of the root resolves at the size of |u| |w|.  All of these
    # vanish (up to 1e-3 and the fp32 floor) for a converged run.  The kernels that form the terms
    # are held to tight bounds on identical inputs in
    # tests/test_gpu_sgpr.py::test_sgpr_dk_traces_match_oracle_formulas.
    tsens, qsens = np.array(g["trace_sens"]), np.array(g["quad_sens"])
    tinc, qinc = np.abs(np.array(g["trace_prev"]) - tr), np.abs(np.array(g["quad_prev"]) - qd)
    rn = np.sqrt(g["n"])
    for h in range(len(tr)):
        btr = TOL * abs(tr[h]) + tinc[h] + 4 * tol_u * tsens[h] / rn + 1e-6 * abs(tr[nl + 1])
        bqd = TOL * abs(qd[h]) + qinc[h] + 4 * tol_u * qsens[h] / rn + 1e-6 * abs(qd[nl + 1])
        assert abs(res.trace[h] - tr[h]) <= btr, (h, res.trace[h], tr[h], btr)
        assert abs(res.quad[h] - qd[h]) <= bqd, (h, res.quad[h], qd[h], bqd)
        assert abs(res.grad_nlml[h] - g["grad"][h]) <= (btr + bqd) / 2 + 1e-9, h
    # the second fp64 run (products in another rounding order) is itself inside those bounds
    dev = float(np.max(g["U_reorder_dev"]))
    assert np.all(np.abs(np.array(g["trace_alt"]) - tr) <= TOL * np.abs(tr) + dev * tsens / rn + 1e-9)
    assert np.all(np.abs(np.array(g["quad_alt"]) - qd) <= TOL * np.abs(qd) + dev * qsens / rn + 1e-9)
    # the plain definition (Woodbury identity, stored): log-det within 1e-2 where the oracle's own
    # estimate is, else no further than the oracle plus the parity bound; solve no further from
    # the exact one than the oracle's iterate is
    exact = g["exact_logdet"]
    assert abs(res.logdet - exact) <= max(1e-2 * abs(exact), abs(g["logdet"] - exact) + TOL * abs(exact))
    ue = np.array(g["u0_sample_exact"])
    gap_oracle = np.linalg.norm(Ug[:, 0] - ue) / np.linalg.norm(ue)
    assert np.linalg.norm(U[:, 0] - ue) / np.linalg.norm(ue) <= gap_oracle + tol_u
    return res, w, g


def _run_sgpr_converged_case(ctx, name):
    """Configuration 5 with the cap raised from 50 to 128 iterations, where the oracle's last update
    is ~1e-5 of the iterate: every solve column, the log-det, y^T K^-1 y, the NLML and the noise
    terms are held to the plain 1e-3.  The lengthscale and outputscale terms u^T dQ w are
    differences of terms thousands of times their size (u^T Q w = z^T w - sigma^2 u^T w up to the
    residual), i.e. conditioned ~1e3-1e4 with respect to the solves: the oracle's own third fp64
    run, through its root rounded once to float32, moves U by 4e-6 and these terms by up to 3e-2 of
    their values ("trace_fp32", "quad_fp32").  Their bound is therefore 1e-3 of the term plus what
    the measured distance eps of the GPU's solves explains: the oracle stores the Cauchy-Schwarz
    bounds "trace_sens", "quad_sens" (|delta term| <= eps * sens when every column moves by eps of
    its norm; the terms' condition numbers sens / |term| are 1e4-1e5 here); a perturbation of the
    solves that is uncorrelated with (dQ) w moves a term by eps * sens / sqrt(n), and a factor
    allows for correlation: 10 here, chosen on oracle-only data -- the oracle's own float32-root
    run with its own distance needs 5.6 at n = 500,000 (where the terms' condition numbers reach
    1e6) and 3.2 at n = 50,000, and is asserted to stay inside the same model below: if that
    assertion fails the model is wrong, not the GPU.  In units of their natural scale sens the
    GPU's terms are off by 6e-8 at most, i.e. at float32 rounding of the root."""
    g = _load(name)
    w = inputs.make(g["config"], n=g["n"], m=g["m"], iters=g["iters_cap"])
    prob = _problem(w, inputs.SGPR)
    prob.pivots_in = np.array(g["pivots"], dtype=np.int64)
    res = ctx.bbmm_solve_logdet_grad(prob)
    assert res.iters_run == g["iters_run"] == g["iters_cap"]
    assert res.pivots.tolist() == g["pivots"]
    assert _iterate_tolerance(g) == TOL and float(np.max(g["U_last_step"])) < 1e-4
    err, worst_row = _solve_errors(res, name, g)
    tr, qd = np.array(g["trace"]), np.array(g["quad"])
    t32, q32 = np.array(g["trace_fp32"]), np.array(g["quad_fp32"])
    tsens, qsens = np.array(g["trace_sens"]), np.array(g["quad_sens"])
    _record(name, n=g["n"], iters=g["iters_run"], solve_err_max=float(err.max()), solve_err_y=float(err[0]),
            worst_row=worst_row, bound=TOL, U_last_step=float(np.max(g["U_last_step"])),
            U_reorder_dev=float(np.max(g["U_reorder_dev"])), U_fp32_dev=float(np.max(g["U_fp32_dev"])),
            logdet_err=float(abs(res.logdet - g["logdet"]) / abs(g["logdet"])),
            yKinvy_err=float(abs(res.yKinvy - g["yKinvy"]) / abs(g["yKinvy"])),
            trace_err=np.abs(res.trace - tr) / np.abs(tr), quad_err=np.abs(res.quad - qd) / np.abs(qd),
            trace_fp32_dev=np.abs(t32 - tr) / np.abs(tr), quad_fp32_dev=np.abs(q32 - qd) / np.abs(qd),
            trace_condition=tsens / np.abs(tr), quad_condition=qsens / np.abs(qd))
    assert err.max() < TOL, err
    assert worst_row < 30 * TOL
    assert res.logdet_precond == pytest.approx(g["logdet_precond"], rel=1e-6)
    assert res.logdet == pytest.approx(g["logdet"], rel=TOL)
    assert res.yKinvy == pytest.approx(g["yKinvy"], rel=TOL)
    assert res.nlml == pytest.approx(g["nlml"], rel=TOL)
    assert np.allclose(res.alpha[:5], np.array(g["alpha"])[:5], rtol=1e-4)
    nl = len(w.lengthscale)
    # the noise terms (dK_hat/dsigma^2 = I) do not cancel: plain 1e-3
    assert res.trace[nl + 1] == pytest.approx(tr[nl + 1], rel=TOL)
    assert res.quad[nl + 1] == pytest.approx(qd[nl + 1], rel=TOL)
    eps_u, eps_0 = float(err[1:].max()), float(err[0])
    rn = np.sqrt(g["n"])
    dev = float(np.max(g["U_fp32_dev"]))
    for h in range(nl + 1):
        btr = TOL * abs(tr[h]) + 10.0 * eps_u * tsens[h] / rn
        bqd = TOL * abs(qd[h]) + 10.0 * eps_0 * qsens[h] / rn
        assert abs(res.trace[h] - tr[h]) <= btr, (h, res.trace[h], tr[h], btr)
        assert abs(res.quad[h] - qd[h]) <= bqd, (h, res.quad[h], qd[h], bqd)
        assert abs(res.grad_nlml[h] - g["grad"][h]) <= (btr + bqd) / 2 + 1e-9, h
        assert abs(t32[h] - tr[h]) <= 10.0 * dev * tsens[h] / rn + 1e-9 * abs(tr[h]), h
        assert abs(q32[h] - qd[h]) <= 10.0 * dev * qsens[h] / rn + 1e-9 * abs(qd[h]), h
        # and in units of the term's natural scale the GPU is at float32 rounding of the root
        assert abs(res.trace[h] - tr[h]) <= 5e-7 * tsens[h] and abs(res.quad[h] - qd[h]) <= 5e-7 * qsens[h], h
    assert res.grad_nlml[nl + 1] == pytest.approx(g["grad"][nl + 1], rel=TOL)
    # the plain definition (Woodbury identity): log-det within 1e-2, the solve as close as the oracle's
    assert res.logdet == pytest.approx(g["exact_logdet"], rel=1e-2)
    return res, w, g


def test_config5_subsample_50000_converged_cap(ctx):
    _run_sgpr_converged_case(ctx, "cfg5_sub_n50000_cap128")


def test_config5_full_size_converged_cap(ctx):
    _run_sgpr_converged_case(ctx, "cfg5_n500000_cap128")


def test_config5_subsample_50000(ctx):
    res, w, g = _run_sgpr_case(ctx, "cfg5_sub_n50000")
    # the GPU's own greedy pivots (no pivots_in): a valid order -- every pivot attains the largest
    # residual diagonal of the oracle's factorisation replayed along that order, within 1e-4
    from oracle import sgpr_oracle as S
    free = ctx.bbmm_solve_logdet_grad(_problem(w, inputs.SGPR), want_U=False)
    assert free.rank == w.k and len(set(free.pivots.tolist())) == w.k
    parts = S.sor_parts(w.kernel, w.X, w.Uind, w.lengthscale, w.outputscale, w.noise, w.jitter_rel)
    diag = parts.q_diag()
    Lf, pf, dmax = O.pivoted_cholesky(diag, parts.q_row, w.k, forced_pivots=free.pivots)
    delta = diag.copy()
    for m in range(w.k):
        assert delta[free.pivots[m]] >= dmax[m] * (1 - 1e-4)
        delta = delta - Lf[:, m] ** 2
    # and a result of the same quality: log-det estimate within 1e-2 of the exact value
    assert free.logdet == pytest.approx(g["exact_logdet"], rel=1e-2)


def test_config5_full_size(ctx):
    res, w, g = _run_sgpr_case(ctx, "cfg5_n500000")
    assert res.iters_run == 50


# ------------------------------------------------------------ sampled fp64 audits -----
def _khat_rows_f64(w, rows):
    K = O.kernel_block(w.kernel, w.X[rows], w.X, w.lengthscale, w.outputscale)
    K[np.arange(len(rows)), rows] += w.noise
    return K


def _audit(ctx, w, mode, n_rows=256):
    """Sampled-row checks that need O(n) oracle work per row."""
    rng = np.random.default_rng(12345)
    rows = np.sort(rng.choice(w.n, size=n_rows, replace=False))
    Krows = _khat_rows_f64(w, rows)                        # fp64, straight from X
    prob = _problem(w, mode)
    # (1) one product on a random block, sampled rows
    ctx.bbmm_setup(prob)
    if mode == inputs.MATERIALISED:
        ctx.bbmm_build_khat()
    M = torch.randn(w.n, w.t + 1, device="cuda:0", generator=torch.Generator("cuda:0").manual_seed(3))
    V = ctx.bbmm_kernel_mm(mode, M)
    ref = Krows @ M.cpu().numpy().astype(np.float64)
    got = V[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - ref)) < 1e-4 * np.max(np.abs(ref))
    # (2) pivoted Cholesky: greedy property and factor against the oracle replaying the pivots,
    #     rows of K_XX produced on demand in fp64
    L, piv, rank = ctx.bbmm_pivoted_cholesky()
    assert rank == w.k
    Xd = w.X.astype(np.float64)
    get_row = lambda i: O.kernel_block(w.kernel, Xd[i:i + 1], Xd, w.lengthscale, w.outputscale)[0]
    diag = np.full(w.n, w.outputscale)
    Lf, pf, dmax = O.pivoted_cholesky(diag, get_row, w.k, forced_pivots=piv)
    delta = diag.copy()
    for m in range(w.k):
        assert delta[piv[m]] >= dmax[m] * (1 - 1e-4)       # the GPU pivot attains the maximum
        delta = delta - Lf[:, m] ** 2
    Lh = L.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(Lh - Lf)) < 1e-5
    logdetP = ctx.bbmm_precond_setup()
    assert logdetP == pytest.approx(O.make_preconditioner(Lh, w.noise).logdet, rel=1e-10)
    # (3) whole call: independent fp64 residual of the returned solve on the sampled rows
    res = ctx.bbmm_solve_logdet_grad(prob)
    u0 = res.u0.cpu().numpy().astype(np.float64)
    r = w.y[rows].astype(np.float64) - Krows @ u0
    est = np.sqrt(np.mean(r * r) * w.n) / np.linalg.norm(w.y.astype(np.float64))
    reported = res.resid[res.iters_run - 1, 0]
    # sampled estimate of |y - K_hat u0| / |y| against the recurrence residual the GPU reports
    # (fp32 output rounding of u0 adds ~1e-7 |K_hat| |u0| / |y|)
    floor = 1e-6 * np.linalg.norm(Krows, axis=1).max() * np.linalg.norm(u0) / np.linalg.norm(w.y)
    assert est < 3.0 * reported + floor
    # (4) identities that tie the trace outputs to the solves (K_hat u_i = z_i up to the residual):
    #     u0^T K u0 = y^T u0 - sigma^2 |u0|^2   =>   quad[outputscale] = that / s
    nl = len(w.lengthscale)
    ident = (res.yKinvy - w.noise * res.quad[nl + 1]) / w.outputscale
    assert res.quad[nl] == pytest.approx(ident, rel=max(1e-3, 10 * reported))
    return res


def test_config3_full_size_audit_materialised(ctx):
    _audit(ctx, inputs.make(3), inputs.MATERIALISED)


def test_config3_full_size_audit_triangle_storage(ctx):
    ctx.bbmm_tune("khat_sym", 1)
    try:
        _audit(ctx, inputs.make(3), inputs.MATERIALISED)
    finally:
        ctx.bbmm_tune("khat_sym", 0)


def test_triangle_storage_audit_at_n_100000(ctx):
    # twice the benchmark size: 98 panels, i.e. more partial-result slots per row (up to 98) than
    # the other modes ever use, 20 GB of stored triangle
    ctx.bbmm_tune("khat_sym", 1)
    try:
        _audit(ctx, inputs.make(3, n=100000), inputs.MATERIALISED)
    finally:
        ctx.bbmm_tune("khat_sym", 0)


def test_config3_full_size_audit_onthefly(ctx):
    _audit(ctx, inputs.make(3), inputs.ONTHEFLY)


def test_config4_full_size_audit(ctx):
    # n = 200,000, t = 16, 100 iterations, on-the-fly only (K_hat would be 160 GB)
    res = _audit(ctx, inputs.make(4), inputs.ONTHEFLY)
    assert res.iters_run == 100
    sub = _load("cfg4_sub_n20000")
    # same mixture at 10x the points: log-det per point stays in the same range
    assert 0.3 < (res.logdet / 200000) / (sub["logdet"] / 20000) < 3.0


@pytest.mark.parametrize("storage", ["whole matrix", "triangle"])
def test_materialised_product_at_n_200000_on_sampled_rows(storage):
    """The largest n of the configurations with K_hat in HBM (Sec. 3, materialised form): 160 GB as a
    whole matrix, 87 GB as its upper triangle -- element offsets far beyond 2^32.  17 columns as in
    config 4 (two 16-column passes over the triangle).  Rows of the product picked at random, and
    the first and last, against the oracle's kernel rows in fp64."""
    from paper_1809_11165_amd import binding
    w = inputs.make(4)
    n, c = w.X.shape[0], w.t + 1
    assert n == 200000 and c == 17
    rng = np.random.default_rng(2024)
    rows = np.sort(rng.choice(n, size=48, replace=False))
    rows[0], rows[-1] = 0, n - 1
    M = rng.standard_normal((n, c)).astype(np.float32)
    Krows = O.kernel_block(w.kernel, w.X[rows], w.X, w.lengthscale, w.outputscale)
    ref = Krows @ M.astype(np.float64) + w.noise * M[rows].astype(np.float64)
    own = binding.Context(0)                 # its own context: the matrix is freed with it
    try:
        own.bbmm_tune("khat_sym", 1 if storage == "triangle" else 0)
        own.bbmm_setup(_problem(w, inputs.MATERIALISED))
        own.bbmm_build_khat()
        V = own.bbmm_kernel_mm(inputs.MATERIALISED, torch.from_numpy(M).to("cuda:0"))
        got = V[torch.from_numpy(rows).to("cuda:0")].cpu().numpy().astype(np.float64)
        finite = bool(torch.isfinite(V).all().item())
    finally:
        own.close()
    assert finite
    err = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
    _record("materialised_n200000_" + storage.replace(" ", "_"), product_rows_max_err=err)
    assert err < 1e-5
