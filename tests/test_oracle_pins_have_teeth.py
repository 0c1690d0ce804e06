"""The pins of tests/test_oracle_pins.py must fail when the oracle is wrong (CPU only).

Each case plants ONE plausible mistake in oracle/bbmm_oracle.py -- the printed-but-garbled
variants of Alg. 1/2, the Observation of App. A and the Woodbury formulas of App. C that the
oracle's readings reject, a dropped factor, a wrong power, a wrong index -- by rebuilding the
function from its own source with one expression changed (the mistake lives in this process
only), and asserts that the pin named beside it does NOT pass.  The unmutated oracle passes all
of them in test_oracle_pins.py."""
import inspect
import textwrap

import numpy as np
import pytest

import test_oracle_pins as pins
import test_sgpr_oracle_pins as spins
from oracle import bbmm_oracle as O
from oracle import sgpr_oracle as S


def _mutated(fn, old, new, count=1, module=O):
    """`fn` rebuilt from its source with `old` replaced by `new`, in its module's namespace."""
    src = textwrap.dedent(inspect.getsource(fn))
    assert src.count(old) >= 1, "the mutation target %r is not in %s" % (old, fn.__name__)
    src = src.replace(old, new, count)
    ns = dict(vars(module))
    exec(compile(src, "<mutated %s>" % fn.__name__, "exec"), ns)
    return ns[fn.__name__]


def _mutated_method(cls, name, old, new):
    fn = _mutated(getattr(cls, name), old, new)
    return fn


# (what is planted, attribute of the oracle module, mutated callable factory, pin, pin arguments)
CASES = [
    ("Alg. 1/2 as printed: d <- z - beta d",
     "mbcg", lambda: _mutated(O.mbcg, "D = Z + D * beta", "D = Z - D * beta"),
     pins.test_cg_with_p_equal_n_is_the_cholesky_solve, ()),
    ("residual update with the wrong sign: r <- r + alpha v",
     "mbcg", lambda: _mutated(O.mbcg, "R = R - V * alpha", "R = R + V * alpha"),
     pins.test_cg_with_p_equal_n_is_the_cholesky_solve, ()),
    ("beta from the printed unpreconditioned form r.r / r.r",
     "mbcg", lambda: _mutated(O.mbcg, "rho_new = np.sum(R * Z, axis=0)", "rho_new = np.sum(R * R, axis=0)"),
     pins.test_cg_with_p_equal_n_is_the_cholesky_solve, ()),
    ("Alg. 2 as printed: off-diagonal sqrt(beta_{j-1}) / alpha_j",
     "tridiag_from_cg", lambda: _mutated(O.tridiag_from_cg, "off[j - 1] = np.sqrt(beta[j - 1]) / alpha[j - 1]",
                                          "off[j - 1] = np.sqrt(beta[j - 1]) / alpha[j]"),
     pins.test_cg_tridiagonal_equals_explicit_lanczos_of_preconditioned_matrix, (3,)),
    ("diagonal of T without the beta / alpha term",
     "tridiag_from_cg", lambda: _mutated(O.tridiag_from_cg, "dg[j] += beta[j - 1] / alpha[j - 1]", "dg[j] += 0.0"),
     pins.test_cg_tridiagonal_equals_explicit_lanczos_of_preconditioned_matrix, (0,)),
    ("quadrature weights from the LAST row of the eigenvector matrix",
     "e1_logT_e1", lambda: _mutated(O.e1_logT_e1, "vec[0, :]", "vec[-1, :]"),
     pins.test_e1_logT_e1_is_gauss_quadrature_also_with_ghost_eigenvalues, ()),
    ("weights not squared",
     "e1_logT_e1", lambda: _mutated(O.e1_logT_e1, "vec[0, :] ** 2", "np.abs(vec[0, :])"),
     pins.test_slq_term_is_exact_quadratic_form_when_p_equals_n, ()),
    ("App. C as printed: capacitance matrix sigma^2 I - L^T L",
     "make_preconditioner", lambda: _mutated(O.make_preconditioner, "C = noise * np.eye(k) + L.T @ L",
                                              "C = noise * np.eye(k) - L.T @ L"),
     pins.test_woodbury_and_determinant_lemma_against_dense, ()),
    ("determinant lemma with n log sigma^2 instead of (n - k) log sigma^2",
     "make_preconditioner", lambda: _mutated(O.make_preconditioner, "(n - k) * np.log(noise)", "n * np.log(noise)"),
     pins.test_woodbury_and_determinant_lemma_against_dense, ()),
    ("probes with sigma^2 in place of sigma",
     "make_probes", lambda: _mutated(O.make_probes, "Z = np.sqrt(noise) * E2", "Z = noise * E2"),
     pins.test_probe_covariance_is_exactly_P_by_enumeration, ()),
    ("Sec. 2 as printed: RBF with the un-squared distance",
     "kernel_block", lambda: _mutated(O.kernel_block, "return s * np.exp(-0.5 * rho2)",
                                       "return s * np.exp(-0.5 * np.sqrt(rho2))"),
     pins.test_rbf_closed_form_values, ()),
    ("Matern-5/2 with the quadratic term's 5/3 dropped",
     "kernel_block", lambda: _mutated(O.kernel_block, "(5.0 / 3.0) * rho2", "rho2"),
     pins.test_matern52_closed_form_values, ()),
    ("lengthscale derivative divided by l^2 instead of l^3",
     "kernel_derivative_blocks", lambda: _mutated(O.kernel_derivative_blocks, "/ l[q] ** 3", "/ l[q] ** 2"),
     pins.test_kernel_derivative_blocks_match_finite_differences, (O.MATERN52, True)),
    ("NLML without its factor 1/2",
     "nlml_from_terms", lambda: _mutated(O.nlml_from_terms, "return 0.5 * (", "return ("),
     pins.test_gradient_sign_and_scale_by_finite_differences_of_cholesky_nlml, (O.RBF, False)),
    ("pivot ties broken towards the HIGHEST index",
     "pivoted_cholesky", lambda: _mutated(O.pivoted_cholesky, "best = int(np.argmax(masked))",
                                           "best = int(len(masked) - 1 - np.argmax(masked[::-1]))"),
     pins.test_pivoted_cholesky_ties_pick_lowest_index_and_forced_order_replays, ()),
    ("pivoted Cholesky column without the earlier columns subtracted",
     "pivoted_cholesky", lambda: _mutated(O.pivoted_cholesky, "col = (row - L[:, :m] @ L[piv, :m]) / root", "col = row / root"),
     pins.test_pivoted_cholesky_full_rank_reconstructs_K, ()),
]


@pytest.mark.parametrize("what,attr,make,pin,args", CASES, ids=[c[0] for c in CASES])
def test_a_planted_mistake_fails_its_pin(monkeypatch, what, attr, make, pin, args):
    pin(*args)                                   # the oracle as it stands passes
    monkeypatch.setattr(O, attr, make())
    with pytest.raises((AssertionError, np.linalg.LinAlgError, FloatingPointError, ValueError)):
        with np.errstate(all="ignore"):
            pin(*args)


def test_preconditioner_solve_without_the_division_by_noise_fails_its_pin(monkeypatch):
    bad = _mutated_method(O.Preconditioner, "solve", "return (R - self.L @ q) / self.noise", "return R - self.L @ q")
    monkeypatch.setattr(O.Preconditioner, "solve", bad)
    with pytest.raises(AssertionError):
        pins.test_woodbury_and_determinant_lemma_against_dense()


# the same for the subset-of-regressors oracle (oracle/sgpr_oracle.py)
SGPR_CASES = [
    ("dQ without its third term  - K_XU Kinv dK_UU Kinv K_UX",
     "sor_derivative_matvec", lambda: _mutated(S.sor_derivative_matvec, "dKW[h] - dUU[h] @ AW", "dKW[h]", module=S),
     spins.test_dq_ds_is_q_over_s_and_matrix_free_products_match_dense, ()),
    ("dQ with the third term added instead of subtracted",
     "sor_derivative_matvec", lambda: _mutated(S.sor_derivative_matvec, "dKW[h] - dUU[h] @ AW", "dKW[h] + dUU[h] @ AW", module=S),
     spins.test_derivative_matvec_against_dense_and_sensitivity_bound_holds, ()),
    ("jitter forgotten in the outputscale derivative of K_UU",
     "sor_derivative_matvec", lambda: _mutated(S.sor_derivative_matvec, "dUU[-1] = dUU[-1] + jitter_rel * np.eye(m)",
                                               "dUU[-1] = dUU[-1]", module=S),
     spins.test_dq_ds_is_q_over_s_and_matrix_free_products_match_dense, ()),
    ("dense dQ with the third term added instead of subtracted",
     "sor_khat_derivatives", lambda: _mutated(S.sor_khat_derivatives, "first + first.T - A.T @ duu @ A",
                                              "first + first.T + A.T @ duu @ A", module=S),
     spins.test_sor_gradient_by_finite_differences_of_the_dense_nlml, (O.RBF, False)),
    ("dense dQ with only one of the two cross terms",
     "sor_khat_derivatives", lambda: _mutated(S.sor_khat_derivatives, "first + first.T - A.T @ duu @ A",
                                              "first - A.T @ duu @ A", module=S),
     spins.test_sor_gradient_by_finite_differences_of_the_dense_nlml, (O.MATERN52, True)),
    ("Woodbury log-determinant with n log sigma^2 instead of (n - m) log sigma^2",
     "sor_woodbury", lambda: _mutated(S.sor_woodbury, "(n - m) * np.log(parts.noise)", "n * np.log(parts.noise)", module=S),
     spins.test_woodbury_solve_and_logdet_against_dense_cholesky, ()),
    ("Woodbury solve without the division by sigma^2",
     "sor_woodbury", lambda: _mutated(S.sor_woodbury, "parts.KXU.T @ y)) / parts.noise", "parts.KXU.T @ y))", module=S),
     spins.test_woodbury_solve_and_logdet_against_dense_cholesky, ()),
]


@pytest.mark.parametrize("what,attr,make,pin,args", SGPR_CASES, ids=[c[0] for c in SGPR_CASES])
def test_a_planted_mistake_in_the_sor_oracle_fails_its_pin(monkeypatch, what, attr, make, pin, args):
    pin(*args)
    monkeypatch.setattr(S, attr, make())
    with pytest.raises((AssertionError, np.linalg.LinAlgError, FloatingPointError, ValueError)):
        with np.errstate(all="ignore"):
            pin(*args)
