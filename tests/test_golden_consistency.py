"""The stored oracle results under tests/golden/ against the oracle as it stands (CPU only).

The files are written by tests/golden/make_golden.py in runs that take minutes to an hour, so they
can be older than the oracle's code.  Everything in them that can be recomputed in seconds is
recomputed here from the stored coefficients: the Lanczos tridiagonals from alpha / beta (App. A,
Observation), e_1^T log(T) e_1 (App. B), the log-det estimate (Eq. (5),(7)) and the NLML; and the
stored solve blocks are checked against the stored samples and norms."""
import glob
import json
import os

import numpy as np
import pytest

from oracle import bbmm_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
FILES = sorted(glob.glob(os.path.join(GOLDEN, "*.json")))


def _name(path):
    return os.path.splitext(os.path.basename(path))[0]


@pytest.mark.parametrize("path", FILES, ids=[_name(p) for p in FILES])
def test_stored_slq_terms_follow_from_the_stored_coefficients(path):
    g = json.load(open(path))
    if "slq_terms" not in g:
        pytest.skip("coefficients only (no log-det stored)")
    alpha, beta, rho0 = np.array(g["alpha"]), np.array(g["beta"]), np.array(g["rho0"])
    it = g["iters_run"]
    assert alpha.shape[0] == it
    m_valid = g.get("m_valid", [it] * alpha.shape[1])
    terms = []
    for i in range(g["t"]):
        dg, off = O.tridiag_from_cg(alpha[:, i + 1], beta[:, i + 1], int(m_valid[i + 1]))
        terms.append(rho0[i + 1] * O.e1_logT_e1(dg, off))
    assert np.allclose(terms, g["slq_terms"], rtol=1e-9, atol=1e-9 * np.abs(g["slq_terms"]).max())
    assert g["logdet"] == pytest.approx(g["logdet_precond"] + np.mean(terms), rel=1e-10)
    assert g["nlml"] == pytest.approx(O.nlml_from_terms(g["yKinvy"], g["logdet"], g["n"]), rel=1e-12)
    assert np.allclose(g["grad"], 0.5 * (np.array(g["trace"]) - np.array(g["quad"])), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("path", FILES, ids=[_name(p) for p in FILES])
def test_stored_solve_blocks_match_the_stored_samples(path):
    g = json.load(open(path))
    upath = os.path.join(GOLDEN, _name(path) + "_U.npy")
    if not os.path.exists(upath):
        pytest.skip("no stored solve block for this case")
    U = np.load(upath)
    every = int(g.get("U_rows_every", 1))
    assert U.dtype == np.float32 and U.shape == (-(-g["n"] // every), g["t"] + 1)
    rows, Us = np.array(g["sample_rows"]), np.array(g["U_sample"])
    keep = rows % every == 0
    assert np.allclose(U[rows[keep] // every], Us[keep], rtol=2e-7, atol=1e-30)
    if every == 1:
        assert np.allclose(np.linalg.norm(U.astype(np.float64), axis=0), g["U_colnorm"], rtol=1e-6)
    else:
        u0 = np.load(os.path.join(GOLDEN, _name(path) + "_u0.npy"))
        assert u0.shape == (g["n"],)
        assert np.allclose(u0[rows], Us[:, 0], rtol=2e-7, atol=1e-30)
        assert np.linalg.norm(u0.astype(np.float64)) == pytest.approx(g["U_colnorm"][0], rel=1e-6)


@pytest.mark.parametrize("path", FILES, ids=[_name(p) for p in FILES])
def test_stored_measures_of_definedness_are_consistent(path):
    g = json.load(open(path))
    if "U_last_step" not in g:
        pytest.skip("early-iteration case")
    c = g["t"] + 1
    for key in ("U_last_step", "U_reorder_dev", "U_fp32_dev"):
        assert len(g[key]) == c and np.all(np.array(g[key]) >= 0)
    if "_cap" in _name(path) and g["tol"] <= 0:
        # a converged-cap case: the last update and both perturbed fp64 runs far inside 1e-3
        assert max(g["U_last_step"]) < 1e-4
        assert max(max(g["U_reorder_dev"]), max(g["U_fp32_dev"])) < 2.5e-4
