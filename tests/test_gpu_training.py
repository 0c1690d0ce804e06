"""End-to-end use of the stochastic NLML gradient (Sec. 2, Eq. (2)): Adam on the raw
hyperparameters must walk downhill on the EXACT negative log marginal likelihood, which the
fp64 oracle evaluates by dense Cholesky at the visited points."""
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


def _exact(w, ls, s, noise, traces=False):
    return O.exact_inference(w.kernel, w.X, w.y, np.atleast_1d(ls), s, noise, with_traces=traces)


@pytest.mark.parametrize("kernel,ard", [(inputs.RBF, False), (inputs.MATERN52, True)])
def test_adam_on_the_bbmm_gradient_descends_the_exact_nlml(ctx, kernel, ard):
    from paper_1809_11165_amd import training
    w = inputs.tiny(800, 3, kernel=kernel, ard=ard, t=10, k=5, iters=20, noise=0.05, seed=21)
    ls0 = np.atleast_1d(w.lengthscale) * 2.5          # start well away from a sensible fit
    s0, noise0 = 0.3 * w.outputscale, 8.0 * w.noise
    traj = training.fit(ctx, w.kernel, inputs.ONTHEFLY, w.X, w.y, ls0, s0, noise0, steps=40, lr=0.1,
                        t=10, k=5, iters=20, seed=1)
    start = _exact(w, ls0, s0, noise0, traces=True)
    end = _exact(w, traj.lengthscale[-1], traj.outputscale[-1], traj.noise[-1])
    mid = _exact(w, traj.lengthscale[20], traj.outputscale[20], traj.noise[20])
    assert mid.nlml < start.nlml and end.nlml < mid.nlml
    assert end.nlml < start.nlml - 0.05 * abs(start.nlml)
    # the very first stochastic gradient against the exact one (raw parameters): same signs on the
    # components that matter, and close in direction
    prob_grad = np.array(traj.grad_norm[0])
    assert np.isfinite(prob_grad)
    from paper_1809_11165_amd import binding
    dev = torch.device("cuda:0")
    rng = np.random.Generator(np.random.Philox(5))
    E1 = torch.from_numpy(inputs.rademacher(rng, (5, 10))).to(dev)
    E2 = torch.from_numpy(inputs.rademacher(rng, (w.n, 10))).to(dev)
    prob = binding.Problem(kernel=w.kernel, mode=inputs.ONTHEFLY, X=torch.from_numpy(w.X).to(dev),
                           y=torch.from_numpy(w.y).to(dev), lengthscale=ls0, outputscale=s0, noise=noise0,
                           E1=E1, E2=E2, k=5, max_iters=20, tol=0.0)
    res = ctx.bbmm_solve_logdet_grad(prob, want_U=False)
    g, ge = np.asarray(res.grad_nlml), start.grad
    cos = float(g @ ge / (np.linalg.norm(g) * np.linalg.norm(ge)))
    assert cos > 0.95, (g, ge)
    assert res.nlml == pytest.approx(start.nlml, rel=2e-2)
