"""The assembled marginal-likelihood step (value + gradient) against the dense oracle."""
import numpy as np
import pytest

import oracle as orc
from workloads import rademacher, well_separated_points

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def egp():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1903_08114_amd as egp
    egp.lib()
    return egp


def _cuda(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("rank", [0, 12])
def test_mll_matches_oracle_with_same_probes(egp, kind, rank):
    """Same Rademacher draws on both sides: the two stochastic estimates must agree up to fp32 effects,
    and both must sit within Monte-Carlo error of the exact dense value."""
    rng = np.random.default_rng(40 + kind + rank)
    n, d, tp = 1200, 3, 16
    X = well_separated_points(77, n, d)
    y = (np.sin(5 * X[:, 0]) + np.cos(3 * X[:, 1]) + 0.2 * rng.standard_normal(n)).astype(np.float32)
    ls = np.array([0.6, 0.9, 1.4], np.float32)   # successive pivot maxima >= 6e-4 apart (relative)
    s, noise = 1.2, 0.15
    h = orc.Hyper(kind, ls, s, noise)
    w1 = rademacher(rng, (max(rank, 1), tp))
    w2 = rademacher(rng, (n, tp))
    got = egp.mll(_cuda(X), _cuda(y), _cuda(w1), _cuda(w2), ls, s, noise, kind, rank=rank, max_iter=400, tol=1e-5)
    assert got["rel_resid_max"] <= 1e-5 and got["rank"] == rank
    if rank:
        L, piv = orc.pivoted_cholesky(orc.kernel_matrix(X, X, h), rank)
        # both sides must build the same P, or the probe vectors (hence the estimates) differ
        assert egp.piv_chol_precond(_cuda(X), ls, s, noise, kind, rank).pivots.tolist() == piv.tolist()
        Z = orc.probes_with_cov_P(L, noise, w1, w2)
    else:
        L, Z = None, w2.astype(np.float64)
    ref = orc.mll_stochastic_terms(X, y, h, Z, L)
    # same estimator, same draws
    assert abs(got["quad"] - y.astype(np.float64) @ ref["u"]) <= 1e-3 * abs(y.astype(np.float64) @ ref["u"])
    assert abs(got["logdet"] - ref["logdet"]) <= 2e-3 * abs(ref["logdet"]) + 0.05
    assert abs(got["mll"] - ref["mll"]) <= 2e-3 * abs(ref["mll"]) + 0.05
    scale = np.abs(ref["grad"]) + 0.02 * np.abs(ref["grad"]).max()
    assert np.all(np.abs(got["grad"] - ref["grad"]) <= 2e-2 * scale), (got["grad"], ref["grad"])
    # and the exact values (dense Cholesky), within a generous Monte-Carlo band
    # (Matern-1/2 decays slowest in the spectrum, so more eigenvalues sit away from the noise level and the 16-probe
    # log-determinant estimate scatters about twice as much: band doubled)
    exact = orc.mll(X, y, h)
    band = 2.0 if kind == orc.MATERN12 else 1.0
    assert abs(got["mll"] - exact) <= band * (0.02 * abs(exact) + 2.0)
    gexact = orc.mll_grad(X, y, h)
    assert np.all(np.abs(got["grad"] - gexact) <= band * (0.25 * np.abs(gexact) + 0.1 * np.abs(gexact).max()))


def test_train_adam_tracks_the_oracle_loop(egp):
    """Three Adam steps with the same probe draws on both sides: parameter trajectories and objective values
    agree up to fp32 effects; the noise floor holds."""
    rng = np.random.default_rng(77)
    n, d, tp, rank = 900, 2, 16, 10
    X = well_separated_points(13, n, d)
    y = (np.sin(5 * X[:, 0]) + np.cos(3 * X[:, 1]) + 0.2 * rng.standard_normal(n)).astype(np.float32)
    ls0, s0, noise0, floor = np.array([0.9, 1.3], np.float32), 0.8, 0.4, 0.1
    kind = orc.RBF
    w1 = rademacher(rng, (rank, tp))
    w2 = rademacher(rng, (n, tp))
    got = egp.train_adam(_cuda(X), _cuda(y), _cuda(w1), _cuda(w2), ls0, s0, noise0, kind, rank=rank, max_iter=400,
                         tol=1e-5, steps=3, lr=0.1, noise_floor=floor)
    href, hist = orc.train_adam(X, y, orc.Hyper(kind, ls0, s0, noise0), steps=3, lr=0.1, noise_floor=floor,
                                rank=rank, W1=w1, W2=w2)
    assert np.allclose(got["lengthscales"], href.lengthscales, rtol=2e-2)
    assert abs(got["outputscale"] - href.outputscale) <= 2e-2 * href.outputscale
    assert abs(got["noise"] - href.noise) <= 2e-2 * href.noise and got["noise"] > floor
    assert np.allclose(got["mll_history"], hist, rtol=3e-3, atol=0.5)
    assert got["mll_history"][-1] > got["mll_history"][0]


@pytest.mark.parametrize("kind,tp", [(orc.MATERN32, 16), (orc.RBF, 15), (orc.RBF, 32)])
def test_mll_with_symmetric_kernels_matches_one_sided(egp, kind, tp):
    """At a size where the default mode runs the symmetric kernels (17, 16 and 33 columns in the solver), the
    likelihood step gives the one-sided kernels' value and gradient up to summation order and the stopping point of
    the solver: same probes, same preconditioner. The one-sided kernels are the ones checked against the dense oracle
    above; n = 33000 is out of reach of a dense factorisation."""
    n, d, rank = 33000, 11, 30
    rng = np.random.default_rng(900 + kind + tp)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    y = (np.sin(5 * X[:, 0]) + np.cos(3 * X[:, 1]) + 0.2 * rng.standard_normal(n)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.3), np.log(1.5), d)).astype(np.float32)
    s, noise = 1.1, 0.5
    w1, w2 = _cuda(rademacher(rng, (rank, tp))), _cuda(rademacher(rng, (n, tp)))
    Xd, yd = _cuda(X), _cuda(y)
    got = egp.mll(Xd, yd, w1, w2, ls, s, noise, kind, rank=rank, max_iter=300, tol=1e-3)
    try:
        egp.set_kmm_mode("fp32_one_sided")
        base = egp.mll(Xd, yd, w1, w2, ls, s, noise, kind, rank=rank, max_iter=300, tol=1e-3)
    finally:
        egp.set_kmm_mode("fp32")
    print(f"mll at n={n} kind={kind} tp={tp}: one-sided {base['mll']:.3f} ({base['iters']} it), default {got['mll']:.3f} "
          f"({got['iters']} it)")
    assert got["rel_resid_max"] <= 1e-3 and base["rel_resid_max"] <= 1e-3
    assert abs(got["iters"] - base["iters"]) <= 2
    assert abs(got["quad"] - base["quad"]) <= 2e-3 * abs(base["quad"])
    assert abs(got["logdet"] - base["logdet"]) <= 1e-3 * abs(base["logdet"]) + 0.5
    assert abs(got["mll"] - base["mll"]) <= 1e-3 * abs(base["mll"]) + 0.5
    scale = np.abs(base["grad"]) + 0.02 * np.abs(base["grad"]).max()
    assert np.all(np.abs(got["grad"] - base["grad"]) <= 2e-2 * scale), (got["grad"], base["grad"])


def test_mll_with_column_shrinking(egp):
    """With the shrink switch the probe columns leave the solve once they meet the tolerance, so their Lanczos
    tridiagonals are shorter. At a tight tolerance the estimate is the one without the switch (every column is
    converged either way) and stays inside the Monte-Carlo band of the exact value; at a loose tolerance it remains a
    usable estimate (the quadrature has fewer nodes, not wrong ones)."""
    rng = np.random.default_rng(71)
    n, d, tp, rank = 1200, 3, 16, 12
    X = well_separated_points(77, n, d)
    y = (np.sin(5 * X[:, 0]) + np.cos(3 * X[:, 1]) + 0.2 * rng.standard_normal(n)).astype(np.float32)
    ls = np.array([0.6, 0.9, 1.4], np.float32)
    s, noise, kind = 1.2, 0.15, orc.RBF
    h = orc.Hyper(kind, ls, s, noise)
    w1, w2 = _cuda(rademacher(rng, (rank, tp))), _cuda(rademacher(rng, (n, tp)))
    Xd, yd = _cuda(X), _cuda(y)
    exact = orc.mll(X, y, h)
    gexact = orc.mll_grad(X, y, h)
    for tol, band in ((1e-5, 1.0), (1e-1, 2.0)):
        off = egp.mll(Xd, yd, w1, w2, ls, s, noise, kind, rank=rank, max_iter=400, tol=tol)
        on = egp.mll(Xd, yd, w1, w2, ls, s, noise, kind, rank=rank, max_iter=400, tol=tol, shrink=True)
        assert egp.lib().egp_get_mbcg_shrink() == 0
        print(f"tol {tol}: mll {off['mll']:.3f} ({off['iters']} it) without, {on['mll']:.3f} ({on['iters']} it) with "
              f"shrinking; exact {exact:.3f}")
        assert on["rel_resid_max"] <= tol and on["iters"] <= off["iters"]
        assert abs(on["mll"] - exact) <= band * (0.02 * abs(exact) + 2.0)
        assert np.all(np.abs(on["grad"] - gexact) <= band * (0.25 * np.abs(gexact) + 0.1 * np.abs(gexact).max()))
        if tol < 1e-4:
            assert abs(on["mll"] - off["mll"]) <= 1e-3 * abs(off["mll"]) + 0.05
