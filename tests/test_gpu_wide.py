"""Inputs of more than 31 dimensions (the paper's UCI sets reach d = 385, Table 1 / dataset list): the fused
multiply, the rectangular multiply, the preconditioner, the solver and prediction against the fp64 oracle."""
import numpy as np
import pytest

import oracle as orc
from workloads import rademacher

pytestmark = pytest.mark.gpu

KMM_TOL = 1e-4


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
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _rel(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def _inputs(seed, n, d, t):
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    # lengthscales of the order sqrt(d): kernel values stay away from 0 and 1
    ls = (np.sqrt(d) * np.exp(rng.uniform(np.log(0.4), np.log(1.5), d))).astype(np.float32)
    return X, V, ls


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,t", [(300, 32, 16), (1000, 77, 17), (2049, 90, 16), (700, 160, 33), (1200, 385, 16),
                                   (513, 399, 5), (40, 35, 1), (3000, 164, 32),
                                   (2047, 159, 18), (1500, 135, 33), (1025, 140, 16)])
def test_kmm_wide_shapes(egp, kind, n, d, t):
    X, V, ls = _inputs(7000 * kind + 10 * d + t, n, d, t)
    s, noise = 1.3, 0.2
    import torch
    out = egp.kmm(_cuda(X), _cuda(V), ls, s, noise, kind)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = orc.kmm(X, V, orc.Hyper(kind, ls, s, noise))
    assert np.isfinite(got).all()
    err = _rel(got, ref)
    print(f"wide kmm n={n} d={d} t={t} kind={kind}: rel err {err:.2e}")
    assert err <= KMM_TOL


def test_kmm_wide_every_mode_runs_fp32(egp):
    """Modes 1 and 2 cover d <= 31; beyond that every mode takes the fp32 path and gives identical bits."""
    X, V, ls = _inputs(5, 900, 64, 16)
    base = egp.kmm(_cuda(X), _cuda(V), ls, 1.0, 0.1, orc.RBF).cpu().numpy()
    L = egp.lib()
    try:
        for mode in (1, 2):
            L.egp_set_kmm_mode(mode)
            got = egp.kmm(_cuda(X), _cuda(V), ls, 1.0, 0.1, orc.RBF).cpu().numpy()
            assert np.array_equal(got, base)
    finally:
        L.egp_set_kmm_mode(0)


@pytest.mark.parametrize("nq,n,d,t", [(100, 1500, 90, 1), (700, 900, 385, 20)])
def test_kmm_cross_wide(egp, nq, n, d, t):
    X, V, ls = _inputs(11 + d, n, d, t)
    Xq = np.random.default_rng(d).uniform(-1, 1, (nq, d)).astype(np.float32)
    got = egp.kmm_cross(_cuda(Xq), _cuda(X), _cuda(V), ls, 0.9, orc.MATERN52).cpu().numpy().astype(np.float64)
    ref = orc.kernel_matrix(Xq, X, orc.Hyper(orc.MATERN52, ls, 0.9, 0.0)) @ V.astype(np.float64)
    assert _rel(got, ref) <= KMM_TOL


def test_materialised_gradient_rejects_wide(egp):
    X, V, ls = _inputs(1, 100, 40, 2)
    with pytest.raises(egp.EgpError):
        egp.kmm_grad(_cuda(X), _cuda(V), ls, 1.0, 0.1, orc.RBF)


GRAD_TOL = 1e-4


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,t", [(600, 32, 17), (1000, 77, 17), (900, 90, 5), (500, 164, 16), (400, 200, 33),
                                   (300, 385, 17), (200, 399, 3), (40, 47, 1)])
def test_bilinear_forms_wide(egp, kind, n, d, t):
    """sum_c w_c a_c^T (dK/dl_k) b_c for every lengthscale and the outputscale form, d > 31 (expanded squared
    difference contracted on the MFMA), against the dense oracle; same Cauchy-Schwarz bound as for d <= 31."""
    X, _, ls = _inputs(900 * kind + d + t, n, d, t)
    rng = np.random.default_rng(n + d)
    A = rng.standard_normal((n, t)).astype(np.float32)
    B = rng.standard_normal((n, t)).astype(np.float32)
    wts = rng.uniform(-1, 1, t).astype(np.float32)
    s, noise = 1.3, 0.1
    h = orc.Hyper(kind, ls, s, noise)
    got = egp.kmm_grad_bilinear(_cuda(X), _cuda(A), _cuda(B), ls, s, noise, kind, weights=wts)
    Aw = A.astype(np.float64) * wts.astype(np.float64)
    worst = 0.0
    # every lengthscale up to d = 64; beyond that the first, the last and a seeded sample (oracle time)
    ks = range(d) if d <= 64 else sorted({0, d - 1, *rng.choice(d, 14, replace=False).tolist()})
    for k in ks:
        dKB = orc.dkernel_dlengthscale(X, X, h, k) @ B.astype(np.float64)
        ref = np.sum(Aw * dKB)
        bound = GRAD_TOL * np.linalg.norm(Aw) * np.linalg.norm(dKB)
        worst = max(worst, abs(got[k] - ref) / bound)
        assert abs(got[k] - ref) <= bound + 1e-12, (k, got[k], ref, bound)
    KB = orc.kernel_matrix(X, X, h) @ B.astype(np.float64) / s
    ref = np.sum(Aw * KB)
    assert abs(got[d] - ref) <= GRAD_TOL * np.linalg.norm(Aw) * np.linalg.norm(KB) + 1e-12
    print(f"wide bilinear n={n} d={d} t={t} kind={kind}: worst error / bound = {worst:.3f}")


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN52])
@pytest.mark.parametrize("rank", [0, 10])
def test_mll_wide_matches_oracle_with_same_probes(egp, kind, rank):
    """Marginal likelihood and gradient at d = 40: same probe draws on both sides."""
    rng = np.random.default_rng(140 + kind + rank)
    n, d, tp = 900, 40, 16
    X, _, ls = _inputs(55, n, d, 1)
    y = (np.sin(X[:, :5].sum(axis=1)) + 0.2 * rng.standard_normal(n)).astype(np.float32)
    s, noise = 1.2, 0.15
    h = orc.Hyper(kind, ls, s, noise)
    w1 = rademacher(rng, (max(rank, 1), tp))
    w2 = rademacher(rng, (n, tp))
    got = egp.mll(_cuda(X), _cuda(y), _cuda(w1), _cuda(w2), ls, s, noise, kind, rank=rank, max_iter=400, tol=1e-5)
    assert got["rel_resid_max"] <= 1e-5 and got["rank"] == rank
    if rank:
        L, piv = orc.pivoted_cholesky(orc.kernel_matrix(X, X, h), rank)
        assert egp.piv_chol_precond(_cuda(X), ls, s, noise, kind, rank).pivots.tolist() == piv.tolist()
        Z = orc.probes_with_cov_P(L, noise, w1, w2)
    else:
        L, Z = None, w2.astype(np.float64)
    ref = orc.mll_stochastic_terms(X, y, h, Z, L)
    assert abs(got["mll"] - ref["mll"]) <= 2e-3 * abs(ref["mll"]) + 0.05
    scale = np.abs(ref["grad"]) + 0.02 * np.abs(ref["grad"]).max()
    assert np.all(np.abs(got["grad"] - ref["grad"]) <= 2e-2 * scale), (got["grad"], ref["grad"])


@pytest.mark.parametrize("d", [77, 385])
def test_solver_and_prediction_wide(egp, d):
    """Preconditioned solve to convergence against a dense Cholesky solve; predictive mean and cached variance."""
    n, t, rank = 1200, 5, 20
    X, _, ls = _inputs(300 + d, n, d, t)
    rng = np.random.default_rng(d)
    y = np.sin(X[:, :4].sum(axis=1)) + 0.1 * rng.standard_normal(n)
    B = np.concatenate([y[:, None], rademacher(rng, (n, t - 1))], axis=1).astype(np.float32)
    s, noise, kind = 1.0, 0.05, orc.RBF
    h = orc.Hyper(kind, ls, s, noise)
    Khat = orc.khat(X, h)
    Lref, pref = orc.pivoted_cholesky(orc.kernel_matrix(X, X, h), rank)
    P = egp.piv_chol_precond(_cuda(X), ls, s, noise, kind, rank)
    # compare what is unique: the approximation L L^T (pivot ties between near-equal diagonals may differ)
    Lg = P.L.cpu().numpy().astype(np.float64).T
    if P.pivots.tolist() == pref.tolist():
        assert np.abs(Lg - Lref).max() <= 5e-4
    res_g = np.trace(Khat - noise * np.eye(n) - Lg @ Lg.T)
    res_o = np.trace(Khat - noise * np.eye(n) - Lref @ Lref.T)
    assert abs(res_g - res_o) <= 1e-3 * abs(res_o)
    sol = egp.mbcg(_cuda(X), _cuda(B), ls, s, noise, kind, precond=P, max_iter=300, tol=1e-5)
    U = sol["U"].cpu().numpy().astype(np.float64)
    Uref = orc.chol_solve(Khat, B.astype(np.float64))
    assert _rel(U, Uref) <= 2e-3
    # prediction
    nq = 64
    Xq = rng.uniform(-1, 1, (nq, d)).astype(np.float32)
    a = Uref[:, 0].astype(np.float32)
    cache = egp.lanczos(_cuda(X), _cuda(y.astype(np.float32)), ls, s, noise, kind, 24)
    mean, var = egp.predict(_cuda(Xq), _cuda(X), _cuda(a), ls, s, noise, kind, cache=cache)
    mref, vref = orc.predict_exact(X, y, Xq, h)
    assert np.abs(mean.cpu().numpy() - mref).max() <= 2e-3 * max(1.0, np.abs(mref).max())
    Qo, ao, bo = orc.lanczos(Khat, y.astype(np.float64), 24)
    vlan = orc.predict_var_lanczos(orc.kernel_matrix(Xq, X, h), Qo, ao, bo, s)
    vg = var.cpu().numpy().astype(np.float64)
    assert np.abs(vg - vlan).max() <= 2e-3
    assert (vg >= vref - 2e-3).all()


@pytest.mark.parametrize("n,d,t,kind", [(32768, 40, 16, orc.RBF), (33000, 90, 16, orc.MATERN32), (34000, 164, 16, orc.RBF),
                                         (33000, 300, 32, orc.MATERN52), (33281, 77, 16, orc.MATERN12),
                                         (33000, 90, 17, orc.RBF), (32768, 36, 17, orc.MATERN52), (33000, 200, 33, orc.MATERN32)])
def test_kmm_wide_symmetric_kernel_rows(egp, n, d, t, kind):
    """The symmetric fp32 mode beyond d = 31 (groups of 16 or 17 columns; wider groups fall back): rows computed
    exactly by the oracle, both row-tile shapes, every stage size, even and odd block counts; and every row against
    the one-sided kernel."""
    X, V, ls = _inputs(31 * d + t + kind, n, d, t)
    rng = np.random.default_rng(d)
    rows = rng.choice(n, 96, replace=False)
    edges = [0, 15, 16, 63, 64, 127, 128, n // 2 - 1, n // 2, n // 2 + 64, n - 129, n - 128, n - 1]
    rows[:len(edges)] = edges
    rows = np.unique(rows)
    ref = orc.kmm_rows(X, V, orc.Hyper(kind, ls, 1.1, 0.3), rows)
    Xd, Vd = _cuda(X), _cuda(V)
    got = egp.kmm(Xd, Vd, ls, 1.1, 0.3, kind).cpu().numpy().astype(np.float64)
    again = egp.kmm(Xd, Vd, ls, 1.1, 0.3, kind).cpu().numpy().astype(np.float64)
    assert np.array_equal(got, again)      # order-independent column-side sums
    L = egp.lib()
    try:
        L.egp_set_kmm_mode(3)      # every tile formed, no use of the symmetry
        base = egp.kmm(Xd, Vd, ls, 1.1, 0.3, kind).cpu().numpy().astype(np.float64)
    finally:
        L.egp_set_kmm_mode(0)
    assert np.isfinite(got).all()
    err = _rel(got[rows], ref)
    print(f"wide symmetric n={n} d={d} t={t} kind={kind}: rel err {err:.2e}; vs one-sided {_rel(got, base):.2e}")
    assert err <= KMM_TOL
    assert _rel(got, base) <= 2e-5


def test_kmm_wide_one_sided_on_other_shapes(egp):
    """d = 385 does not fit the symmetric wide kernel's LDS budget; 32 columns are not built for it: the default mode
    runs the one-sided kernel there (same bits as with the symmetry switched off)."""
    for d, t in ((385, 16), (90, 32)):
        X, V, ls = _inputs(d + t, 33000, d, t)
        Xd, Vd = _cuda(X), _cuda(V)
        base = egp.kmm(Xd, Vd, ls, 1.0, 0.1, orc.RBF).cpu().numpy()
        L = egp.lib()
        try:
            L.egp_set_kmm_mode(3)
            got = egp.kmm(Xd, Vd, ls, 1.0, 0.1, orc.RBF).cpu().numpy()
        finally:
            L.egp_set_kmm_mode(0)
        assert np.array_equal(got, base)


@pytest.mark.parametrize("t", [16, 17])
def test_mbcg_wide_with_symmetric_kernels(egp, t):
    """Solver at d = 90 with 16 / 17 right-hand sides: the symmetric wide kernel (default mode at this size) with the
    column-major state arrays gives the one-sided kernel's iterates up to summation order."""
    n, d = 33000, 90
    X, B, ls = _inputs(901, n, d, t)
    s, noise, kind = 1.0, 0.5, orc.RBF
    Xd, Bd = _cuda(X), _cuda(B)
    res = egp.mbcg(Xd, Bd, ls, s, noise, kind, max_iter=12, tol=0.0)
    L = egp.lib()
    try:
        L.egp_set_kmm_mode(3)      # one-sided kernels
        base = egp.mbcg(Xd, Bd, ls, s, noise, kind, max_iter=12, tol=0.0)
    finally:
        L.egp_set_kmm_mode(0)
    assert np.allclose(res["alphas"][:3], base["alphas"][:3], rtol=1e-4)
    U = res["U"].cpu().numpy().astype(np.float64)
    Ub = base["U"].cpu().numpy().astype(np.float64)
    assert _rel(U, Ub) <= 1e-3
    rows = np.random.default_rng(3).choice(n, 64, replace=False)
    KU = orc.kmm_rows(X, U, orc.Hyper(kind, ls, s, noise), rows)
    true_res = np.linalg.norm(KU - B[rows], axis=0) / np.linalg.norm(B[rows], axis=0)
    assert true_res.max() <= max(3.0 * float(res["rel_resid"].max()), 1e-3)
