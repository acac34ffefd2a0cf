"""Prediction path on the GPU: rectangular products, Lanczos cache, predictive mean and variance."""
import numpy as np
import pytest

import oracle as orc
from workloads import make_workload, rademacher, well_separated_points

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
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _rel(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("nq,n,d,t", [(1, 1, 1, 1), (7, 300, 3, 1), (1000, 777, 8, 16), (33, 2500, 11, 17),
                                      (600, 900, 18, 40), (2100, 50, 25, 33)])
def test_kmm_cross_matches_oracle(egp, kind, nq, n, d, t):
    rng = np.random.default_rng(nq + 3 * n + 5 * d + t + kind)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    Xq = rng.uniform(-1.2, 1.2, (nq, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.4), np.log(2.5), d)).astype(np.float32)
    h = orc.Hyper(kind, ls, 1.6, 0.0)
    got = egp.kmm_cross(_cuda(Xq), _cuda(X), _cuda(V), ls, 1.6, kind).cpu().numpy().astype(np.float64)
    ref = orc.kernel_matrix(Xq, X, h) @ V.astype(np.float64)
    assert got.shape == (nq, t)
    assert _rel(got, ref) <= KMM_TOL


def test_kmm_cross_equal_sizes_is_not_taken_for_symmetric(egp):
    """Two different point sets of the same (large) size are not a symmetric product: the default mode must leave
    such a call to the one-sided kernel. Checked against oracle rows and against the bits of the mode that never
    uses the symmetry."""
    nq = n = 33000
    d, t, kind = 11, 16, orc.RBF
    rng = np.random.default_rng(2024)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    Xq = rng.uniform(-1, 1, (nq, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.4), np.log(2.5), d)).astype(np.float32)
    got = egp.kmm_cross(_cuda(Xq), _cuda(X), _cuda(V), ls, 1.1, kind).cpu().numpy()
    try:
        egp.set_kmm_mode("fp32_one_sided")
        base = egp.kmm_cross(_cuda(Xq), _cuda(X), _cuda(V), ls, 1.1, kind).cpu().numpy()
    finally:
        egp.set_kmm_mode("fp32")
    assert np.array_equal(got, base)
    rows = rng.choice(nq, 64, replace=False)
    ref = orc.kernel_matrix(Xq[rows], X, orc.Hyper(kind, ls, 1.1, 0.0)) @ V.astype(np.float64)
    assert _rel(got[rows].astype(np.float64), ref) <= KMM_TOL


def test_lanczos_cache_properties_and_parity(egp):
    n, d, r = 700, 3, 40
    rng = np.random.default_rng(8)
    X = well_separated_points(31, n, d)
    y = (np.sin(5 * X[:, 0]) + X[:, 1] ** 2 + 0.1 * rng.standard_normal(n)).astype(np.float32)
    ls = np.array([0.3, 0.5, 0.9], np.float32)
    s, noise, kind = 1.3, 0.1, orc.MATERN52
    h = orc.Hyper(kind, ls, s, noise)
    c = egp.lanczos(_cuda(X), _cuda(y), ls, s, noise, kind, r)
    assert c.steps == r
    Q = c.Q.cpu().numpy().astype(np.float64)
    assert np.abs(Q @ Q.T - np.eye(r)).max() <= 5e-5          # full re-orthogonalisation holds in fp32
    Kh = orc.khat(X, h)
    T = Q @ Kh @ Q.T
    scale = np.abs(np.diag(T)).max()
    assert np.abs(np.diag(T) - c.alpha).max() <= 1e-4 * scale
    assert np.abs(np.diag(T, 1) - c.beta).max() <= 1e-4 * scale
    assert np.abs(np.triu(T, 2)).max() <= 2e-4 * scale
    # against the oracle's Lanczos: the early coefficients agree tightly (later ones drift with rounding)
    Qr, ar, br = orc.lanczos(Kh, y, r)
    assert np.allclose(c.alpha[:8], ar[:8], rtol=2e-4)
    assert np.allclose(c.beta[:8], br[:8], rtol=2e-4)
    assert np.abs(np.abs(Q[:4] @ Qr[:4].T) - np.eye(4)).max() <= 1e-3


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32])
def test_predict_mean_and_cached_variance(egp, kind):
    n, nq, d = 900, 257, 2
    rng = np.random.default_rng(11 + kind)
    X = well_separated_points(5, n, d)
    Xq = rng.uniform(0, 1, (nq, d)).astype(np.float32)
    y = (np.sin(6 * X[:, 0]) * np.cos(4 * X[:, 1]) + 0.1 * rng.standard_normal(n)).astype(np.float32)
    ls = np.array([0.25, 0.35], np.float32)
    s, noise = 1.2, 0.05
    h = orc.Hyper(kind, ls, s, noise)
    Xd, yd = _cuda(X), _cuda(y[:, None])
    sol = egp.mbcg(Xd, yd, ls, s, noise, kind, precond=egp.piv_chol_precond(Xd, ls, s, noise, kind, 30),
                   max_iter=500, tol=1e-5)             # tight tolerance for the one-time cache (paper: eps <= 0.01)
    a = sol["U"][:, 0].contiguous()
    mean_ref, var_ref = orc.predict_exact(X, y, Xq, h)
    mean, _ = egp.predict(_cuda(Xq), Xd, a, ls, s, noise, kind)
    assert _rel(mean.cpu().numpy().astype(np.float64), mean_ref) <= 2e-3
    # cached variance at two ranks: parity with the oracle's Lanczos variance, never below exact, improves with r
    Kh = orc.khat(X, h)
    Kq = orc.kernel_matrix(Xq, X, h)
    prev = None
    for r in (20, 120):
        cache = egp.lanczos(Xd, _cuda(y), ls, s, noise, kind, r)
        _, var = egp.predict(_cuda(Xq), Xd, a, ls, s, noise, kind, cache=cache)
        var = var.cpu().numpy().astype(np.float64)
        Qr, ar, br = orc.lanczos(Kh, y, r)
        vr = orc.predict_var_lanczos(Kq, Qr, ar, br, s)
        assert np.abs(var - vr).max() <= 5e-3 * s
        assert np.all(var >= var_ref - 5e-3 * s)
        if prev is not None:
            assert np.mean(var) < np.mean(prev)
        prev = var


def test_predict_c4_recipe_timing_shape(egp):
    """1000 query points against 2^17 training points of the C4 recipe: sampled parity of the mean."""
    w = make_workload("C4", n=131072, with_targets=False)
    rng = np.random.default_rng(1)
    Xq = w.X[rng.choice(w.n, 1000, replace=False)] + 0.01 * rng.standard_normal((1000, w.d)).astype(np.float32)
    a = rng.standard_normal(w.n).astype(np.float32)
    mean, _ = egp.predict(_cuda(Xq), _cuda(w.X), _cuda(a), w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, 0.0)
    ref = orc.kernel_matrix(Xq[:64], w.X, h) @ a.astype(np.float64)
    assert _rel(mean.cpu().numpy()[:64].astype(np.float64), ref) <= KMM_TOL


@pytest.mark.parametrize("kind,b,blocks", [(orc.RBF, 16, 6), (orc.MATERN32, 4, 20), (orc.MATERN52, 32, 3), (orc.RBF, 1, 25)])
def test_block_lanczos_cache(egp, kind, b, blocks):
    """Block Krylov variance cache against the oracle's block process from the same start block: orthonormal Q,
    T = Q Khat Q^T, and the subspace-invariant quantity — the cached variance — equal to the oracle's; never below
    the exact variance; with b = 1 it coincides with the single-vector cache."""
    n, nq, d = 900, 200, 2
    rng = np.random.default_rng(31 + kind + b)
    X = well_separated_points(6, n, d)
    Xq = rng.uniform(0, 1, (nq, d)).astype(np.float32)
    y = (np.sin(6 * X[:, 0]) * np.cos(4 * X[:, 1]) + 0.1 * rng.standard_normal(n)).astype(np.float32)
    ls = np.array([0.25, 0.35], np.float32)
    s, noise = 1.2, 0.05
    h = orc.Hyper(kind, ls, s, noise)
    B0 = np.concatenate([y[:, None], rademacher(rng, (n, b - 1))], axis=1) if b > 1 else y[:, None].copy()
    Xd = _cuda(X)
    cache = egp.block_lanczos(Xd, _cuda(B0), ls, s, noise, kind, blocks)
    assert cache.steps == b * blocks
    Kh = orc.khat(X, h)
    Kq = orc.kernel_matrix(Xq, X, h)
    Q = cache.Q.cpu().numpy().astype(np.float64)
    assert np.abs(Q @ Q.T - np.eye(cache.steps)).max() <= 5e-5
    Tq = Q @ Kh @ Q.T
    assert np.abs(cache.T - Tq).max() <= 2e-4 * np.abs(Tq).max()
    assert np.allclose(cache.T, cache.T.T)
    Qo, To = orc.block_lanczos(Kh, B0.astype(np.float64), blocks)
    assert Qo.shape[0] == cache.steps
    # the first two blocks span the same space on both sides; later Krylov blocks are ill-conditioned functions of
    # the start block (fp32 storage on one side, fp64 on the other), so from there on only what the subspaces are
    # used for is compared: the variances
    k2 = min(2 * b, cache.steps)
    assert np.abs(Qo[:k2] - (Qo[:k2] @ Q[:k2].T) @ Q[:k2]).max() <= 2e-3
    a = _cuda(orc.chol_solve(Kh, y.astype(np.float64)).astype(np.float32))
    _, var = egp.predict(_cuda(Xq), Xd, a, ls, s, noise, kind, cache=cache)
    var = var.cpu().numpy().astype(np.float64)
    vo = orc.predict_var_galerkin(Kq, Qo, To, s)
    _, exact = orc.predict_exact(X, y, Xq, h)
    assert np.abs(var - vo).max() <= 5e-3 * s
    assert np.all(var >= exact - 5e-3 * s)
    if b == 1:
        single = egp.lanczos(Xd, _cuda(y), ls, s, noise, kind, blocks)
        _, v1 = egp.predict(_cuda(Xq), Xd, a, ls, s, noise, kind, cache=single)
        assert np.abs(var - v1.cpu().numpy()).max() <= 2e-3 * s


def test_block_lanczos_stops_at_an_invariant_subspace_and_rejects_bad_blocks(egp):
    n, d = 64, 1
    X = np.linspace(0, 1, n, dtype=np.float32)[:, None]
    rng = np.random.default_rng(2)
    B0 = rademacher(rng, (n, 16))
    cache = egp.block_lanczos(_cuda(X), _cuda(B0), [0.3], 1.0, 0.1, orc.MATERN32, 4)      # 4 * 16 = n
    assert cache.steps == 64
    bad = B0.copy()
    bad[:, 3] = bad[:, 1]                                                                 # rank-deficient start block
    with pytest.raises(egp.EgpError):
        egp.block_lanczos(_cuda(X), _cuda(bad), [0.3], 1.0, 0.1, orc.MATERN32, 2)
    with pytest.raises(egp.EgpError):
        egp.block_lanczos(_cuda(X), _cuda(B0), [0.3], 1.0, 0.1, orc.MATERN32, 5)          # b * blocks > n
