"""Pins for the oracle's kernel matrix, KMM and derivative products (CPU only)."""
import math
import os

import numpy as np
import pytest

import oracle as orc
from workloads import make_workload, well_separated_points

KINDS = [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12]


def _scalar_kernel(x, z, ls, s, kind):
    """Brute force on python floats: written independently of the oracle's vectorised code."""
    r2 = 0.0
    for a, b, l in zip(x, z, ls):
        r2 += ((float(a) - float(b)) / float(l)) ** 2
    r = math.sqrt(r2)
    if kind == orc.RBF:
        return s * math.exp(-r2 / 2.0)
    if kind == orc.MATERN32:
        return s * (1.0 + math.sqrt(3.0) * r) * math.exp(-math.sqrt(3.0) * r)
    if kind == orc.MATERN12:
        return s * math.exp(-r)
    return s * (1.0 + math.sqrt(5.0) * r + 5.0 * r2 / 3.0) * math.exp(-math.sqrt(5.0) * r)


def test_closed_forms_at_unit_distance(golden_dir):
    rows = np.loadtxt(os.path.join(golden_dir, "kernel_closed_forms.txt"))
    for kind, g1, h1 in rows:
        h = orc.Hyper(int(kind), [1.0], 1.0, 0.0)
        K = orc.kernel_matrix([[0.0]], [[1.0]], h)
        assert abs(K[0, 0] - g1) < 1e-12
        dK = orc.dkernel_dlengthscale([[0.0]], [[1.0]], h, 0)
        assert abs(dK[0, 0] - h1) < 1e-9
        # k(x,x) = outputscale
        h2 = orc.Hyper(int(kind), [0.7, 1.3], 2.5, 0.0)
        assert abs(orc.kernel_matrix([[0.3, 0.1]], [[0.3, 0.1]], h2)[0, 0] - 2.5) < 1e-14


@pytest.mark.parametrize("kind", KINDS)
def test_brute_force_entries_and_product(kind):
    rng = np.random.default_rng(5)
    n, d, t = 23, 3, 4
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.array([0.4, 1.1, 2.0])
    h = orc.Hyper(kind, ls, 1.7, 0.3)
    Kh = orc.khat(X, h)
    expect = np.zeros((n, t))
    for i in range(n):
        for j in range(n):
            kij = _scalar_kernel(X[i], X[j], ls, 1.7, kind) + (0.3 if i == j else 0.0)
            assert abs(Kh[i, j] - kij) < 1e-13
            for c in range(t):
                expect[i, c] += kij * float(V[j, c])
    assert np.allclose(orc.kmm(X, V, h), expect, rtol=0, atol=1e-12)
    rows = [3, 0, 22, 7]
    assert np.allclose(orc.kmm_rows(X, V, h, rows), expect[rows], rtol=0, atol=1e-12)


@pytest.mark.parametrize("kind", KINDS)
def test_symmetric_and_psd(kind):
    w = make_workload("C1", n=300)
    h = orc.Hyper(kind, w.lengthscales, w.outputscale, w.noise)
    K = orc.kernel_matrix(w.X, w.X, h)
    assert np.array_equal(K, K.T)
    lam = np.linalg.eigvalsh(K)
    assert lam.min() >= -1e-10 * 300
    lam_hat = np.linalg.eigvalsh(orc.khat(w.X, h))
    assert lam_hat.min() >= w.noise - 1e-10 * 300


@pytest.mark.parametrize("kind", KINDS)
def test_lengthscale_limits_and_structure(kind):
    rng = np.random.default_rng(9)
    n, d, t = 40, 4, 3
    X = rng.uniform(0, 1, (n, d))
    V = rng.standard_normal((n, t))
    s, noise = 1.3, 0.2
    # l -> infinity: K -> s 1 1^T
    big = orc.Hyper(kind, np.full(d, 1e7), s, noise)
    expect = s * np.ones((n, 1)) * V.sum(axis=0, keepdims=True) + noise * V
    assert np.allclose(orc.kmm(X, V, big), expect, atol=1e-9)
    # l -> 0 with distinct points: K -> s I
    tiny = orc.Hyper(kind, np.full(d, 1e-7), s, noise)
    assert np.allclose(orc.kmm(X, V, tiny), (s + noise) * V, atol=1e-12)
    # identical points behave like l -> infinity
    same = np.tile(X[:1], (n, 1))
    h = orc.Hyper(kind, np.full(d, 0.5), s, noise)
    assert np.allclose(orc.kmm(same, V, h), expect, atol=1e-12)
    # V = e_j picks column j of Khat; linearity; permutation equivariance
    E = np.eye(n)
    assert np.allclose(orc.kmm(X, E, h), orc.khat(X, h))
    assert np.allclose(orc.kmm(X, 2 * V + E[:, :t], h), 2 * orc.kmm(X, V, h) + orc.khat(X, h)[:, :t])
    perm = rng.permutation(n)
    assert np.allclose(orc.kmm(X[perm], V[perm], h), orc.kmm(X, V, h)[perm])


def test_partition_invariance():
    """The partitioned product equals the unpartitioned one for any p (Method, 'Partitioned kernel MVMs')."""
    w = make_workload("C2", n=257)
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    full = orc.kmm(w.X, w.V, h)
    for p in (1, 2, 5, 257):
        parts = np.array_split(np.arange(257), p)
        cat = np.concatenate([orc.kmm_rows(w.X, w.V, h, rows) for rows in parts])
        assert np.allclose(cat, full, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("kind", KINDS)
def test_derivative_vs_finite_differences(kind):
    pts = well_separated_points(3, 30, 3).astype(np.float64)
    ls = np.array([0.3, 0.8, 1.5])
    h = orc.Hyper(kind, ls, 1.4, 0.1)
    eps = 1e-5
    for k in range(3):
        lp, lm = ls.copy(), ls.copy()
        lp[k] += eps
        lm[k] -= eps
        fd = (orc.kernel_matrix(pts, pts, orc.Hyper(kind, lp, 1.4)) -
              orc.kernel_matrix(pts, pts, orc.Hyper(kind, lm, 1.4))) / (2 * eps)
        an = orc.dkernel_dlengthscale(pts, pts, h, k)
        assert np.abs(fd - an).max() <= 1e-7 * max(1.0, np.abs(an).max())
    # Euler homogeneity: sum_k l_k dK/dl_k = s h(r) r^2
    r2 = orc.sq_dist(pts, pts, ls)
    total = sum(ls[k] * orc.dkernel_dlengthscale(pts, pts, h, k) for k in range(3))
    from oracle.gp_dense import _h
    assert np.allclose(total, 1.4 * _h(r2, kind) * r2, atol=1e-12)
    V = np.random.default_rng(1).standard_normal((30, 2))
    G = orc.kmm_grad(pts, V, h)
    assert G.shape == (3, 30, 2)
    assert np.allclose(G[1], orc.dkernel_dlengthscale(pts, pts, h, 1) @ V)
    assert np.allclose(orc.kmm_grad_rows(pts, V, h, [4, 9]), G[:, [4, 9], :])


def test_mll_gradient_vs_finite_differences():
    """Eq. 2 as printed is inconsistent; the oracle uses the standard identity, pinned here
    against central differences of Eq. 1."""
    rng = np.random.default_rng(2)
    n, d = 35, 2
    X = rng.uniform(0, 1, (n, d))
    y = np.sin(4 * X[:, 0]) + 0.1 * rng.standard_normal(n)
    theta = np.array([0.4, 0.9, 1.3, 0.05])
    for kind in KINDS:
        def f(th):
            return orc.mll(X, y, orc.Hyper(kind, th[:d], th[d], th[d + 1]))
        g = orc.mll_grad(X, y, orc.Hyper(kind, theta[:d], theta[d], theta[d + 1]))
        for k in range(d + 2):
            e = np.zeros_like(theta)
            e[k] = 1e-6
            fd = (f(theta + e) - f(theta - e)) / 2e-6
            assert abs(fd - g[k]) <= 2e-5 * max(1.0, abs(g[k]))
    # Eq. 1 against the multivariate normal log-density
    from scipy.stats import multivariate_normal
    h = orc.Hyper(orc.RBF, theta[:d], theta[d], theta[d + 1])
    ref = multivariate_normal(mean=np.zeros(n), cov=orc.khat(X, h)).logpdf(y)
    assert abs(orc.mll(X, y, h) - ref) < 1e-8


def test_matern12_is_the_ornstein_uhlenbeck_kernel():
    """In one dimension exp(-|x - x'| / l) is the covariance of a Markov process: the inverse of the kernel matrix
    of sorted points is tridiagonal, with the textbook closed form (rho_i = exp(-gap_i / l))."""
    rng = np.random.default_rng(12)
    x = np.sort(rng.uniform(0, 5, 12))
    ell, s = 0.7, 1.9
    K = orc.kernel_matrix(x[:, None], x[:, None], orc.Hyper(orc.MATERN12, [ell], s, 0.0))
    Kinv = np.linalg.inv(K)
    off = np.abs(np.triu(Kinv, 2)).max()
    assert off <= 1e-9 * np.abs(Kinv).max()
    rho = np.exp(-np.diff(x) / ell)
    expect_off = -rho / (1.0 - rho ** 2) / s
    assert np.allclose(np.diag(Kinv, 1), expect_off, rtol=1e-8)
