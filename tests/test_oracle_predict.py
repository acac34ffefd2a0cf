"""Pins for the oracle's prediction functions (CPU only)."""
import numpy as np
import pytest

import oracle as orc
from workloads import well_separated_points


def _problem(n=80, nq=15, kind=orc.MATERN32, seed=3):
    rng = np.random.default_rng(seed)
    X = well_separated_points(seed, n, 2)
    Xq = rng.uniform(0, 1, (nq, 2)).astype(np.float32)
    y = np.sin(6 * X[:, 0]) * np.cos(4 * X[:, 1]) + 0.1 * rng.standard_normal(n)
    h = orc.Hyper(kind, [0.3, 0.5], 1.4, 0.05)
    return X, Xq, y, h


def test_predict_exact_against_joint_gaussian_conditioning():
    """Mean and variance must equal the conditional of the joint Gaussian over (f(xq), y)."""
    X, Xq, y, h = _problem()
    mean, var = orc.predict_exact(X, y, Xq, h)
    for j in range(len(Xq)):
        Z = np.vstack([Xq[j:j + 1].astype(np.float64), X.astype(np.float64)])
        J = orc.kernel_matrix(Z, Z, h)
        J[1:, 1:] += h.noise * np.eye(len(X))         # noise on the observations only
        # Schur complement of the (y,y) block
        w = np.linalg.solve(J[1:, 1:], J[1:, 0])
        assert abs(mean[j] - w @ y) < 1e-9
        assert abs(var[j] - (J[0, 0] - J[0, 1:] @ w)) < 1e-9
    assert np.all(var > 0) and np.all(var <= h.outputscale + 1e-12)
    # at a training point with tiny noise the mean interpolates and the variance collapses
    h0 = orc.Hyper(h.kernel_type, h.lengthscales, h.outputscale, 1e-8)
    m0, v0 = orc.predict_exact(X, y, X[:5], h0)
    assert np.allclose(m0, y[:5], atol=1e-4) and np.all(np.abs(v0) < 1e-5)


def test_lanczos_invariants_and_cached_variance():
    X, Xq, y, h = _problem(n=60)
    Kh = orc.khat(X, h)
    Kq = orc.kernel_matrix(Xq, X, h)
    _, exact = orc.predict_exact(X, y, Xq, h)
    prev = None
    for r in (5, 20, 60):
        Q, al, be = orc.lanczos(Kh, y, r)
        m = len(al)
        assert np.allclose(Q @ Q.T, np.eye(m), atol=1e-10)
        T = Q @ Kh @ Q.T
        assert np.allclose(np.diag(T), al, atol=1e-9) and np.allclose(np.diag(T, 1), be, atol=1e-9)
        assert np.abs(np.triu(T, 2)).max() < 1e-8
        v = orc.predict_var_lanczos(Kq, Q, al, be, h.outputscale)
        assert np.all(v >= exact - 1e-9)              # Galerkin: Q^T T^-1 Q <= Khat^-1
        if prev is not None:
            assert np.all(v <= prev + 1e-9)           # monotone in the rank
        prev = v
    assert np.allclose(prev, exact, atol=1e-8)        # full Krylov space: exact
    # first Lanczos vector is the normalised start vector
    assert np.allclose(Q[0], y / np.linalg.norm(y))
    # the smallest ranks against the Galerkin formula with the projected matrix formed densely
    for r in (1, 2, 3):
        Q, al, be = orc.lanczos(Kh, y, r)
        G = Kq @ Q.T
        dense = h.outputscale - np.sum(G * np.linalg.solve(Q @ Kh @ Q.T, G.T).T, axis=1)
        assert np.allclose(orc.predict_var_lanczos(Kq, Q, al, be, h.outputscale), dense, atol=1e-10)


def test_block_lanczos_pins():
    """Block Krylov basis: reduces to the single-vector process for one start vector, spans the block Krylov space,
    gives a block-tridiagonal projection, and its Galerkin variance is an upper bound that decreases with the
    number of blocks and is exact once the space is the whole of R^n."""
    X, Xq, y, h = _problem(n=60)
    rng = np.random.default_rng(8)
    Kh = orc.khat(X, h)
    Kq = orc.kernel_matrix(Xq, X, h)
    _, exact = orc.predict_exact(X, y, Xq, h)
    # (1) one start vector: same subspace, same tridiagonal (up to the sign of each basis vector), same variance
    Q1, T1 = orc.block_lanczos(Kh, y, 12)
    Ql, al, be = orc.lanczos(Kh, y, 12)
    sign = np.sign(np.sum(Q1 * Ql, axis=1))
    assert np.allclose(Q1 * sign[:, None], Ql, atol=1e-8)
    assert np.allclose(np.diag(T1), al, atol=1e-9) and np.allclose(np.abs(np.diag(T1, 1)), be, atol=1e-9)
    assert np.allclose(orc.predict_var_galerkin(Kq, Q1, T1, h.outputscale),
                       orc.predict_var_lanczos(Kq, Ql, al, be, h.outputscale), atol=1e-10)
    # (2) a block of 4: orthonormal, T = Q Khat Q^T block tridiagonal, spans [B, Khat B, Khat^2 B]
    B0 = np.concatenate([y[:, None], rng.choice([-1.0, 1.0], size=(60, 3))], axis=1)
    Q, T = orc.block_lanczos(Kh, B0, 3)
    assert Q.shape == (12, 60) and np.allclose(Q @ Q.T, np.eye(12), atol=1e-10)
    assert np.allclose(T, Q @ Kh @ Q.T, atol=1e-9)
    assert np.abs(T[:4, 8:]).max() < 1e-8               # blocks (0, 2) vanish
    Kry = np.concatenate([B0, Kh @ B0, Kh @ Kh @ B0], axis=1)
    resid = Kry - Q.T @ (Q @ Kry)
    assert np.abs(resid).max() <= 1e-8 * np.abs(Kry).max()
    # (3) Galerkin bound, monotone in the number of blocks, exact at full dimension
    prev = None
    for m in (1, 3, 8, 15):
        Qm, Tm = orc.block_lanczos(Kh, B0, m)
        v = orc.predict_var_galerkin(Kq, Qm, Tm, h.outputscale)
        assert np.all(v >= exact - 1e-9)
        if prev is not None:
            assert np.all(v <= prev + 1e-9)
        prev = v
    assert Qm.shape[0] == 60 and np.allclose(prev, exact, atol=1e-8)
    # (4) planted mistake check: T without the projection (plain Khat block) must fail the identity
    assert not np.allclose(T, Kh[:12, :12], atol=1e-3)


def test_block_lanczos_start_block_conditions():
    """A start block with a repeated column is refused; columns of very different length are not (only the directions
    matter); asking for more blocks than the space holds stops at n basis vectors."""
    X, Xq, y, h = _problem(n=24)
    Kh = orc.khat(X, h)
    rng = np.random.default_rng(2)
    B = rng.standard_normal((24, 4))
    with pytest.raises(ValueError):
        orc.block_lanczos(Kh, np.concatenate([B, B[:, :1]], axis=1), 2)
    Bs = B * np.array([1.0, 1e-3, 1e3, 1e-6])
    Q1, T1 = orc.block_lanczos(Kh, B, 3)
    Q2, T2 = orc.block_lanczos(Kh, Bs, 3)
    assert Q2.shape == Q1.shape == (12, 24)
    assert np.allclose(Q1.T @ Q1, Q2.T @ Q2, atol=1e-8)          # same subspace: same orthogonal projector
    Qf, Tf = orc.block_lanczos(Kh, B, 10)
    assert Qf.shape[0] == 24 and np.allclose(Qf @ Qf.T, np.eye(24), atol=1e-9)
