"""Pins for the oracle's pivoted Cholesky, preconditioner, PCG and stochastic log-determinant (CPU only)."""
import numpy as np
import pytest
import scipy.linalg as sla
from scipy.linalg import lapack

import oracle as orc
from workloads import make_workload, well_separated_points, rademacher


def _setup(n=60, d=2, kind=orc.RBF, noise=0.05, ls=0.35, seed=11):
    X = well_separated_points(seed, n, d)
    h = orc.Hyper(kind, np.full(d, ls), 1.2, noise)
    return X, h, orc.kernel_matrix(X, X, h), orc.khat(X, h)


def test_pivoted_cholesky_full_rank_reproduces_K():
    X, h, K, _ = _setup(n=40, ls=0.15)
    L, piv = orc.pivoted_cholesky(K, 40)
    assert L.shape == (40, 40) and sorted(piv.tolist()) == list(range(40))
    assert np.linalg.norm(L @ L.T - K) / np.linalg.norm(K) <= 1e-10


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
def test_pivoted_cholesky_invariants_and_greedy_pivots(kind):
    X, h, K, _ = _setup(n=80, kind=kind)
    k = 12
    L, piv = orc.pivoted_cholesky(K, k)
    assert piv[0] == 0                      # diag K = s everywhere: n-way tie -> lowest index
    assert len(set(piv.tolist())) == k
    # pivot rows are interpolated exactly
    A = L @ L.T
    assert np.allclose(A[piv, :], K[piv, :], atol=1e-12)
    # residual diagonal non-negative, trace non-increasing, pivots = greedy arg-max of dense Schur complement
    S = K.copy()
    prev_trace = np.trace(S)
    for m in range(k):
        dg = np.diag(S).copy()
        dg[piv[:m]] = -np.inf
        assert int(np.argmax(dg)) == piv[m]
        p = piv[m]
        S = S - np.outer(S[:, p], S[p, :]) / S[p, p]
        assert np.diag(S).min() >= -1e-12
        assert np.trace(S) <= prev_trace + 1e-12
        prev_trace = np.trace(S)
        Lm = L[:, :m + 1]
        assert np.allclose(K - Lm @ Lm.T, S, atol=1e-10)


def test_pivoted_cholesky_matches_lapack_dpstrf():
    X, h, K, _ = _setup(n=50, ls=0.2)
    k = 50
    L, piv = orc.pivoted_cholesky(K, k)
    c, lpiv, rank, info = lapack.dpstrf(K, lower=1)
    lpiv = lpiv - 1
    # LAPACK swaps rows physically; selection order must agree while the maxima are well separated
    assert list(piv[:15]) == list(lpiv[:15])
    Lp = np.tril(c)
    # rows of LAPACK's factor are in pivoted order: L_lapack[j,:] corresponds to original row lpiv[j]
    assert np.allclose(L[lpiv][:, :15], Lp[:, :15], atol=1e-9)


def test_pivoted_cholesky_early_stop():
    X = np.tile(np.array([[0.2, 0.4]], np.float32), (10, 1))      # rank-1 K
    h = orc.Hyper(orc.RBF, [1.0, 1.0], 1.0, 0.0)
    L, piv = orc.pivoted_cholesky(orc.kernel_matrix(X, X, h), 5, tol_abs=1e-12)
    assert L.shape[1] == 1 and piv.tolist() == [0]


def test_preconditioner_woodbury_and_determinant_lemma():
    X, h, K, Kh = _setup(n=70)
    L, _ = orc.pivoted_cholesky(K, 9)
    R = np.random.default_rng(0).standard_normal((70, 3))
    s2 = h.noise
    small = s2 * np.eye(9) + L.T @ L
    woodbury = (R - L @ np.linalg.solve(small, L.T @ R)) / s2
    assert np.allclose(orc.precond_solve(L, s2, R), woodbury, atol=1e-9)
    lemma = np.linalg.slogdet(small)[1] + (70 - 9) * np.log(s2)
    assert abs(orc.precond_logdet(L, s2) - lemma) < 1e-9
    P = orc.precond_matrix(L, s2)
    assert np.allclose(orc.precond_solve(L, s2, P), np.eye(70), atol=1e-9)


def test_pcg_matches_cholesky_and_terminates():
    X, h, K, Kh = _setup(n=60)
    b = np.random.default_rng(3).standard_normal(60)
    ref = orc.chol_solve(Kh, b)
    assert np.allclose(Kh @ ref, b, atol=1e-10)
    assert np.allclose(ref, np.linalg.solve(Kh, b), atol=1e-9)
    res = orc.pcg(Kh, b, None, max_iter=200, tol=1e-13)
    assert np.allclose(res["u"], ref, rtol=1e-8, atol=1e-10)
    assert res["rel_resid"][-1] <= 1e-13
    # tolerance controls the gap to the exact solve, monotonically in tol
    errs = []
    for tol in (1e-1, 1e-3, 1e-6):
        u = orc.pcg(Kh, b, None, 500, tol)["u"]
        errs.append(np.linalg.norm(u - ref))
        assert np.linalg.norm(Kh @ u - b) / np.linalg.norm(b) <= tol * 1.0001
    assert errs[0] > errs[1] > errs[2]
    # exact preconditioner -> one iteration
    one = orc.pcg(Kh, b, np.linalg.inv(Kh), 50, 1e-10)
    assert len(one["alphas"]) == 1 and np.allclose(one["u"], ref, atol=1e-9)
    # preconditioned and plain systems share the solution (Method, 'Preconditioning'), in fewer iterations
    L, _ = orc.pivoted_cholesky(K, 10)
    Pinv = np.linalg.inv(orc.precond_matrix(L, h.noise))
    pre = orc.pcg(Kh, b, Pinv, 200, 1e-10)
    plain = orc.pcg(Kh, b, None, 200, 1e-10)
    assert np.allclose(pre["u"], plain["u"], atol=1e-7)
    assert len(pre["alphas"]) < len(plain["alphas"])


def test_cg_tridiagonal_is_lanczos_of_preconditioned_operator():
    X, h, K, Kh = _setup(n=30, ls=0.25, noise=0.3)
    n = 30
    L, _ = orc.pivoted_cholesky(K, 4)
    P = orc.precond_matrix(L, h.noise)
    Pinv = np.linalg.inv(P)
    z = np.random.default_rng(8).standard_normal(n)
    res = orc.pcg(Kh, z, Pinv, max_iter=n, tol=1e-15)
    T = orc.tridiag_from_cg(res["alphas"], res["betas"])
    # Ritz values inside the spectrum of P^{-1/2} Khat P^{-1/2}
    w, Q = np.linalg.eigh(P)
    Pmh = Q @ np.diag(w ** -0.5) @ Q.T
    M = Pmh @ Kh @ Pmh
    lam = np.linalg.eigvalsh(M)
    ritz = np.linalg.eigvalsh(T)
    assert ritz.min() >= lam.min() * (1 - 1e-8) and ritz.max() <= lam.max() * (1 + 1e-8)
    # Gauss quadrature exact after full Lanczos: gamma0 e1^T log(T) e1 = z^T P^{-1/2} log(M) P^{-1/2} z
    lm, Qm = np.linalg.eigh(M)
    logM = Qm @ np.diag(np.log(lm)) @ Qm.T
    exact = z @ Pmh @ logM @ Pmh @ z
    # (the Krylov space is exhausted once the residual vanishes, which happens within n steps)
    assert res["rel_resid"][-1] < 1e-12 and len(res["alphas"]) <= n
    assert abs(res["gamma0"] * orc.slq_quadrature(T) - exact) <= 1e-6 * abs(exact) + 1e-8
    # identity e1^T T^{-1} e1 * gamma0 = z^T Khat^{-1} z  (CG solves the system through T)
    e1 = np.zeros(len(T)); e1[0] = 1
    assert abs(res["gamma0"] * (e1 @ np.linalg.solve(T, e1)) - z @ orc.chol_solve(Kh, z)) < 1e-8


def test_slq_logdet_within_monte_carlo_error():
    w = make_workload("C1", n=256)
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, 0.1)
    Kh = orc.khat(w.X, h)
    exact = orc.logdet(Kh)
    assert abs(exact - np.linalg.slogdet(Kh)[1]) < 1e-8
    rng = np.random.default_rng(4)
    tp = 512
    # no preconditioner: identity-covariance Rademacher probes
    est, terms = orc.slq_logdet(Kh, rademacher(rng, (256, tp)), max_iter=256)
    se = terms.std(ddof=1) / np.sqrt(tp)
    assert abs(est - exact) <= 4 * se + 1e-6
    # with preconditioner: probes need covariance P
    L, _ = orc.pivoted_cholesky(orc.kernel_matrix(w.X, w.X, h), 8)
    Z = orc.probes_with_cov_P(L, h.noise, rademacher(rng, (8, tp)), rademacher(rng, (256, tp)))
    est2, terms2 = orc.slq_logdet(Kh, Z, L, h.noise, max_iter=256)
    se2 = terms2.std(ddof=1) / np.sqrt(tp)
    assert abs(est2 - exact) <= 4 * se2 + 1e-6
    assert se2 < se          # the preconditioner removes variance


def test_stochastic_mll_terms_within_monte_carlo_error():
    rng = np.random.default_rng(6)
    n, d, tp = 120, 2, 400
    X = well_separated_points(21, n, d)
    y = np.sin(5 * X[:, 0]) + 0.2 * rng.standard_normal(n)
    h = orc.Hyper(orc.MATERN32, [0.3, 0.6], 1.1, 0.2)
    K = orc.kernel_matrix(X, X, h)
    L, _ = orc.pivoted_cholesky(K, 6)
    Z = orc.probes_with_cov_P(L, h.noise, rademacher(rng, (6, tp)), rademacher(rng, (n, tp)))
    out = orc.mll_stochastic_terms(X, y, h, Z, L)
    assert abs(out["mll"] - orc.mll(X, y, h)) < 0.5
    g = orc.mll_grad(X, y, h)
    assert np.all(np.abs(out["grad"] - g) <= 0.15 * np.abs(g) + 0.5)


def test_adam_loop_pins():
    """Oracle training loop: no-op at zero steps; the first Adam step moves every log-parameter by exactly
    +-lr in the direction of its gradient sign; the exact objective rises with exact gradients."""
    rng = np.random.default_rng(10)
    n, d = 60, 2
    X = well_separated_points(41, n, d)
    y = np.sin(5 * X[:, 0]) + 0.3 * rng.standard_normal(n)
    h0 = orc.Hyper(orc.RBF, [0.8, 0.8], 0.7, 0.6)
    h_same, hist = orc.train_adam(X, y, h0, steps=0)
    assert np.allclose(h_same.lengthscales, h0.lengthscales) and len(hist) == 1
    assert abs(hist[0] - orc.mll(X, y, h0)) < 1e-12
    floor = 0.05
    h1, _ = orc.train_adam(X, y, h0, steps=1, lr=0.1, noise_floor=floor)
    g = orc.mll_grad(X, y, orc.Hyper(orc.RBF, h0.lengthscales, h0.outputscale, h0.noise))
    moved = np.log(np.concatenate([h1.lengthscales / h0.lengthscales, [h1.outputscale / h0.outputscale],
                                   [(h1.noise - floor) / (h0.noise - floor)]]))
    assert np.allclose(moved, 0.1 * np.sign(g), atol=1e-6)
    _, hist = orc.train_adam(X, y, h0, steps=15, lr=0.05)
    assert hist[-1] > hist[0] + 1.0 and all(b > a - 0.05 for a, b in zip(hist, hist[1:]))
    hf, _ = orc.train_adam(X, y, h0, steps=3, lr=0.5, noise_floor=0.3)
    assert hf.noise > 0.3


def test_pcg_history_is_the_true_relative_residual():
    """Entry j of the residual history is ||b - Khat u_{j+1}|| / ||b||, for a b whose norm is far from one, with and
    without a preconditioner (in fp64 the recurrence residual and the true one agree to rounding at these sizes)."""
    X, h, K, Kh = _setup(n=50, noise=0.2)
    b = 7.3 * np.random.default_rng(5).standard_normal(50)
    L, _ = orc.pivoted_cholesky(K, 6)
    for Pinv in (None, np.linalg.inv(orc.precond_matrix(L, h.noise))):
        for j in (1, 3, 8):
            res = orc.pcg(Kh, b, Pinv, max_iter=j, tol=0.0)
            assert len(res["rel_resid"]) == j and len(res["alphas"]) == j and len(res["betas"]) == j
            true = np.linalg.norm(b - Kh @ res["u"]) / np.linalg.norm(b)
            assert abs(res["rel_resid"][-1] - true) <= 1e-9 * true
        full = orc.pcg(Kh, b, Pinv, max_iter=8, tol=0.0)["rel_resid"]
        part = orc.pcg(Kh, b, Pinv, max_iter=3, tol=0.0)["rel_resid"]
        assert np.allclose(full[:3], part, rtol=1e-12)


def test_truncated_cg_tridiagonal_equals_explicit_lanczos():
    """After m < n iterations the tridiagonal built from the CG coefficients is, entry by entry, the one that m
    explicit Lanczos steps on P^{-1/2} Khat P^{-1/2} from the start vector P^{-1/2} z produce (the Lanczos routine
    is pinned on its own by orthonormality and Q A Q^T = T). Off-diagonals are positive in both conventions."""
    X, h, K, Kh = _setup(n=40, ls=0.25, noise=0.3)
    L, _ = orc.pivoted_cholesky(K, 5)
    P = orc.precond_matrix(L, h.noise)
    w, Q = np.linalg.eigh(P)
    Pmh = Q @ np.diag(w ** -0.5) @ Q.T
    M = Pmh @ Kh @ Pmh
    z = np.random.default_rng(12).standard_normal(40)
    for m in (1, 2, 7):
        res = orc.pcg(Kh, z, np.linalg.inv(P), max_iter=m, tol=0.0)
        T = orc.tridiag_from_cg(res["alphas"], res["betas"])
        assert T.shape == (m, m) and np.allclose(T, T.T)
        _, a, b = orc.lanczos(M, Pmh @ z, m)
        assert np.allclose(np.diag(T), a, rtol=1e-9)
        assert np.allclose(np.diag(T, 1), b, rtol=1e-8)
        assert np.allclose(np.triu(T, 2), 0.0)
    # no preconditioner: the same against Lanczos on Khat itself
    res = orc.pcg(Kh, z, None, max_iter=6, tol=0.0)
    T = orc.tridiag_from_cg(res["alphas"], res["betas"])
    _, a, b = orc.lanczos(Kh, z, 6)
    assert np.allclose(np.diag(T), a, rtol=1e-9) and np.allclose(np.diag(T, 1), b, rtol=1e-8)
    assert abs(res["gamma0"] - z @ z) <= 1e-12 * (z @ z)


def test_stochastic_estimators_are_exact_for_a_complete_probe_set():
    """With n probe columns Z such that Z Z^T / n = P exactly (P^{1/2} times a Hadamard matrix; P = I without a
    preconditioner) the probe averages are exact traces and, after full Lanczos runs, Gauss quadrature is exact:
    the stochastic log-determinant, value and gradient must equal the dense ones — no Monte-Carlo band."""
    n, d = 32, 2
    X = well_separated_points(5, n, d)
    rng = np.random.default_rng(6)
    y = np.sin(4 * X[:, 0]) + 0.3 * rng.standard_normal(n)
    H = sla.hadamard(n).astype(np.float64)
    for kind in (orc.RBF, orc.MATERN32, orc.MATERN12):
        h = orc.Hyper(kind, [0.3, 0.45], 1.3, 0.25)
        Kh = orc.khat(X, h)
        exact_ld = np.linalg.slogdet(Kh)[1]
        est, terms = orc.slq_logdet(Kh, H)
        assert abs(est - exact_ld) <= 1e-7 * abs(exact_ld) + 1e-7
        L, _ = orc.pivoted_cholesky(orc.kernel_matrix(X, X, h), 5)
        P = orc.precond_matrix(L, h.noise)
        Z = np.linalg.cholesky(P) @ H
        assert np.allclose(Z @ Z.T / n, P, atol=1e-12)
        est, _ = orc.slq_logdet(Kh, Z, L, h.noise)
        assert abs(est - exact_ld) <= 1e-7 * abs(exact_ld) + 1e-7
        for LL, ZZ in ((None, H), (L, Z)):
            out = orc.mll_stochastic_terms(X, y, h, ZZ, LL)
            assert abs(out["mll"] - orc.mll(X, y, h)) <= 1e-7 * abs(orc.mll(X, y, h)) + 1e-7
            g = orc.mll_grad(X, y, h)
            assert np.allclose(out["grad"], g, rtol=1e-6, atol=1e-7 * np.abs(g).max())


def test_adam_second_step_follows_the_published_recurrences():
    """Two steps of the loop against the Adam recurrences written out (first and second moment with decay 0.9 and
    0.999, bias correction, step lr * m^ / (sqrt(v^) + 1e-8)) on the gradient of L / n in the log-parameters; the
    gradient in natural parameters comes from the dense formula, which is pinned by finite differences. The noise
    enters as log(noise - floor)."""
    rng = np.random.default_rng(10)
    n, d = 60, 2
    X = well_separated_points(41, n, d)
    y = np.sin(5 * X[:, 0]) + 0.3 * rng.standard_normal(n)
    floor, lr = 0.05, 0.07
    h0 = orc.Hyper(orc.MATERN52, [0.6, 1.1], 0.7, 0.6)
    h1, _ = orc.train_adam(X, y, h0, steps=1, lr=lr, noise_floor=floor)
    h2, hist = orc.train_adam(X, y, h0, steps=2, lr=lr, noise_floor=floor)
    assert len(hist) == 3 and abs(hist[1] - orc.mll(X, y, h1)) <= 1e-9 * abs(hist[1])
    assert abs(hist[2] - orc.mll(X, y, h2)) <= 1e-9 * abs(hist[2])

    def phi(h):
        return np.log(np.concatenate([h.lengthscales, [h.outputscale], [h.noise - floor]]))

    def glog(h):      # chain rule: d/d log(theta) = theta d/d theta; for the noise theta = noise - floor
        return np.concatenate([h.lengthscales, [h.outputscale], [h.noise - floor]]) * orc.mll_grad(X, y, h) / n

    g1, g2 = glog(h0), glog(h1)
    m2 = 0.9 * (0.1 * g1) + 0.1 * g2
    v2 = 0.999 * (0.001 * g1 * g1) + 0.001 * g2 * g2
    step2 = lr * (m2 / (1 - 0.9 ** 2)) / (np.sqrt(v2 / (1 - 0.999 ** 2)) + 1e-8)
    assert np.allclose(phi(h1) - phi(h0), lr * np.sign(g1), atol=1e-6)
    assert np.allclose(phi(h2) - phi(h1), step2, rtol=1e-7, atol=1e-10)
    assert np.abs(step2).max() <= lr * 1.0001 and np.abs(np.abs(step2) - lr).max() > 1e-4   # not again a pure sign step


def test_probe_covariance_is_P_for_a_complete_sign_design():
    """z = L w1 + sigma w2 over a complete orthogonal design of sign vectors (rows of a Hadamard matrix as the
    coordinates of [w1; w2]) has second moment exactly L L^T + sigma^2 I; with such draws the stochastic training loop
    (preconditioned, probes of covariance P) retraces the loop with exact values and gradients."""
    n, d, k, N = 60, 2, 4, 64
    X = well_separated_points(41, n, d)
    rng = np.random.default_rng(3)
    y = np.sin(5 * X[:, 0]) + 0.3 * rng.standard_normal(n)
    h0 = orc.Hyper(orc.RBF, [0.8, 0.6], 0.9, 0.4)
    H = sla.hadamard(N).astype(np.float64)
    W1, W2 = H[:k], H[k:k + n]                        # (k, N) and (n, N): orthogonal rows, N probe columns
    L, _ = orc.pivoted_cholesky(orc.kernel_matrix(X, X, h0), k)
    Z = orc.probes_with_cov_P(L, h0.noise, W1, W2)
    assert np.allclose(Z @ Z.T / N, orc.precond_matrix(L, h0.noise), atol=1e-12)
    assert np.allclose(Z @ Z.T / N, L @ L.T + h0.noise * np.eye(n), atol=1e-12)
    _, hist0 = orc.train_adam(X, y, h0, steps=0, rank=k, W1=W1, W2=W2)
    assert abs(hist0[0] - orc.mll_stochastic_terms(X, y, h0, Z, L)["mll"]) <= 1e-10 * abs(hist0[0])
    hs, hist_s = orc.train_adam(X, y, h0, steps=3, lr=0.1, noise_floor=0.05, rank=k, W1=W1, W2=W2)
    he, hist_e = orc.train_adam(X, y, h0, steps=3, lr=0.1, noise_floor=0.05)
    assert np.allclose(hist_s, hist_e, rtol=1e-6)
    assert np.allclose(hs.lengthscales, he.lengthscales, rtol=1e-5)
    assert abs(hs.outputscale - he.outputscale) <= 1e-5 * he.outputscale and abs(hs.noise - he.noise) <= 1e-5 * he.noise
    # without a preconditioner the probes are W2 itself (identity covariance): the same holds
    # (rank 0 is the default)
    hs0, hist_s0 = orc.train_adam(X, y, h0, steps=2, lr=0.1, noise_floor=0.05, W2=H[:n])
    assert np.allclose(hist_s0, hist_e[:3], rtol=1e-6)
    # rank 1 is a preconditioner like any other
    L1, _ = orc.pivoted_cholesky(orc.kernel_matrix(X, X, h0), 1)
    Z1 = orc.probes_with_cov_P(L1, h0.noise, H[:1], H[1:1 + n])
    assert np.allclose(Z1 @ Z1.T / N, orc.precond_matrix(L1, h0.noise), atol=1e-12)
    # (eight probes only, so that the estimate is not exact and depends on the preconditioner being used)
    _, hist1 = orc.train_adam(X, y, h0, steps=0, rank=1, W1=H[:1, :8], W2=H[1:1 + n, :8])
    want = orc.mll_stochastic_terms(X, y, h0, Z1[:, :8], L1)["mll"]
    assert abs(hist1[0] - want) <= 1e-10 * abs(want)
    assert abs(want - orc.mll_stochastic_terms(X, y, h0, H[1:1 + n, :8], None)["mll"]) > 1e-6 * abs(want)


def test_adam_defaults_and_noise_floor_edge():
    """Defaults follow the paper's experiment details (Adam, learning rate 0.1) with no floor; a start value at or
    below the floor is lifted just above it, never onto it (log(noise - floor) must exist)."""
    rng = np.random.default_rng(10)
    n, d = 40, 2
    X = well_separated_points(41, n, d)
    y = np.sin(5 * X[:, 0]) + 0.3 * rng.standard_normal(n)
    h0 = orc.Hyper(orc.RBF, [0.8, 0.8], 0.7, 0.6)
    h1, _ = orc.train_adam(X, y, h0, steps=1)
    g = orc.mll_grad(X, y, h0)
    moved = np.log(np.concatenate([h1.lengthscales / h0.lengthscales, [h1.outputscale / h0.outputscale],
                                   [h1.noise / h0.noise]]))
    assert np.allclose(moved, 0.1 * np.sign(g), atol=1e-6)      # lr = 0.1, floor 0: the noise itself is the parameter
    for floor, start in ((0.3, 0.3), (0.3, 0.1), (0.0, 0.0)):
        hz, _ = orc.train_adam(X, y, orc.Hyper(orc.RBF, [0.8, 0.8], 0.7, start), steps=0, noise_floor=floor)
        lift = 1e-4 * (floor if floor > 0 else 1.0)
        assert floor < hz.noise <= floor + 1.0001 * lift
