"""Parity of the HIP pivoted-Cholesky preconditioner and batched PCG with the dense fp64 oracle."""
import numpy as np
import pytest

import oracle as orc
from workloads import make_workload, well_separated_points, rademacher

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
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,rank", [(64, 2, 8), (300, 3, 20), (1000, 2, 12), (4100, 2, 12), (4101, 2, 12)])
def test_pivots_bit_exact_and_factor(egp, kind, n, d, rank):
    """Pivot order must equal the oracle's exactly on well-separated tiny inputs (no near-ties). n = 4100 takes the
    step kernel's four-points-per-thread path (n a multiple of 4, at least 4096), n = 4101 the scalar one."""
    X = well_separated_points(100 + n + kind, n, d)
    ls = np.full(d, 0.3, np.float32)
    s, noise = 1.5, 0.05
    h = orc.Hyper(kind, ls, s, noise)
    K = orc.kernel_matrix(X, X, h)
    Lref, pref = orc.pivoted_cholesky(K, rank)
    P = egp.piv_chol_precond(_cuda(X), ls, s, noise, kind, rank)
    assert P.rank == rank
    assert P.pivots.tolist() == pref.tolist()
    Lg = P.L.cpu().numpy().astype(np.float64).T
    assert np.abs(Lg - Lref).max() <= 2e-4 * np.sqrt(s)
    # small factor and log|P| (determinant lemma on the GPU side vs dense slogdet in the oracle)
    small_ref = np.linalg.cholesky(noise * np.eye(rank) + Lref.T @ Lref)
    assert np.abs(P.chol_small - small_ref).max() <= 1e-3
    assert abs(P.logdet - orc.precond_logdet(Lref, noise)) <= 1e-3 * max(1.0, abs(orc.precond_logdet(Lref, noise)))


def test_pivchol_early_stop_and_errors(egp):
    import torch
    X = np.tile(np.array([[0.2, 0.4]], np.float32), (40, 1))
    P = egp.piv_chol_precond(_cuda(X), [1.0, 1.0], 1.0, 0.1, orc.RBF, 5, tol_abs=1e-5)
    assert P.rank == 1 and P.pivots.tolist() == [0]
    with pytest.raises(egp.EgpError):
        egp.piv_chol_precond(_cuda(X), [1.0, 1.0], 1.0, 0.0, orc.RBF, 5)     # noise must be > 0
    with pytest.raises(egp.EgpError):
        egp.piv_chol_precond(_cuda(X), [1.0, 1.0], 1.0, 0.1, orc.RBF, 41)    # rank > n


@pytest.mark.parametrize("t", [1, 16, 17, 33])
def test_precond_apply_matches_dense_solve(egp, t):
    n, d, rank = 777, 3, 16
    X = well_separated_points(5, n, d)
    ls = np.full(d, 0.4, np.float32)
    noise = 0.2
    P = egp.piv_chol_precond(_cuda(X), ls, 1.0, noise, orc.MATERN32, rank)
    R = np.random.default_rng(t).standard_normal((n, t)).astype(np.float32)
    Z = egp.precond_apply(P, _cuda(R)).cpu().numpy().astype(np.float64)
    Lg = P.L.cpu().numpy().astype(np.float64).T
    ref = orc.precond_solve(Lg, noise, R)
    assert np.linalg.norm(Z - ref) / np.linalg.norm(ref) <= 1e-4


@pytest.mark.parametrize("rank", [300, 1024])
def test_high_rank_preconditioner_small_noise(egp, rank):
    """Rank up to EGP_RANK_MAX with lambda_max / noise ~ 10^6: P^{-1} R loses everything to cancellation unless the
    k x k algebra and its n-term sums are carried in fp64. Checked against the dense fp64 solve with the GPU's own L
    (P is defined by the stored factor), on a smooth right-hand side that lives in the range of L."""
    n, d = 3000, 2
    rng = np.random.default_rng(rank)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    ls = np.full(d, 0.3, np.float32)
    s, noise, kind = 2.0, 1e-3, orc.MATERN32      # slowly decaying spectrum: every requested step is taken
    P = egp.piv_chol_precond(_cuda(X), ls, s, noise, kind, rank)
    assert P.rank == rank
    Lg = P.L.cpu().numpy().astype(np.float64).T
    R = np.stack([np.sin(3 * X[:, 0]) + X[:, 1], np.cos(2 * X[:, 1]), rng.standard_normal(n)], axis=1).astype(np.float32)
    Z = egp.precond_apply(P, _cuda(R)).cpu().numpy().astype(np.float64)
    ref = orc.precond_solve(Lg, noise, R)
    for c in range(3):
        assert np.linalg.norm(Z[:, c] - ref[:, c]) / np.linalg.norm(ref[:, c]) <= 1e-4, c
    # r^T P^{-1} r stays positive and accurate for the smooth columns (where the fp32 version produced noise)
    for c in range(2):
        assert abs(R[:, c].astype(np.float64) @ Z[:, c] - R[:, c].astype(np.float64) @ ref[:, c]) <= \
            1e-4 * abs(R[:, c].astype(np.float64) @ ref[:, c])
    assert abs(P.logdet - orc.precond_logdet(Lg, noise)) <= 1e-6 * abs(orc.precond_logdet(Lg, noise)) + 1e-3
    # the solver uses it: convergence to the dense solution
    B = R[:, :2].copy()
    res = egp.mbcg(_cuda(X), _cuda(B), ls, s, noise, kind, precond=P, max_iter=300, tol=1e-4)
    assert res["rel_resid"].max() <= 1e-4
    Kh = orc.khat(X, orc.Hyper(kind, ls, s, noise))
    true_res = np.linalg.norm(Kh @ res["U"].cpu().numpy().astype(np.float64) - B, axis=0) / np.linalg.norm(B, axis=0)
    assert true_res.max() <= 5e-3


def test_mbcg_c1(egp):
    """C1: 20 iterations, rank-5 preconditioner; compared with the oracle's column-by-column PCG run with
    the same preconditioner, and with the Cholesky solution."""
    w = make_workload("C1")
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    Xd, Bd = _cuda(w.X), _cuda(w.V)
    P = egp.piv_chol_precond(Xd, w.lengthscales, w.outputscale, w.noise, w.kernel_type, w.rank)
    K = orc.kernel_matrix(w.X, w.X, h)
    Lref, pref = orc.pivoted_cholesky(K, w.rank)
    assert P.pivots.tolist() == pref.tolist()
    res = egp.mbcg(Xd, Bd, w.lengthscales, w.outputscale, w.noise, w.kernel_type, precond=P, max_iter=20, tol=0.0)
    assert res["iters"] == 20
    U = res["U"].cpu().numpy().astype(np.float64)
    Kh = K + w.noise * np.eye(w.n)
    Pinv = np.linalg.inv(orc.precond_matrix(Lref, w.noise))
    B = w.V.astype(np.float64)
    for c in (0, 1, 15):
        ref = orc.pcg(Kh, B[:, c], Pinv, max_iter=20, tol=0.0)
        # early coefficients agree tightly, later ones drift with fp32 rounding
        assert np.allclose(res["alphas"][:5, c], ref["alphas"][:5], rtol=2e-3)
        assert np.allclose(res["betas"][:4, c], ref["betas"][:4], rtol=5e-3)
        assert abs(res["gamma0"][c] - ref["gamma0"]) <= 1e-4 * abs(ref["gamma0"])
        # after 20 iterations of this ill-conditioned, unconverged solve rounding has moved the iterates:
        # same order of magnitude only (the 4-iteration run below is compared tightly)
        assert 0.5 * ref["rel_resid"][-1] <= res["rel_resid"][c] <= 2.0 * ref["rel_resid"][-1]
        # unconverged iterates of an ill-conditioned system drift apart with rounding; what is fixed is
        # that both satisfy the system to their residuals: ||Khat (u - u_ref)|| <= ||r|| + ||r_ref||
        gap = np.linalg.norm(Kh @ (U[:, c] - ref["u"])) / np.linalg.norm(B[:, c])
        assert gap <= 1.05 * (res["rel_resid"][c] + ref["rel_resid"][-1]) + 1e-4
    # a short run is compared iterate for iterate
    short = egp.mbcg(Xd, Bd, w.lengthscales, w.outputscale, w.noise, w.kernel_type, precond=P, max_iter=4, tol=0.0)
    Us = short["U"].cpu().numpy().astype(np.float64)
    for c in (0, 7):
        ref = orc.pcg(Kh, B[:, c], Pinv, max_iter=4, tol=0.0)
        assert np.linalg.norm(Us[:, c] - ref["u"]) / np.linalg.norm(ref["u"]) <= 2e-3
        assert abs(short["rel_resid"][c] - ref["rel_resid"][-1]) <= 2e-3 * ref["rel_resid"][-1]
    # the recurrence residual the solver reports equals the true residual
    true_res = np.linalg.norm(Kh @ U - B, axis=0) / np.linalg.norm(B, axis=0)
    assert np.allclose(true_res, res["rel_resid"], rtol=0.05, atol=2e-4)


@pytest.mark.parametrize("use_precond", [False, True])
@pytest.mark.parametrize("t", [1, 5, 17])
def test_mbcg_converges_to_cholesky(egp, use_precond, t):
    n, d = 1500, 4
    rng = np.random.default_rng(17 + t)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    B = rademacher(rng, (n, t))
    B[:, 0] = np.sin(4 * X[:, 0]) + 0.1 * rng.standard_normal(n)
    ls = np.full(d, 0.35, np.float32)
    s, noise = 1.0, 0.05
    kind = orc.MATERN52
    Xd, Bd = _cuda(X), _cuda(B)
    P = egp.piv_chol_precond(Xd, ls, s, noise, kind, 30) if use_precond else None
    res = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=P, max_iter=400, tol=1e-4)
    assert res["rel_resid"].max() <= 1e-4
    Kh = orc.khat(X, orc.Hyper(kind, ls, s, noise))
    ref = orc.chol_solve(Kh, B)
    U = res["U"].cpu().numpy().astype(np.float64)
    assert np.linalg.norm(U - ref) / np.linalg.norm(ref) <= 5e-3
    true_res = np.linalg.norm(Kh @ U - B, axis=0) / np.linalg.norm(B, axis=0)
    assert true_res.max() <= 5e-4
    if use_precond:
        plain = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=None, max_iter=400, tol=1e-4)
        assert res["iters"] < plain["iters"]


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32])
def test_mbcg_in_bf16_split_modes(egp, mode, kind):
    """The opt-in contraction modes keep the multiply's relative error near 1e-5, so the solver converges to the
    same solution; the attainable true residual is that error times ||Khat|| ||u|| / ||b|| (here ~1e-3)."""
    n, d, t = 3000, 11, 17
    rng = np.random.default_rng(300 + mode + kind)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    B = rademacher(rng, (n, t))
    B[:, 0] = np.sin(4 * X[:, 0]) + 0.1 * rng.standard_normal(n)
    ls = np.exp(rng.uniform(np.log(0.3), np.log(1.5), d)).astype(np.float32)
    s, noise = 1.0, 0.05
    Xd, Bd = _cuda(X), _cuda(B)
    L = egp.lib()
    try:
        L.egp_set_kmm_mode(mode)
        P = egp.piv_chol_precond(Xd, ls, s, noise, kind, 30)
        res = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=P, max_iter=400, tol=1e-3)
    finally:
        L.egp_set_kmm_mode(0)
    assert res["rel_resid"].max() <= 1e-3
    Kh = orc.khat(X, orc.Hyper(kind, ls, s, noise))
    ref = orc.chol_solve(Kh, B)
    U = res["U"].cpu().numpy().astype(np.float64)
    assert np.linalg.norm(U - ref) / np.linalg.norm(ref) <= 5e-3
    true_res = np.linalg.norm(Kh @ U - B, axis=0) / np.linalg.norm(B, axis=0)
    assert true_res.max() <= 3e-3


def test_mbcg_batched_equals_single_and_duplicates(egp):
    n, d = 900, 3
    rng = np.random.default_rng(2)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    b = rng.standard_normal((n, 1)).astype(np.float32)
    B = np.concatenate([b, rademacher(rng, (n, 3)), b], axis=1)
    ls = np.full(d, 0.5, np.float32)
    Xd = _cuda(X)
    batched = egp.mbcg(Xd, _cuda(B), ls, 1.0, 0.1, orc.RBF, max_iter=15, tol=0.0)
    Ub = batched["U"].cpu().numpy()
    assert np.array_equal(Ub[:, 0], Ub[:, 4])                       # duplicate columns: identical results
    # a column solved alone takes the single-column kernel (contraction on the VALU, another summation order):
    # the first coefficients agree to rounding; unconverged iterates of this ill-conditioned system drift apart,
    # so the solutions are compared after convergence
    single = egp.mbcg(Xd, _cuda(b), ls, 1.0, 0.1, orc.RBF, max_iter=15, tol=0.0)
    assert np.allclose(batched["alphas"][:3, 0], single["alphas"][:3, 0], rtol=1e-4)
    # each side against the oracle's textbook PCG on the dense matrix: coefficients of the first iterations to 1e-3
    # and the residual history while it is above the fp32 floor (later fp32 iterates drift, as the solver's
    # specification expects of CG in single precision)
    ref = orc.pcg(orc.khat(X, orc.Hyper(orc.RBF, ls, 1.0, 0.1)), b[:, 0], max_iter=15)
    for side in (batched, single):
        assert np.allclose(side["alphas"][:5, 0], ref["alphas"][:5], rtol=1e-3)
        assert np.allclose(side["betas"][:4, 0], ref["betas"][:4], rtol=1e-3)
        assert np.allclose(side["resid_hist"][:6, 0], ref["rel_resid"][:6], rtol=2e-2)
    both = egp.mbcg(Xd, _cuda(B), ls, 1.0, 0.1, orc.RBF, max_iter=400, tol=1e-6)
    alone = egp.mbcg(Xd, _cuda(b), ls, 1.0, 0.1, orc.RBF, max_iter=400, tol=1e-6)
    u1, u2 = both["U"].cpu().numpy()[:, 0], alone["U"].cpu().numpy()[:, 0]
    assert np.linalg.norm(u1 - u2) <= 1e-3 * np.linalg.norm(u1)


def test_mbcg_slq_logdet_from_gpu_coefficients(egp):
    """The tridiagonals built from the GPU's CG coefficients give the log-determinant within Monte-Carlo
    error (probes with covariance P built on the host from Rademacher draws)."""
    n, d, tp, rank = 2000, 3, 32, 10
    rng = np.random.default_rng(12)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    ls = np.full(d, 0.3, np.float32)
    s, noise, kind = 1.0, 0.1, orc.RBF
    h = orc.Hyper(kind, ls, s, noise)
    Xd = _cuda(X)
    P = egp.piv_chol_precond(Xd, ls, s, noise, kind, rank)
    Lg = P.L.cpu().numpy().astype(np.float64).T
    Z = orc.probes_with_cov_P(Lg, noise, rademacher(rng, (rank, tp)), rademacher(rng, (n, tp))).astype(np.float32)
    res = egp.mbcg(Xd, _cuda(Z), ls, s, noise, kind, precond=P, max_iter=60, tol=1e-5)
    terms = []
    for c in range(tp):
        T = orc.tridiag_from_cg(res["alphas"][:, c], res["betas"][:-1, c])
        terms.append(res["gamma0"][c] * orc.slq_quadrature(T))
    terms = np.array(terms)
    est = P.logdet + terms.mean()
    exact = orc.logdet(orc.khat(X, h))
    assert abs(est - exact) <= 4 * terms.std(ddof=1) / np.sqrt(tp) + 1e-3 * abs(exact)


@pytest.mark.parametrize("t", [16, 17, 1, 32, 33])
def test_mbcg_with_symmetric_kernels(egp, t):
    """The solver at a size where the default mode runs the symmetric kernels (column-major state): same iterates as
    with the one-sided kernels up to summation order, a true residual (rows computed exactly by the oracle) at the
    level the recurrence reports, and the same bits when the solve is repeated."""
    n, d = 33000, 11
    rng = np.random.default_rng(77 + t)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    B = rademacher(rng, (n, t))
    B[:, 0] = np.sin(4 * X[:, 0]) + 0.1 * rng.standard_normal(n)
    ls = np.exp(rng.uniform(np.log(0.3), np.log(1.5), d)).astype(np.float32)
    s, noise, kind = 1.0, 0.5, orc.RBF
    Xd, Bd = _cuda(X), _cuda(B)
    P = egp.piv_chol_precond(Xd, ls, s, noise, kind, 50)
    res = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=P, max_iter=200, tol=1e-3)
    L = egp.lib()
    try:
        L.egp_set_kmm_mode(3)      # one-sided kernels
        base = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=P, max_iter=200, tol=1e-3)
    finally:
        L.egp_set_kmm_mode(0)
    assert res["rel_resid"].max() <= 1e-3
    assert abs(res["iters"] - base["iters"]) <= 2
    # the column-side sums are order-independent: the whole solve repeats bit for bit
    res2 = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=P, max_iter=200, tol=1e-3)
    assert res2["iters"] == res["iters"] and bool((res2["U"] == res["U"]).all())
    U = res["U"].cpu().numpy().astype(np.float64)
    Ub = base["U"].cpu().numpy().astype(np.float64)
    assert np.linalg.norm(U - Ub) / np.linalg.norm(Ub) <= 5e-3
    rows = rng.choice(n, 96, replace=False)
    KU = orc.kmm_rows(X, U, orc.Hyper(kind, ls, s, noise), rows)
    true_res = np.linalg.norm(KU - B[rows], axis=0) / np.linalg.norm(B[rows], axis=0)
    assert true_res.max() <= 5e-3


@pytest.mark.parametrize("mode", ["fp32", "fp32_one_sided"])
def test_lanczos_three_term_recurrence_at_size(egp, mode):
    """Lanczos (single vector) and block Lanczos at a size where the symmetric kernels run: the basis is orthonormal
    and Khat q_j = beta_{j-1} q_{j-1} + alpha_j q_j + beta_j q_{j+1} holds on rows of Khat Q^T computed exactly by the
    oracle; the block variant's projected matrix equals Q Khat Q^T on sampled-row evidence (Khat Q^T rows against
    (T Q)^T rows for the interior blocks)."""
    n, d, r = 33000, 3, 10
    rng = np.random.default_rng(321)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    y = (np.sin(6 * X[:, 0]) + X[:, 1] ** 2 + 0.1 * rng.standard_normal(n)).astype(np.float32)
    ls = np.array([0.3, 0.5, 0.9], np.float32)
    s, noise, kind = 1.3, 0.1, orc.MATERN52
    h = orc.Hyper(kind, ls, s, noise)
    rows = rng.choice(n, 96, replace=False)
    try:
        egp.set_kmm_mode(mode)
        c = egp.lanczos(_cuda(X), _cuda(y), ls, s, noise, kind, r)
        B0 = np.concatenate([y[:, None], rademacher(rng, (n, 15))], axis=1)
        bc = egp.block_lanczos(_cuda(X), _cuda(B0), ls, s, noise, kind, 3)
    finally:
        egp.set_kmm_mode("fp32")
    assert c.steps == r
    Q = c.Q.cpu().numpy().astype(np.float64)
    assert np.abs(Q @ Q.T - np.eye(r)).max() <= 5e-5
    KQ = orc.kmm_rows(X, Q.T.astype(np.float32), h, rows)          # (rows, r)
    scale = np.abs(c.alpha).max()
    for j in range(r - 1):
        rhs = c.alpha[j] * Q[j, rows] + c.beta[j] * Q[j + 1, rows]
        if j > 0:
            rhs = rhs + c.beta[j - 1] * Q[j - 1, rows]
        assert np.linalg.norm(KQ[:, j] - rhs) <= 2e-4 * scale * np.linalg.norm(Q[j, rows]) + 1e-7, j
    # block variant: Khat Q_b^T lies in the span of blocks b-1, b, b+1 with coefficients T
    m = bc.steps
    assert m == 48
    Qb = bc.Q.cpu().numpy().astype(np.float64)
    assert np.abs(Qb @ Qb.T - np.eye(m)).max() <= 5e-5
    KQb = orc.kmm_rows(X, Qb.T.astype(np.float32), h, rows)        # (rows, m)
    T = np.asarray(bc.T, dtype=np.float64)
    assert np.abs(T - T.T).max() <= 1e-4 * np.abs(T).max()
    recon = Qb[:, rows].T @ T                                      # (rows, m): sum_i Q[i, row] T[i, j]
    inner = slice(0, 32)                                           # blocks whose successor is in the basis
    assert np.linalg.norm(KQb[:, inner] - recon[:, inner]) <= 3e-4 * np.abs(T).max() * np.linalg.norm(Qb[:32, rows])


@pytest.mark.parametrize("n,t", [(3000, 17), (3000, 9), (33000, 17)])
def test_mbcg_shrink_drops_converged_trailing_columns(egp, n, t):
    """With the shrink switch, trailing columns leave the iteration once they have met the tolerance. B = [y | probes]
    with a smooth y in front. Every column keeps a valid
    solution (true residual at tolerance level: dense oracle at the small size, oracle rows at the large one) and takes
    the same steps as without the switch."""
    d = 3
    rng = np.random.default_rng(50 + n + t)
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    B = rademacher(rng, (n, t))
    B[:, 0] = np.sin(3 * X[:, 0]) + np.cos(2 * X[:, 1])
    ls = np.array([0.25, 0.3, 0.4], np.float32)
    s, noise, kind, tol = 1.0, 0.05, orc.RBF, 1e-2
    Xd, Bd = _cuda(X), _cuda(B)
    P = egp.piv_chol_precond(Xd, ls, s, noise, kind, 20)
    full = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=P, max_iter=400, tol=tol)
    res = egp.mbcg(Xd, Bd, ls, s, noise, kind, precond=P, max_iter=400, tol=tol, shrink=True)
    assert egp.lib().egp_get_mbcg_shrink() == 0                      # the switch is back off
    assert np.array_equal(full["col_iters"], np.full(t, full["iters"]))
    ci = res["col_iters"]
    print(f"n={n} t={t}: {full['iters']} iterations without shrink; with it {res['iters']}, per column {ci.tolist()}")
    assert res["iters"] <= full["iters"] and ci[0] == res["iters"]
    assert np.all(np.diff(ci) <= 0)                                  # a column leaves only after all those behind it
    assert ci[-1] < res["iters"]                                     # and some did leave early
    assert np.all(res["rel_resid"] <= tol)
    first = ci[-1]      # until the first column leaves both runs launch the same kernels: identical bits
    assert np.array_equal(res["alphas"][:first], full["alphas"][:first])
    for c in range(t):
        m = ci[c]
        # afterwards the multiply runs on fewer columns (other launch shapes, other summation order) and the
        # coefficients drift apart the way CG coefficients do in fp32; the first steps after the change still agree
        k = min(m, first + 3)
        assert np.allclose(res["alphas"][:k, c], full["alphas"][:k, c], rtol=1e-3), c
        assert np.all(res["alphas"][m:, c] == 0.0) and np.all(res["betas"][m:, c] == 0.0)
    U = res["U"].cpu().numpy().astype(np.float64)
    h = orc.Hyper(kind, ls, s, noise)
    if n <= 4000:
        KU = orc.khat(X, h) @ U
        true_res = np.linalg.norm(KU - B, axis=0) / np.linalg.norm(B, axis=0)
    else:
        rows = rng.choice(n, 128, replace=False)
        KU = orc.kmm_rows(X, U.astype(np.float32), h, rows)
        true_res = np.linalg.norm(KU - B[rows], axis=0) / np.linalg.norm(B[rows], axis=0)
    assert true_res.max() <= (1.3 if n <= 4000 else 2.0) * tol


def test_mbcg_without_iterations_reports_the_start_residual(egp):
    """max_iter = 0: no iteration runs, U = 0, and the relative residual of the start vector is 1 for every column with
    b != 0 (0 for a zero column)."""
    rng = np.random.default_rng(40)
    n, d = 700, 3
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    B = rng.standard_normal((n, 4)).astype(np.float32)
    B[:, 2] = 0.0
    res = egp.mbcg(_cuda(X), _cuda(B), np.full(d, 0.5, np.float32), 1.0, 0.1, orc.RBF, max_iter=0, tol=0.5)
    assert res["iters"] == 0
    assert res["rel_resid"].tolist() == [1.0, 1.0, 0.0, 1.0]
    assert float(res["U"].abs().max()) == 0.0
