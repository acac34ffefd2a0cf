"""Plain, slow, dense fp64 implementation of what the exact-GP hot path computes.

TEST INFRASTRUCTURE: the oracle the HIP path is compared against. It shares no
code, constants or helpers with the HIP path.

The paper's method reaches the dense result exactly (it is "exact GP inference
without approximations", Method section): the kernel matrix is only ever used
through products with it, so the oracle is the textbook definition written out:
materialise K, multiply, Cholesky-solve, exact log-determinant (Background,
"The Cholesky decomposition"). Where the outcome is an algorithm's output rather
than a closed form (pivot order, CG coefficients, Lanczos tridiagonals) the
oracle runs the textbook algorithm step by step on the dense matrix.

The paper names the kernels (RBF, Matern; Background and Experiment details) and
cites the modified PCG, pivoted-Cholesky preconditioner and stochastic
log-determinant without stating them; the forms used here are the standard ones
(Rasmussen & Williams ch. 4 for the kernels, Matern-1/2 = exp(-r) included; Golub & Van Loan for PCG and for
diagonal-pivoted Cholesky; the CG<->Lanczos identity and Gauss quadrature for
the log-determinant).

Pins (tests/test_oracle_*.py, CPU only): closed-form kernel values, brute-force
scalar loops, symmetry/PSD, limits of the lengthscale, finite differences,
LAPACK dpstrf pivots, greedy Schur-complement pivots, CG vs Cholesky, finite
termination, the CG tridiagonal against explicit Lanczos at truncations, exact
Gauss quadrature at m=n Lanczos steps, stochastic estimators exact for complete
(Hadamard) probe sets and within Monte-Carlo error for random ones, Adam's
second step against the published recurrences. No function here is "parity
unpinned".

All functions take array-likes, cast to float64, and return float64.
"""
from __future__ import annotations

import numpy as np
import scipy.linalg as sla

RBF, MATERN32, MATERN52, MATERN12 = 0, 1, 2, 3

__all__ = [
    "RBF", "MATERN32", "MATERN52", "MATERN12", "Hyper", "sq_dist", "kernel_matrix", "khat", "kmm",
    "kmm_rows", "dkernel_dlengthscale", "kmm_grad", "kmm_grad_rows", "chol_solve", "logdet",
    "mll", "mll_grad", "pivoted_cholesky", "precond_matrix", "precond_solve", "precond_logdet",
    "pcg", "tridiag_from_cg", "slq_quadrature", "slq_logdet", "probes_with_cov_P",
    "mll_stochastic_terms", "predict_exact", "lanczos", "predict_var_lanczos", "block_lanczos",
    "predict_var_galerkin", "train_adam",
]


class Hyper:
    """Kernel hyper-parameters: k(x,x') = outputscale * g(r), r^2 = sum_k (x_k-x'_k)^2 / l_k^2,
    and Khat = K + noise * I (Background, Notation: noise is sigma^2, the diagonal addend)."""

    def __init__(self, kernel_type, lengthscales, outputscale=1.0, noise=0.0):
        self.kernel_type = int(kernel_type)
        self.lengthscales = np.asarray(lengthscales, dtype=np.float64).reshape(-1)
        self.outputscale = float(outputscale)
        self.noise = float(noise)


def sq_dist(X, Z, lengthscales):
    """r^2[i,j] = sum_k ((X[i,k]-Z[j,k])/l_k)^2 by direct differences (no norm expansion)."""
    X = np.asarray(X, np.float64)
    Z = np.asarray(Z, np.float64)
    ls = np.asarray(lengthscales, np.float64)
    out = np.zeros((X.shape[0], Z.shape[0]))
    for k in range(X.shape[1]):
        diff = (X[:, k][:, None] - Z[:, k][None, :]) / ls[k]
        out += diff * diff
    return out


def _g(r2, kernel_type):
    """Stationary correlation g(r) as a function of r^2."""
    if kernel_type == RBF:
        return np.exp(-0.5 * r2)
    r = np.sqrt(r2)
    if kernel_type == MATERN32:
        a = np.sqrt(3.0) * r
        return (1.0 + a) * np.exp(-a)
    if kernel_type == MATERN52:
        a = np.sqrt(5.0) * r
        return (1.0 + a + a * a / 3.0) * np.exp(-a)
    if kernel_type == MATERN12:
        return np.exp(-r)
    raise ValueError("unknown kernel type")


def _h(r2, kernel_type):
    """h(r) with d g / d l_k = h(r) * (x_k - x'_k)^2 / l_k^3 (chain rule; for RBF and Matern-3/2, 5/2 r cancels, so
    r=0 is regular; Matern-1/2 keeps a 1/r)."""
    if kernel_type == RBF:
        return np.exp(-0.5 * r2)
    r = np.sqrt(r2)
    if kernel_type == MATERN32:
        return 3.0 * np.exp(-np.sqrt(3.0) * r)
    if kernel_type == MATERN52:
        a = np.sqrt(5.0) * r
        return (5.0 / 3.0) * (1.0 + a) * np.exp(-a)
    if kernel_type == MATERN12:
        # g = exp(-r): d g / d l_k = exp(-r) (x_k - x'_k)^2 / (r l_k^3); at r = 0 the squared difference is 0 too
        # and the entry (a point against itself) does not depend on the lengthscales: 0
        safe = np.where(r > 0.0, r, 1.0)
        return np.where(r > 0.0, np.exp(-r) / safe, 0.0)
    raise ValueError("unknown kernel type")


def kernel_matrix(X, Z, hyper: Hyper):
    """K[i,j] = s * g(r_ij) between the rows of X and the rows of Z (noise-free)."""
    return hyper.outputscale * _g(sq_dist(X, Z, hyper.lengthscales), hyper.kernel_type)


def khat(X, hyper: Hyper):
    """Khat = K(X,X) + sigma^2 I (Background, Notation)."""
    K = kernel_matrix(X, X, hyper)
    K[np.diag_indices_from(K)] += hyper.noise
    return K


def kmm(X, V, hyper: Hyper):
    """Khat @ V with K materialised: the 'full GP setting' product the partitioned MVM must equal
    (Method, 'O(n) memory MVM-based inference' and 'Partitioned kernel MVMs')."""
    return khat(X, hyper) @ np.asarray(V, np.float64)


def kmm_rows(X, V, hyper: Hyper, rows):
    """Selected rows of Khat @ V, each computed exactly: one row partition of the partitioned MVM
    (Method, 'Partitioned kernel MVMs') with the partition being `rows`."""
    X = np.asarray(X, np.float64)
    V = np.asarray(V, np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    out = kernel_matrix(X[rows], X, hyper) @ V
    out += hyper.noise * V[rows]
    return out


def dkernel_dlengthscale(X, Z, hyper: Hyper, k):
    """dK/dl_k [i,j] = s * h(r_ij) * (X[i,k]-Z[j,k])^2 / l_k^3."""
    X = np.asarray(X, np.float64)
    Z = np.asarray(Z, np.float64)
    r2 = sq_dist(X, Z, hyper.lengthscales)
    delta = X[:, k][:, None] - Z[:, k][None, :]
    return hyper.outputscale * _h(r2, hyper.kernel_type) * delta * delta / hyper.lengthscales[k] ** 3


def kmm_grad(X, V, hyper: Hyper):
    """Stack over k of (dK/dl_k) @ V, shape (d, n, t): the products the gradient (Eq. 2) needs."""
    V = np.asarray(V, np.float64)
    return np.stack([dkernel_dlengthscale(X, X, hyper, k) @ V for k in range(len(hyper.lengthscales))])


def kmm_grad_rows(X, V, hyper: Hyper, rows):
    X = np.asarray(X, np.float64)
    V = np.asarray(V, np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    return np.stack([dkernel_dlengthscale(X[rows], X, hyper, k) @ V
                     for k in range(len(hyper.lengthscales))])


def chol_solve(Khat, B):
    """Khat^{-1} B through the Cholesky factor (Background, 'The Cholesky decomposition')."""
    c = sla.cho_factor(np.asarray(Khat, np.float64), lower=True)
    return sla.cho_solve(c, np.asarray(B, np.float64))


def logdet(Khat):
    """log|Khat| = 2 sum log diag(chol(Khat))."""
    L = np.linalg.cholesky(np.asarray(Khat, np.float64))
    return 2.0 * np.log(np.diag(L)).sum()


def mll(X, y, hyper: Hyper):
    """Log marginal likelihood, Eq. 1 with the constants the proportionality sign drops:
    L = -1/2 y^T Khat^{-1} y - 1/2 log|Khat| - n/2 log(2 pi) (zero prior mean)."""
    y = np.asarray(y, np.float64)
    Kh = khat(X, hyper)
    u = chol_solve(Kh, y)
    return -0.5 * y @ u - 0.5 * logdet(Kh) - 0.5 * len(y) * np.log(2.0 * np.pi)


def mll_grad(X, y, hyper: Hyper):
    """Gradient of Eq. 1 w.r.t. (l_1..l_d, outputscale, noise):
    dL/dtheta = 1/2 u^T (dKhat/dtheta) u - 1/2 tr(Khat^{-1} dKhat/dtheta), u = Khat^{-1} y.
    (Eq. 2 as printed is inconsistent; this is the standard identity, pinned by finite
    differences of mll in the tests.)"""
    y = np.asarray(y, np.float64)
    X = np.asarray(X, np.float64)
    Kh = khat(X, hyper)
    Kinv = chol_solve(Kh, np.eye(len(y)))
    u = Kinv @ y
    d = len(hyper.lengthscales)
    grads = np.zeros(d + 2)
    for k in range(d + 2):
        if k < d:
            dK = dkernel_dlengthscale(X, X, hyper, k)
        elif k == d:
            dK = kernel_matrix(X, X, hyper) / hyper.outputscale
        else:
            dK = np.eye(len(y))
        grads[k] = 0.5 * u @ dK @ u - 0.5 * np.sum(Kinv * dK)
    return grads


def pivoted_cholesky(K, rank, tol_abs=0.0):
    """Partial Cholesky of the noise-free K with diagonal pivoting (Method, 'Preconditioning':
    a rank-k factor from k kernel rows). Greedy: at each step take the largest remaining
    residual diagonal (ties -> lowest index), form that row of the residual, scale.
    Returns (L of shape (n, steps) in original row order, pivots)."""
    K = np.asarray(K, np.float64)
    n = K.shape[0]
    diag = np.diag(K).copy()
    L = np.zeros((n, rank))
    pivots = []
    chosen = np.zeros(n, dtype=bool)
    for m in range(rank):
        masked = np.where(chosen, -np.inf, diag)
        piv = int(np.argmax(masked))          # first occurrence of the maximum
        if not masked[piv] > tol_abs:
            break
        root = np.sqrt(diag[piv])
        col = (K[piv, :] - L[:, :m] @ L[piv, :m]) / root
        col[chosen] = 0.0
        col[piv] = root
        L[:, m] = col
        chosen[piv] = True
        pivots.append(piv)
        diag = diag - col * col
        diag[chosen] = 0.0
    steps = len(pivots)
    return L[:, :steps], np.asarray(pivots, dtype=np.int64)


def precond_matrix(L, noise):
    """P = L L^T + sigma^2 I, dense."""
    L = np.asarray(L, np.float64)
    return L @ L.T + noise * np.eye(L.shape[0])


def precond_solve(L, noise, R):
    """P^{-1} R by a dense solve (no Woodbury here on purpose)."""
    return np.linalg.solve(precond_matrix(L, noise), np.asarray(R, np.float64))


def precond_logdet(L, noise):
    sign, val = np.linalg.slogdet(precond_matrix(L, noise))
    assert sign > 0
    return val


def pcg(Khat, b, Pinv=None, max_iter=100, tol=0.0):
    """Textbook preconditioned CG on one right-hand side b (Background, 'Conjugate gradients';
    Method: four vectors u, r, p, z). Stopping rule: relative residual ||r||/||b|| <= tol,
    tested after each completed iteration. Returns dict with u, alphas, betas, rel residual
    history (entry j = after iteration j+1) and gamma0 = r0^T P^{-1} r0."""
    Khat = np.asarray(Khat, np.float64)
    b = np.asarray(b, np.float64)
    apply_P = (lambda r: r.copy()) if Pinv is None else (lambda r: Pinv @ r)
    u = np.zeros_like(b)
    r = b.copy()
    z = apply_P(r)
    p = z.copy()
    gamma = r @ z
    gamma0 = gamma
    bnorm = np.linalg.norm(b)
    alphas, betas, hist = [], [], []
    for _ in range(max_iter):
        w = Khat @ p
        alpha = gamma / (p @ w)
        u = u + alpha * p
        r = r - alpha * w
        alphas.append(alpha)
        hist.append(np.linalg.norm(r) / bnorm)
        if hist[-1] <= tol:
            break
        z = apply_P(r)
        gamma_new = r @ z
        beta = gamma_new / gamma
        betas.append(beta)
        p = z + beta * p
        gamma = gamma_new
    return {"u": u, "alphas": np.array(alphas), "betas": np.array(betas),
            "rel_resid": np.array(hist), "gamma0": gamma0}


def tridiag_from_cg(alphas, betas):
    """Lanczos tridiagonal of the preconditioned operator from CG coefficients:
    T[j,j] = 1/alpha_j + beta_{j-1}/alpha_{j-1}; T[j,j+1] = sqrt(beta_j)/alpha_j."""
    m = len(alphas)
    T = np.zeros((m, m))
    for j in range(m):
        T[j, j] = 1.0 / alphas[j] + (betas[j - 1] / alphas[j - 1] if j > 0 else 0.0)
        if j + 1 < m:
            T[j, j + 1] = T[j + 1, j] = np.sqrt(betas[j]) / alphas[j]
    return T


def slq_quadrature(T):
    """e_1^T log(T) e_1 by symmetric eigendecomposition (Gauss quadrature rule of the Lanczos process)."""
    lam, Q = np.linalg.eigh(T)
    return float(np.sum(Q[0, :] ** 2 * np.log(lam)))


def probes_with_cov_P(L, noise, w1, w2):
    """Probe vectors with covariance P = L L^T + sigma^2 I from Rademacher draws:
    z = L w1 + sigma w2, w1 of shape (k, t_p), w2 of shape (n, t_p)."""
    return np.asarray(L, np.float64) @ np.asarray(w1, np.float64) + np.sqrt(noise) * np.asarray(w2, np.float64)


def slq_logdet(Khat, Z, L=None, noise=None, max_iter=None):
    """Stochastic Lanczos estimate log|Khat| ~= log|P| + mean_c gamma0_c * e1^T log(T_c) e1, with probe
    columns Z of covariance P (identity when L is None) and T_c from PCG on z_c.
    Returns (estimate, per-probe terms)."""
    Khat = np.asarray(Khat, np.float64)
    Z = np.asarray(Z, np.float64)
    n = Khat.shape[0]
    if L is None:
        Pinv, ldP = None, 0.0
    else:
        Pinv = np.linalg.inv(precond_matrix(L, noise))
        ldP = precond_logdet(L, noise)
    max_iter = max_iter or n
    terms = []
    for c in range(Z.shape[1]):
        res = pcg(Khat, Z[:, c], Pinv, max_iter=max_iter, tol=1e-14)
        T = tridiag_from_cg(res["alphas"], res["betas"])
        terms.append(res["gamma0"] * slq_quadrature(T))
    terms = np.array(terms)
    return ldP + terms.mean(), terms


def mll_stochastic_terms(X, y, hyper: Hyper, Z, L=None, max_iter=None):
    """The three quantities modified PCG delivers in one batched solve (Background, last paragraph):
    u = Khat^{-1} y, the log-determinant estimate, and the probe estimate of tr(Khat^{-1} dKhat/dtheta)
    for theta = (l_1..l_d, outputscale, noise): mean_c (Khat^{-1} z_c)^T (dKhat/dtheta) (P^{-1} z_c)."""
    X = np.asarray(X, np.float64)
    y = np.asarray(y, np.float64)
    Z = np.asarray(Z, np.float64)
    Kh = khat(X, hyper)
    n = len(y)
    u = chol_solve(Kh, y)
    ld, _ = slq_logdet(Kh, Z, L, hyper.noise, max_iter)
    KinvZ = chol_solve(Kh, Z)
    PinvZ = Z if L is None else precond_solve(L, hyper.noise, Z)
    d = len(hyper.lengthscales)
    traces = np.zeros(d + 2)
    quad = np.zeros(d + 2)
    for k in range(d + 2):
        if k < d:
            dK = dkernel_dlengthscale(X, X, hyper, k)
        elif k == d:
            dK = kernel_matrix(X, X, hyper) / hyper.outputscale
        else:
            dK = np.eye(n)
        traces[k] = np.mean(np.sum(KinvZ * (dK @ PinvZ), axis=0))
        quad[k] = u @ dK @ u
    value = -0.5 * y @ u - 0.5 * ld - 0.5 * n * np.log(2.0 * np.pi)
    grad = 0.5 * quad - 0.5 * traces
    return {"u": u, "logdet": ld, "mll": value, "grad": grad, "trace": traces, "quad": quad}


def predict_exact(X, y, Xq, hyper: Hyper):
    """Predictive moments of the latent function at the rows of Xq with zero prior mean (predictive mean and
    variance equations of the Background section), by dense Cholesky:
    mean = K(Xq,X) Khat^{-1} y,  var = k(xq,xq) - k_q^T Khat^{-1} k_q."""
    X = np.asarray(X, np.float64)
    Xq = np.asarray(Xq, np.float64)
    Kh = khat(X, hyper)
    Kq = kernel_matrix(Xq, X, hyper)
    mean = Kq @ chol_solve(Kh, np.asarray(y, np.float64))
    var = hyper.outputscale - np.sum(Kq * chol_solve(Kh, Kq.T).T, axis=1)
    return mean, var


def lanczos(Khat, b, r):
    """Textbook Lanczos process on the symmetric matrix Khat from start vector b, with full
    re-orthogonalisation (two Gram-Schmidt passes per step). Returns Q (steps x n, orthonormal rows),
    alpha (steps), beta (steps-1): T = Q Khat Q^T is tridiagonal with these entries."""
    Khat = np.asarray(Khat, np.float64)
    b = np.asarray(b, np.float64)
    n = len(b)
    Q = np.zeros((r, n))
    alpha, beta = [], []
    Q[0] = b / np.linalg.norm(b)
    for j in range(r):
        w = Khat @ Q[j]
        alpha.append(Q[j] @ w)
        if j + 1 == r:
            break
        for _ in range(2):
            w = w - Q[:j + 1].T @ (Q[:j + 1] @ w)
        bj = np.linalg.norm(w)
        if not bj > 1e-12 * (abs(alpha[0]) + (beta[0] if beta else bj)):
            break
        beta.append(bj)
        Q[j + 1] = w / bj
    m = len(alpha)
    return Q[:m], np.array(alpha), np.array(beta[:m - 1])


def predict_var_lanczos(Kq, Q, alpha, beta, outputscale):
    """Cached predictive variance: s - g^T T^{-1} g with g = Q k_q, T = tridiag(alpha, beta): the Galerkin
    approximation Q^T T^{-1} Q of Khat^{-1} on the Krylov space spanned by the rows of Q. Kq is K(Xq, X)."""
    m = len(alpha)
    T = np.diag(alpha) + (np.diag(beta, 1) + np.diag(beta, -1) if m > 1 else 0.0)
    G = np.asarray(Kq, np.float64) @ np.asarray(Q, np.float64).T
    return outputscale - np.sum(G * np.linalg.solve(T, G.T).T, axis=1)


def block_lanczos(Khat, B0, m):
    """Orthonormal basis of the block Krylov space span{B0, Khat B0, .., Khat^(m-1) B0} and the projected matrix.

    The variance cache only needs an orthonormal Q and T = Q Khat Q^T (the Galerkin approximation Q^T T^{-1} Q of
    Khat^{-1}, never above Khat^{-1}); a block of b start vectors makes every multiply with Khat carry b columns.
    Plain block Gram-Schmidt: W = Khat Q_j, two projection passes against all earlier vectors, thin QR of the
    remainder gives Q_{j+1}. Stops when a remainder loses rank. Returns Q (r x n, orthonormal rows) and T (r x r),
    which is block tridiagonal up to rounding (it is formed as Q Khat Q^T, not assumed)."""
    Khat = np.asarray(Khat, np.float64)
    B0 = np.asarray(B0, np.float64)
    if B0.ndim == 1:
        B0 = B0[:, None]
    Qb, R0 = np.linalg.qr(B0)
    if np.min(np.abs(np.diag(R0))) <= 1e-12 * np.max(np.abs(np.diag(R0))):
        raise ValueError("start block is rank deficient")
    blocks = [Qb]
    for _ in range(m - 1):
        W = Khat @ blocks[-1]
        Qall = np.concatenate(blocks, axis=1)
        for _ in range(2):
            W = W - Qall @ (Qall.T @ W)
        Qn, Rn = np.linalg.qr(W)
        dr = np.abs(np.diag(Rn))
        if np.min(dr) <= 1e-10 * np.linalg.norm(Khat @ blocks[-1]):
            break
        blocks.append(Qn)
    Q = np.concatenate(blocks, axis=1).T
    T = Q @ Khat @ Q.T
    return Q, 0.5 * (T + T.T)


def predict_var_galerkin(Kq, Q, T, outputscale):
    """Cached predictive variance s - g^T T^{-1} g, g = Q k_q, for any orthonormal Q with T = Q Khat Q^T."""
    G = np.asarray(Kq, np.float64) @ np.asarray(Q, np.float64).T
    return outputscale - np.sum(G * np.linalg.solve(np.asarray(T, np.float64), G.T).T, axis=1)


def train_adam(X, y, hyper: Hyper, steps, lr=0.1, noise_floor=0.0, rank=0, W1=None, W2=None,
               beta1=0.9, beta2=0.999, eps=1e-8):
    """Adam ascent on L / n in log-parameters phi = (log l_k, log s, log(noise - floor)) (Experiment details:
    Adam, step size 0.1, noise kept above a floor). With W2 given, value and gradient are the stochastic
    estimates of mll_stochastic_terms with probes of covariance P built from the Rademacher draws W1, W2 and a
    rank-`rank` pivoted Cholesky recomputed at every step; with W2 = None they are the exact dense ones.
    Returns (final Hyper, list of L before each step and at the end)."""
    X = np.asarray(X, np.float64)
    y = np.asarray(y, np.float64)
    d = len(hyper.lengthscales)
    n = len(y)
    phi = np.concatenate([np.log(hyper.lengthscales), [np.log(hyper.outputscale)],
                          [np.log(max(hyper.noise - noise_floor, 1e-4 * (noise_floor if noise_floor > 0 else 1.0)))]])
    m = np.zeros(d + 2)
    v = np.zeros(d + 2)
    history = []

    def current():
        return Hyper(hyper.kernel_type, np.exp(phi[:d]), np.exp(phi[d]), noise_floor + np.exp(phi[d + 1]))

    def evaluate(h):
        if W2 is None:
            return mll(X, y, h), mll_grad(X, y, h)
        if rank > 0:
            L, _ = pivoted_cholesky(kernel_matrix(X, X, h), rank)
            Z = probes_with_cov_P(L, h.noise, W1, W2)
        else:
            L, Z = None, np.asarray(W2, np.float64)
        out = mll_stochastic_terms(X, y, h, Z, L)
        return out["mll"], out["grad"]

    for step in range(steps + 1):
        h = current()
        value, grad = evaluate(h)
        history.append(value)
        if step == steps:
            break
        theta = np.concatenate([h.lengthscales, [h.outputscale], [np.exp(phi[d + 1])]])
        g = theta * grad / n
        m = beta1 * m + (1 - beta1) * g
        v = beta2 * v + (1 - beta2) * g * g
        phi = phi + lr * (m / (1 - beta1 ** (step + 1))) / (np.sqrt(v / (1 - beta2 ** (step + 1))) + eps)
    return current(), history
