"""Parity of the fused derivative products (dK/dl_k) V with the dense fp64 oracle."""
import numpy as np
import pytest

import oracle as orc
from workloads import make_workload

pytestmark = pytest.mark.gpu

# same arithmetic as the KMM (fp32 MFMA, fp32 transform): same 1e-4 relative Frobenius bound per lengthscale
GRAD_TOL = 1e-4


@pytest.fixture(scope="module")
def egp():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1903_08114_amd as egp
    egp.lib()
    return egp


def _run(egp, X, V, ls, s, noise, kind):
    import torch
    out = egp.kmm_grad(torch.from_numpy(X).cuda(), torch.from_numpy(V).cuda(), ls, s, noise, kind)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,t", [(1, 1, 1), (33, 3, 2), (500, 8, 16), (1030, 11, 17), (700, 25, 16),
                                   (300, 14, 5), (257, 27, 33), (1300, 31, 4)])
def test_kmm_grad_shapes(egp, kind, n, d, t):
    rng = np.random.default_rng(31 * n + 7 * d + t + kind)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.5), np.log(3.0), d)).astype(np.float32)
    s, noise = 1.4, 0.1
    got = _run(egp, X, V, ls, s, noise, kind)
    ref = orc.kmm_grad(X, V, orc.Hyper(kind, ls, s, noise))
    assert got.shape == ref.shape == (d, n, t)
    assert np.isfinite(got).all()
    for k in range(d):
        denom = np.linalg.norm(ref[k])
        if denom == 0:
            assert np.abs(got[k]).max() == 0
        else:
            assert np.linalg.norm(got[k] - ref[k]) / denom <= GRAD_TOL, k


def test_kmm_grad_c3_recipe_rows(egp):
    """C3 recipe (d = 25, RBF, 16 Gaussian columns) at reduced n, big enough for the unsplit launch shape;
    sampled rows computed exactly by the oracle."""
    w = make_workload("C3", n=140000)
    got = _run(egp, w.X, w.V, w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    rows = np.random.default_rng(5).choice(w.n, 48, replace=False)
    rows[:2] = [0, w.n - 1]
    ref = orc.kmm_grad_rows(w.X, w.V, orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise), rows)
    for k in range(w.d):
        assert np.linalg.norm(got[k][rows] - ref[k]) / np.linalg.norm(ref[k]) <= GRAD_TOL, k


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,t", [(1, 1, 1), (50, 2, 3), (700, 3, 17), (1500, 11, 17), (900, 18, 16), (400, 25, 5),
                                   (300, 31, 33)])
def test_bilinear_forms_match_oracle(egp, kind, n, d, t):
    """sum_c w_c a_c^T (dK/dl_k) b_c and the outputscale form against the dense oracle. The bound is the one
    the KMM tolerance implies through Cauchy-Schwarz: 1e-4 * ||A diag(w)||_F * ||(dK/dl_k) B||_F."""
    import torch
    rng = np.random.default_rng(17 * n + 3 * d + t + kind)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    A = rng.standard_normal((n, t)).astype(np.float32)
    B = rng.standard_normal((n, t)).astype(np.float32)
    wts = rng.uniform(-1, 1, t).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.5), np.log(3.0), d)).astype(np.float32)
    s, noise = 1.3, 0.1
    h = orc.Hyper(kind, ls, s, noise)
    got = egp.kmm_grad_bilinear(torch.from_numpy(X).cuda(), torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(),
                                ls, s, noise, kind, weights=wts)
    Aw = A.astype(np.float64) * wts.astype(np.float64)
    dKB = orc.kmm_grad(X, B, h)
    for k in range(d):
        ref = np.sum(Aw * dKB[k])
        bound = GRAD_TOL * np.linalg.norm(Aw) * np.linalg.norm(dKB[k])
        assert abs(got[k] - ref) <= bound + 1e-12, (k, got[k], ref, bound)
    KB = orc.kernel_matrix(X, X, h) @ B.astype(np.float64) / s
    ref = np.sum(Aw * KB)
    assert abs(got[d] - ref) <= GRAD_TOL * np.linalg.norm(Aw) * np.linalg.norm(KB) + 1e-12
    # unweighted call == weights of one
    if t <= 5:
        ones = egp.kmm_grad_bilinear(torch.from_numpy(X).cuda(), torch.from_numpy(A).cuda(),
                                     torch.from_numpy(B).cuda(), ls, s, noise, kind)
        for k in range(d):
            assert abs(ones[k] - np.sum(A.astype(np.float64) * dKB[k])) <= \
                GRAD_TOL * np.linalg.norm(A) * np.linalg.norm(dKB[k]) + 1e-12
