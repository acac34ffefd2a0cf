"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: sampled output rows that the
oracle computes exactly one by one (K cannot be materialised at these sizes)."""
import numpy as np
import pytest

import oracle as orc
from workloads import make_workload

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


def _rows(n, m, seed):
    rows = np.random.default_rng(seed).choice(n, m, replace=False)
    rows[:2] = [0, n - 1]
    return rows


def _rel(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


# Worst single entry on the sampled rows, relative to the root-mean-square entry of the reference: the distance
# step's rounding (2^-24 times the largest squared norm of the scaled points) puts it at a few 1e-6 for the
# lengthscales of these configurations; the bound leaves a factor of about ten.
MAX_ENTRY_TOL = 3e-5


# The derivative product sums n terms per output in one fp32 accumulator (no second accumulation level): its worst
# entry carries about 2^-24 sqrt(n) of the sum of magnitudes, several 1e-5 of the rms entry at n = 2^18.
GRAD_MAX_ENTRY_TOL = 3e-4


def _max_entry(a, b):
    return np.abs(a - b).max() / np.sqrt(np.mean(b * b))


def test_c4_kmm_full_size_sampled_rows(egp):
    """n = 2^20, d = 11: the bench workload, t = 16 (probe columns) and t = 17 (y + probes)."""
    import torch
    w = make_workload("C4", with_targets=False)
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    X = _cuda(w.X)
    rows = _rows(w.n, 48, 1)
    L = egp.lib()
    for cols in (slice(1, 17), slice(0, 17)):
        V = np.ascontiguousarray(w.V[:, cols])
        ref = orc.kmm_rows(w.X, V, h, rows)
        for mode in (0, 3):      # the default (symmetric kernels at this size, bench.py's headline) and one-sided
            try:
                L.egp_set_kmm_mode(mode)
                out = egp.kmm(X, _cuda(V), w.lengthscales, w.outputscale, w.noise, w.kernel_type)
                torch.cuda.synchronize()
            finally:
                L.egp_set_kmm_mode(0)
            got = out[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
            err = _rel(got, ref)
            print("C4 t=%d mode %d sampled-row rel err %.3e, worst entry / rms %.3e" % (V.shape[1], mode, err,
                                                                                       _max_entry(got, ref)))
            assert err <= KMM_TOL
            assert _max_entry(got, ref) <= MAX_ENTRY_TOL
            assert torch.isfinite(out).all()


def test_c5_kmm_full_size_sampled_rows(egp):
    """n = 2^21, Matern-3/2, t = 17."""
    import torch
    w = make_workload("C5", with_targets=False)
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    rows = _rows(w.n, 24, 2)
    out = egp.kmm(_cuda(w.X), _cuda(w.V), w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    torch.cuda.synchronize()
    got = out[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    ref = orc.kmm_rows(w.X, w.V, h, rows)
    print("C5 sampled-row rel err %.3e, worst entry / rms %.3e" % (_rel(got, ref), _max_entry(got, ref)))
    assert _rel(got, ref) <= KMM_TOL
    assert _max_entry(got, ref) <= MAX_ENTRY_TOL


def test_c3_kmm_and_grad_full_size_sampled_rows(egp):
    """n = 2^18, d = 25: KMM and all 25 derivative products."""
    import torch
    w = make_workload("C3")
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    X, V = _cuda(w.X), _cuda(w.V)
    rows = _rows(w.n, 24, 3)
    idx = torch.from_numpy(rows).cuda()
    ref_rows = orc.kmm_rows(w.X, w.V, h, rows)
    for mode in (0, 3):
        try:
            egp.lib().egp_set_kmm_mode(mode)
            out = egp.kmm(X, V, w.lengthscales, w.outputscale, w.noise, w.kernel_type)
            torch.cuda.synchronize()
        finally:
            egp.lib().egp_set_kmm_mode(0)
        got_rows = out[idx].cpu().numpy().astype(np.float64)
        print("C3 mode %d sampled-row rel err %.3e, worst entry / rms %.3e" % (mode, _rel(got_rows, ref_rows),
                                                                               _max_entry(got_rows, ref_rows)))
        assert _rel(got_rows, ref_rows) <= KMM_TOL
        assert _max_entry(got_rows, ref_rows) <= MAX_ENTRY_TOL
    g = egp.kmm_grad(X, V, w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    torch.cuda.synchronize()
    ref = orc.kmm_grad_rows(w.X, w.V, h, rows)
    got = g[:, idx, :].cpu().numpy().astype(np.float64)
    worst = max(_max_entry(got[k], ref[k]) for k in range(w.d))
    print("C3 derivative products: worst rel err %.3e, worst entry / rms %.3e"
          % (max(_rel(got[k], ref[k]) for k in range(w.d)), worst))
    for k in range(w.d):
        assert _rel(got[k], ref[k]) <= KMM_TOL, k
        assert _max_entry(got[k], ref[k]) <= GRAD_MAX_ENTRY_TOL, k


def test_c2_full_solve_residual(egp):
    """C2 (n = 65536, d = 18, Matern-5/2, t = 17): mBCG to relative residual 1e-2 with a rank-20 preconditioner.
    The solution is pinned through the true residual on sampled rows (oracle rows of Khat U against B)."""
    w = make_workload("C2")
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    X, B = _cuda(w.X), _cuda(w.V)
    P = egp.piv_chol_precond(X, w.lengthscales, w.outputscale, w.noise, w.kernel_type, w.rank)
    assert P.rank == w.rank and len(set(P.pivots.tolist())) == w.rank and P.pivots[0] == 0
    res = egp.mbcg(X, B, w.lengthscales, w.outputscale, w.noise, w.kernel_type, precond=P, max_iter=w.max_iter,
                   tol=w.tol)
    print("C2 solve: %d iterations, worst residual %.3e" % (res["iters"], res["rel_resid"].max()))
    assert res["rel_resid"].max() <= w.tol and res["iters"] < w.max_iter
    U = res["U"].cpu().numpy()
    rows = _rows(w.n, 256, 4)
    KU = orc.kmm_rows(w.X, U, h, rows)
    scale = np.linalg.norm(w.V.astype(np.float64), axis=0) / np.sqrt(w.n)      # rms of each right-hand side
    resid_rms = np.sqrt(np.mean((KU - w.V[rows].astype(np.float64)) ** 2, axis=0))
    # sampled estimate of ||Khat u - b|| / ||b|| per column: same order as the reported recurrence residual
    assert np.all(resid_rms / scale <= 3.0 * w.tol)


# ------------------------------------------------------------------------------------------------------------------
# The solver configurations at the size they run. K cannot be materialised, so a solution is pinned through its true
# residual on sampled rows: row i of Khat U comes from the oracle (dense fp64 row against all n points), and the
# root-mean-square of (Khat U - B)[rows, c] estimates ||Khat u_c - b_c|| / sqrt(n). Dividing by rms(b_c) gives the
# sampled true relative residual, which must agree with the relative residual of the recurrence that the solver
# reports. The estimate's own scatter over m sampled rows is about sqrt(2/m) for Gaussian-like residual entries and
# larger for the clustered inputs here; RESID_FACTOR covers both it and the fp32 drift between the recurrence and the
# true residual.
# ------------------------------------------------------------------------------------------------------------------
BILINEAR_MAG_TOL = 2.0 ** -23      # see test_c5_gradient_bilinear_forms_on_sampled_rows
RESID_ROWS = 256
RESID_FACTOR = 1.6      # sampled true residual within [1/1.6, 1.6] x the reported recurrence residual, per column


def _sampled_true_residual(w, h, U, B, rows, chunk=64):
    """Per column: rms over `rows` of (Khat U - B) divided by the rms of the column of B over all points."""
    KU = np.concatenate([orc.kmm_rows(w.X, U, h, rows[i:i + chunk]) for i in range(0, len(rows), chunk)])
    num = np.sqrt(np.mean((KU - B[rows].astype(np.float64)) ** 2, axis=0))
    den = np.linalg.norm(B.astype(np.float64), axis=0) / np.sqrt(B.shape[0])
    return num / den


@pytest.fixture(scope="module")
def c4(egp):
    """C4 with its targets (n = 2^20, d = 11, RBF, [y | 16 probes]) and its rank-100 preconditioner, built once."""
    w = make_workload("C4")
    X, B = _cuda(w.X), _cuda(w.V)
    P = egp.piv_chol_precond(X, w.lengthscales, w.outputscale, w.noise, w.kernel_type, w.rank)
    assert P.rank == w.rank and len(set(P.pivots.tolist())) == w.rank and P.pivots[0] == 0
    return w, X, B, P


@pytest.mark.parametrize("shrink", [False, True])
def test_c4_full_solve_true_residual(egp, c4, shrink):
    """C4's full solve as bench.py runs it (Experiment details: tolerance 1, rank-100 pivoted Cholesky; t = 17, default
    mode = symmetric kernels): for every column the true relative residual on oracle rows agrees with the recurrence
    residual the solver reports, with and without column shrinking."""
    w, X, B, P = c4
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    res = egp.mbcg(X, B, w.lengthscales, w.outputscale, w.noise, w.kernel_type, precond=P, max_iter=w.max_iter,
                   tol=w.tol, shrink=shrink)
    rel = res["rel_resid"].astype(np.float64)
    print("C4 solve shrink=%s: %d iterations, per-column iterations %s" % (shrink, res["iters"], res["col_iters"].tolist()))
    assert res["iters"] < w.max_iter and rel.max() <= w.tol
    if shrink:
        assert res["col_iters"][1:].max() < res["iters"]      # the probe columns left before the y column was done
    else:
        assert np.all(res["col_iters"] == res["iters"])
    U = res["U"].cpu().numpy()
    assert np.isfinite(U).all()
    rows = _rows(w.n, RESID_ROWS, 11)
    true_rel = _sampled_true_residual(w, h, U, w.V, rows)
    ratio = true_rel / rel
    print("   recurrence residual", np.array2string(rel, precision=3))
    print("   sampled true       ", np.array2string(true_rel, precision=3))
    print("   ratio min %.3f max %.3f" % (ratio.min(), ratio.max()))
    assert np.all(ratio <= RESID_FACTOR) and np.all(ratio >= 1.0 / RESID_FACTOR)
    assert true_rel.max() <= RESID_FACTOR * w.tol


@pytest.fixture(scope="module")
def c5(egp):
    """C5 (n = 2^21, d = 11, Matern-3/2, y + 16 probes of covariance P) with its rank-100 preconditioner and a solve
    capped at 8 iterations. The configuration's rank 100 does not reach tolerance 1 within its 100 iterations; what the
    tests below pin holds at any iteration."""
    import torch
    cap, tp = 8, 16
    w = make_workload("C5")
    hyp = (w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    rng = np.random.default_rng(55)
    X, y = _cuda(w.X), _cuda(w.y)
    W1 = _cuda(2.0 * rng.integers(0, 2, size=(w.rank, tp)) - 1.0)
    W2 = _cuda(w.V[:, 1:])
    P = egp.piv_chol_precond(X, *hyp, w.rank)
    assert P.rank == w.rank and P.pivots[0] == 0 and len(set(P.pivots.tolist())) == w.rank
    # right-hand sides [y | L W1 + sigma W2] (test-side plumbing; egp_mll builds the same inside)
    Bd = torch.cat([y[:, None], P.L.T @ W1 + float(np.sqrt(w.noise)) * W2], dim=1).contiguous()
    res = egp.mbcg(X, Bd, *hyp, precond=P, max_iter=cap, tol=w.tol)
    assert res["iters"] == cap      # (not converged at this rank: stated, not hidden)
    U = res["U"].cpu().numpy()
    assert np.isfinite(U).all()
    del P
    return {"w": w, "hyp": hyp, "X": X, "y": y, "W1": W1, "W2": W2, "B": Bd.cpu().numpy(), "res": res, "U": U,
            "cap": cap, "tp": tp}


def test_c5_capped_solve_true_residual(egp, c5):
    """True residual of every column of the capped C5 solve on oracle rows against the recurrence residual."""
    w, res = c5["w"], c5["res"]
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    rel = res["rel_resid"].astype(np.float64)
    rows = _rows(w.n, 64, 12)
    true_rel = _sampled_true_residual(w, h, c5["U"], c5["B"], rows, chunk=32)
    ratio = true_rel / rel
    print("C5 capped solve (%d iterations): recurrence residual %s" % (c5["cap"], np.array2string(rel, precision=3)))
    print("   sampled true %s, ratio min %.3f max %.3f" % (np.array2string(true_rel, precision=3), ratio.min(), ratio.max()))
    assert np.all(ratio <= RESID_FACTOR) and np.all(ratio >= 1.0 / RESID_FACTOR)


def test_c5_mll_quadratic_term_matches_the_solve(egp, c5):
    """egp_mll at C5 (Eq. 1): its quadratic term y^T u equals the one of the pinned solve (the y column does not
    depend on the probe columns), same iteration count, same worst residual up to the probes' rounding."""
    w, cap = c5["w"], c5["cap"]
    out = egp.mll(c5["X"], c5["y"], c5["W1"], c5["W2"], *c5["hyp"], rank=w.rank, max_iter=cap, tol=w.tol)
    quad = float(w.y.astype(np.float64) @ c5["U"][:, 0].astype(np.float64))
    rel = c5["res"]["rel_resid"].astype(np.float64)
    print("C5 egp_mll capped: mll %.1f, quad %.3f (solve: %.3f), %d iterations, worst residual %.3f"
          % (out["mll"], out["quad"], quad, out["iters"], out["rel_resid_max"]))
    assert out["iters"] == cap and out["rank"] == w.rank
    assert abs(out["quad"] - quad) <= 1e-4 * abs(quad)
    assert abs(out["rel_resid_max"] - rel.max()) <= 0.05 * rel.max()      # probe columns built by another kernel: rounding
    assert np.all(np.isfinite(out["grad"])) and np.isfinite(out["mll"])


def test_c5_gradient_bilinear_forms_on_sampled_rows(egp, c5):
    """The gradient's bilinear forms (Eq. 2) at C5 with A zero outside a sampled row set, which makes each form equal
    sum_{i in rows} a_i^T ((dK/dl_k) B)_i, rows the oracle computes exactly. A = rows of U, B = U, the step's weights.
    Tolerance: the forms have no stated bound, so it follows from the arithmetic. Each is a sum of |rows| n t products
    held in per-lane fp32 accumulators (fp64 beyond the lane), so its error scales with the sum of the terms'
    magnitudes M_k = sum_c |w_c| sum_{i in rows} |a_ic| ((dK/dl_k) |B|)_ic (every dK/dl_k entry is >= 0), not with the
    value: B = Khat^{-1}[y | z] oscillates, and K B cancels to a 1e-5 fraction of K |B| here. The bound is 2^-23 M_k
    (two fp32 roundings of the magnitude sum); the Cauchy-Schwarz bound that the KMM tolerance implies,
    1e-4 ||A w|| ||(dK/dl_k) B||, is accepted as well where it is the looser one."""
    w, U, tp = c5["w"], c5["U"], c5["tp"]
    h = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise)
    m = 8
    brow = _rows(w.n, m, 13)
    wts = np.full(tp + 1, -0.5 / tp)
    wts[0] = 0.5
    A = np.zeros_like(U)
    A[brow] = U[brow]
    got = egp.kmm_grad_bilinear(c5["X"], _cuda(A), c5["res"]["U"], *c5["hyp"], weights=wts)
    Aw = A[brow].astype(np.float64) * wts
    h0 = orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, 0.0)
    absU = np.abs(U)
    ref_rows = orc.kmm_grad_rows(w.X, U, h, brow)
    mag_rows = orc.kmm_grad_rows(w.X, absU, h, brow)
    Krows = orc.kmm_rows(w.X, U, h0, brow) / w.outputscale
    Kmag = orc.kmm_rows(w.X, absU, h0, brow) / w.outputscale
    worst_cs, worst_mag = 0.0, 0.0
    for k in range(w.d + 1):
        rr, mm = (ref_rows[k], mag_rows[k]) if k < w.d else (Krows, Kmag)
        ref = np.sum(Aw * rr)
        cs = np.linalg.norm(Aw) * np.linalg.norm(rr)
        mag = np.sum(np.abs(Aw) * mm)
        err = abs(got[k] - ref)
        worst_cs, worst_mag = max(worst_cs, err / cs), max(worst_mag, err / mag)
        assert err <= max(KMM_TOL * cs, BILINEAR_MAG_TOL * mag), (k, got[k], ref, cs, mag)
    print("C5 sampled bilinear forms: worst error %.2e of the Cauchy-Schwarz bound, %.2e of the sum of magnitudes"
          % (worst_cs, worst_mag))
