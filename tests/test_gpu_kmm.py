"""Parity of the fused HIP kernel-matrix multiply with the dense fp64 oracle (through the C ABI)."""
import numpy as np
import pytest

import oracle as orc
from workloads import make_workload

pytestmark = pytest.mark.gpu

# the stated bound of this build: relative Frobenius error of the KMM <= 1e-4 at fp32 (no reduced-precision MFMA is used)
KMM_TOL = 1e-4


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
    Xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
    Vd = torch.from_numpy(np.ascontiguousarray(V)).cuda()
    out = egp.kmm(Xd, Vd, ls, s, noise, kind)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def _rel(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def test_kmm_c1_full(egp):
    w = make_workload("C1")
    got = _run(egp, w.X, w.V, w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    ref = orc.kmm(w.X, w.V, orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise))
    err = _rel(got, ref)
    print("C1 KMM rel err", err)
    assert err <= KMM_TOL
    # per-column too
    for c in range(w.t):
        assert _rel(got[:, c], ref[:, c]) <= KMM_TOL


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,t", [(1, 1, 1), (15, 3, 2), (16, 4, 16), (17, 7, 17), (257, 11, 16), (1000, 8, 5),
                                   (2049, 18, 17), (3001, 25, 16), (777, 31, 33), (1300, 12, 32),
                                   (600, 2, 40), (513, 5, 70)])
def test_kmm_shapes(egp, kind, n, d, t):
    rng = np.random.default_rng(1000 * n + 10 * d + t + kind)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.3), np.log(3.0), d)).astype(np.float32)
    s, noise = 1.7, 0.3
    got = _run(egp, X, V, ls, s, noise, kind)
    ref = orc.kmm(X, V, orc.Hyper(kind, ls, s, noise))
    assert got.shape == ref.shape
    assert np.isfinite(got).all()
    assert _rel(got, ref) <= KMM_TOL


def test_kmm_c2_recipe_rows(egp):
    """Larger case, big-tile launch shape with column splits: sampled rows computed exactly by the oracle."""
    w = make_workload("C2", n=40000)
    got = _run(egp, w.X, w.V, w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    rows = np.random.default_rng(7).choice(w.n, 192, replace=False)
    rows[:3] = [0, w.n - 1, w.n // 2]
    ref = orc.kmm_rows(w.X, w.V, orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise), rows)
    assert _rel(got[rows], ref) <= KMM_TOL


def test_kmm_special_cases(egp):
    rng = np.random.default_rng(3)
    n, d, t = 700, 4, 16
    X = rng.uniform(0, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    s, noise = 1.3, 0.2
    # huge lengthscale: K -> s 1 1^T
    got = _run(egp, X, V, np.full(d, 1e6, np.float32), s, noise, orc.RBF)
    expect = s * V.astype(np.float64).sum(axis=0, keepdims=True) + noise * V.astype(np.float64)
    assert _rel(got, expect) <= KMM_TOL
    # identical points
    same = np.tile(X[:1], (n, 1))
    got = _run(egp, same, V, np.full(d, 0.5, np.float32), s, noise, orc.MATERN32)
    assert _rel(got, expect) <= KMM_TOL
    # noise = 0 gives K V; determinism: two runs bitwise equal
    a = _run(egp, X, V, np.full(d, 0.5, np.float32), s, 0.0, orc.MATERN52)
    b = _run(egp, X, V, np.full(d, 0.5, np.float32), s, 0.0, orc.MATERN52)
    assert np.array_equal(a, b)
    ref = orc.kmm(X, V, orc.Hyper(orc.MATERN52, np.full(d, 0.5), s, 0.0))
    assert _rel(a, ref) <= KMM_TOL


def test_kmm_argument_errors(egp):
    import torch
    X = torch.zeros(32, 3, device="cuda")
    V = torch.zeros(32, 2, device="cuda")
    with pytest.raises(egp.EgpError):
        egp.kmm(X, V, [1.0, -1.0, 1.0], 1.0, 0.1, 0)
    with pytest.raises(egp.EgpError):
        egp.kmm(X, V, [1.0, 1.0, 1.0], 1.0, 0.1, 7)
    with pytest.raises(egp.EgpError):
        egp.kmm(X, V, [1.0, 1.0, 1.0], 1.0, -0.1, 0)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(egp.EgpError) as ei:
        egp.kmm(X, V, [1.0, 1.0, 1.0], 1.0, 0.1, 0, ws=small)
    assert ei.value.code == -2


def _set_mode(egp, mode):
    import ctypes as C
    L = egp.lib()
    L.egp_set_kmm_mode.argtypes = [C.c_int32]
    assert L.egp_set_kmm_mode(mode) == 0
    assert L.egp_get_kmm_mode() == mode


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,t", [(257, 11, 16), (2049, 18, 17), (3001, 25, 16), (777, 31, 33), (600, 2, 40),
                                   (1, 1, 1), (1000, 15, 5), (513, 16, 17)])
def test_kmm_split_bf16_mode(egp, mode, kind, n, d, t):
    """The bf16-split modes (reported separately from the fp32 mode) meet the same 1e-4 bound."""
    rng = np.random.default_rng(7 * n + d + t + kind)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.3), np.log(3.0), d)).astype(np.float32)
    ref = orc.kmm(X, V, orc.Hyper(kind, ls, 1.7, 0.3))
    try:
        _set_mode(egp, mode)
        got = _run(egp, X, V, ls, 1.7, 0.3, kind)
    finally:
        _set_mode(egp, 0)
    err = _rel(got, ref)
    assert err <= KMM_TOL, err
    with pytest.raises(AssertionError):
        _set_mode(egp, 5)


@pytest.mark.parametrize("mode", [1, 2])
def test_kmm_split_bf16_c2_recipe_rows(egp, mode):
    w = make_workload("C2", n=40000)
    ref_rows = np.random.default_rng(7).choice(w.n, 128, replace=False)
    ref = orc.kmm_rows(w.X, w.V, orc.Hyper(w.kernel_type, w.lengthscales, w.outputscale, w.noise), ref_rows)
    try:
        _set_mode(egp, mode)
        got = _run(egp, w.X, w.V, w.lengthscales, w.outputscale, w.noise, w.kernel_type)
    finally:
        _set_mode(egp, 0)
    err = _rel(got[ref_rows], ref)
    print("C2-recipe split-mode rel err", err)
    assert err <= KMM_TOL


@pytest.mark.parametrize("kind", [orc.RBF, orc.MATERN32, orc.MATERN52, orc.MATERN12])
@pytest.mark.parametrize("n,d,t", [(32768, 11, 16), (33000, 3, 16), (40000, 14, 48), (65536, 8, 16), (33281, 11, 17),
                                   (33000, 18, 17), (34000, 25, 16), (32768, 31, 17), (40000, 2, 33), (33000, 8, 1), (40000, 25, 1),
                                   (32768, 11, 18), (33000, 11, 33), (33281, 25, 32), (32768, 31, 32), (34000, 18, 33),
                                   (33000, 11, 65)])
def test_kmm_symmetric_kernels_rows(egp, kind, n, d, t):
    """The default fp32 mode at sizes where the symmetric kernels run (every off-diagonal tile used for the row-side
    and the column-side output) against rows computed exactly by the oracle: even and odd block counts, rows at the block edges and around the half-way
    block, several column groups (1, 16, 17, 32, 33 columns, ragged ones), every stage shape; a 33-column group
    beyond d = 11 takes the one-sided kernel."""
    rng = np.random.default_rng(11 * n + d + t + kind)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.3), np.log(3.0), d)).astype(np.float32)
    rows = rng.choice(n, 160, replace=False)
    edges = [0, 1, 15, 16, 511, 512, 513, n // 2 - 1, n // 2, n // 2 + 511, n // 2 + 512, n - 513, n - 512, n - 2, n - 1]
    rows[:len(edges)] = edges
    rows = np.unique(rows)
    ref = orc.kmm_rows(X, V, orc.Hyper(kind, ls, 1.3, 0.2), rows)
    got = _run(egp, X, V, ls, 1.3, 0.2, kind)
    try:
        _set_mode(egp, 3)      # every tile formed, no use of the symmetry
        base = _run(egp, X, V, ls, 1.3, 0.2, kind)
    finally:
        _set_mode(egp, 0)
    assert np.isfinite(got).all()
    err = _rel(got[rows], ref)
    print(f"symmetric kernels n={n} d={d} t={t} kind={kind}: rel err {err:.2e}; vs one-sided kernel {_rel(got, base):.2e}")
    assert err <= KMM_TOL
    assert _rel(got, base) <= 2e-5      # every row: same arithmetic, different summation order


@pytest.mark.parametrize("n,d,t", [(33000, 11, 17), (40000, 14, 48), (33000, 8, 1), (33000, 40, 17)])
def test_kmm_symmetric_kernels_are_bit_reproducible(egp, n, d, t):
    """The column-side sums travel between workgroups as 64-bit fixed-point atomic adds, which commute exactly: the
    same call gives the same bits every time, also with other work in between, and for right-hand sides whose columns
    differ by many orders of magnitude (each column has its own fixed-point scale)."""
    rng = np.random.default_rng(n + d + t)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    V *= np.exp(rng.uniform(np.log(1e-12), np.log(1e12), t)).astype(np.float32)      # column scales 1e-12 .. 1e12
    ls = np.exp(rng.uniform(np.log(0.3), np.log(3.0), d)).astype(np.float32)
    try:
        first = _run(egp, X, V, ls, 1.3, 0.2, orc.MATERN32)
        _run(egp, X, np.flipud(V).copy(), ls, 0.7, 0.1, orc.RBF)
        for _ in range(3):
            again = _run(egp, X, V, ls, 1.3, 0.2, orc.MATERN32)
            assert np.array_equal(first, again)
        _set_mode(egp, 3)
        base = _run(egp, X, V, ls, 1.3, 0.2, orc.MATERN32)
    finally:
        _set_mode(egp, 0)
    # column by column (their scales differ by 24 orders of magnitude): the one-sided kernel's result up to summation order
    for c in range(t):
        assert _rel(first[:, c], base[:, c]) <= 2e-5, c
    # a zero column stays exactly zero beside non-zero ones
    V0 = V.copy()
    V0[:, 0] = 0.0
    z = _run(egp, X, V0, ls, 1.3, 0.2, orc.MATERN32)
    assert np.all(z[:, 0] == 0.0) and (t == 1 or np.array_equal(z[:, 1:], first[:, 1:]))


def test_kmm_symmetric_kernels_keep_small_entries_beside_an_outlier(egp):
    """One entry of every right-hand-side column is 10^12 times the others, at a point so far from all others that
    its kernel values with them vanish: no other row's result depends on it. The fixed-point scale of the column-side
    sums comes from the column's sum of absolute values, so one unit is 2^-61 of about that entry (5e-7 here) and the
    other rows still agree with the one-sided kernel entry by entry at fp32 summation-order level. (A scale taken from
    n * max |V| would put the unit at 1e-2.)"""
    n, d, t = 33000, 3, 16
    rng = np.random.default_rng(99)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    X[12345] = 10.0
    V = rng.standard_normal((n, t)).astype(np.float32)
    V[12345, :] = 1e12
    ls = np.full(d, 0.5, np.float32)
    got = _run(egp, X, V, ls, 1.0, 0.1, orc.RBF)
    try:
        _set_mode(egp, 3)
        base = _run(egp, X, V, ls, 1.0, 0.1, orc.RBF)
    finally:
        _set_mode(egp, 0)
    others = np.arange(n) != 12345
    scale = np.abs(base[others]).mean()
    assert scale < 1e3      # the outlier has not leaked into the other rows
    worst = np.abs(got[others] - base[others]) / (3e-5 * np.abs(base[others]) + 3e-5 * scale)
    print("outlier test: mean |entry| %.3g, worst difference ratio %.3g" % (scale, worst.max()))
    assert worst.max() <= 1.0
    assert abs(got[12345, 0] - base[12345, 0]) <= 1e-5 * abs(base[12345, 0])


@pytest.mark.parametrize("ls_value,bound", [(0.3, 3e-6), (0.1, 1.5e-5), (0.05, 5e-5)])
def test_kmm_accuracy_envelope_at_short_lengthscales(egp, ls_value, bound):
    """The distance step is the norm expansion accumulated in fp32: its error grows with the squared norm of the
    centred, scaled points, i.e. with (extent / lengthscale)^2. The figures the design notes quote, with head room."""
    n, d, t = 4000, 3, 16
    rng = np.random.default_rng(5)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.full(d, ls_value, np.float32)
    ref = orc.kmm(X, V, orc.Hyper(orc.RBF, ls, 1.0, 0.0))
    got = _run(egp, X, V, ls, 1.0, 0.0, orc.RBF)
    err = _rel(got, ref)
    print(f"lengthscale {ls_value}: rel err {err:.2e}")
    assert err <= bound and err <= KMM_TOL


def test_kmm_one_sided_kernels_on_other_shapes(egp):
    """Shapes the symmetric kernels do not cover (small n, a group of 33 columns beyond d = 11) run the one-sided
    kernels in the default mode: same bits as with the symmetry switched off."""
    for n, d, t in ((3000, 11, 16), (33000, 18, 33)):
        rng = np.random.default_rng(n + d)
        X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
        V = rng.standard_normal((n, t)).astype(np.float32)
        ls = np.full(d, 0.8, np.float32)
        base = _run(egp, X, V, ls, 1.0, 0.1, orc.RBF)
        try:
            _set_mode(egp, 3)
            got = _run(egp, X, V, ls, 1.0, 0.1, orc.RBF)
        finally:
            _set_mode(egp, 0)
        assert np.array_equal(got, base)


@pytest.mark.parametrize("n,d,t", [(4000, 8, 16), (33000, 11, 17), (33000, 40, 16)])
def test_kmm_under_hip_graph_capture(egp, n, d, t):
    """egp_kmm with a caller-provided workspace enqueues kernels only (no allocation, no memset node, no host
    synchronisation), so a caller can capture it into a HIP graph. The graph is replayed several times with new
    right-hand sides, with eager calls and synchronisations in between, and every replay must give the eager result
    bit for bit (one-sided kernel, symmetric kernel with its fixed-point column-side sums, wide symmetric kernel)."""
    import torch
    L = egp.lib()
    rng = np.random.default_rng(n + d)
    X = torch.from_numpy(rng.uniform(0, 1, (n, d)).astype(np.float32)).cuda()
    V = torch.from_numpy(rng.standard_normal((n, t)).astype(np.float32)).cuda()
    ls = np.full(d, 0.7 * np.sqrt(d / 8), np.float32)
    out = torch.empty_like(V)
    ws = torch.empty(L.egp_kmm_ws_bytes(n, d, t), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        egp.kmm(X, V, ls, 1.1, 0.2, orc.MATERN52, out=out, ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        egp.kmm(X, V, ls, 1.1, 0.2, orc.MATERN52, out=out, ws=ws)
    for _ in range(3):
        V.copy_(torch.from_numpy(rng.standard_normal((n, t)).astype(np.float32)).cuda())
        want = egp.kmm(X, V, ls, 1.1, 0.2, orc.MATERN52).clone()
        torch.cuda.synchronize()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert bool((out == want).all())


def test_per_call_mode_equals_the_process_default_and_leaves_it_alone(egp):
    """The arithmetic mode as a per-call option (egp_kmm_ex / egp_mbcg_ex) gives the bits that the same mode gives as
    process-wide default, whatever the default is while the call runs, and never changes the default."""
    import torch
    rng = np.random.default_rng(5)
    n, d, t = 33000, 5, 17      # large enough for the symmetric kernels in the default mode
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.full(d, 0.7, np.float32)
    Xd, Vd = torch.from_numpy(X).cuda(), torch.from_numpy(V).cuda()
    L = egp.lib()
    by_default = {}
    try:
        for mode in range(4):
            egp.set_kmm_mode(mode)
            by_default[mode] = egp.kmm(Xd, Vd, ls, 1.0, 0.1, orc.RBF).clone()
        for default in (0, 2):
            egp.set_kmm_mode(default)
            for mode in range(4):
                out = egp.kmm(Xd, Vd, ls, 1.0, 0.1, orc.RBF, mode=mode)
                assert torch.equal(out, by_default[mode]), (default, mode)
                assert L.egp_get_kmm_mode() == default
    finally:
        egp.set_kmm_mode(0)
    assert not torch.equal(by_default[0], by_default[3])      # symmetric and one-sided sums differ in the last bits
    rows = np.random.default_rng(6).choice(n, 64, replace=False)
    ref = orc.kmm_rows(X, V, orc.Hyper(orc.RBF, ls, 1.0, 0.1), rows)
    for mode in range(4):
        assert _rel(by_default[mode].cpu().numpy().astype(np.float64)[rows], ref) <= KMM_TOL
    # the solver takes both options per call
    a = egp.mbcg(Xd, Vd, ls, 1.0, 0.1, orc.RBF, max_iter=5, tol=0.0, mode=3, shrink=False)
    egp.set_kmm_mode(3)
    try:
        b = egp.mbcg(Xd, Vd, ls, 1.0, 0.1, orc.RBF, max_iter=5, tol=0.0)
    finally:
        egp.set_kmm_mode(0)
    assert torch.equal(a["U"], b["U"]) and L.egp_get_mbcg_shrink() == 0
