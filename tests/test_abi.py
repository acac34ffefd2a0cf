"""The C-ABI library loads and exports every symbol include/egp.h declares; host-side argument checks.
No compute call is made here (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "egp.h")


@pytest.fixture(scope="module")
def lib():
    import paper_1903_08114_amd as egp
    if not os.path.exists(egp.lib_path()):
        from paper_1903_08114_amd import build
        build.build(verbose=False)
    return egp.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(egp_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_entry_points():
    names = declared_functions()
    for required in ("egp_kmm", "egp_mbcg", "egp_piv_chol_precond", "egp_kmm_grad"):
        assert required in names


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), f"{name} declared in egp.h but not exported"


def test_version_and_error_string(lib):
    assert lib.egp_version().decode().count(".") == 1
    assert isinstance(lib.egp_last_error(), bytes)


def test_workspace_queries_are_host_only(lib):
    n, d, t = 1 << 20, 11, 17
    kmm = lib.egp_kmm_ws_bytes(n, d, t)
    # O(n (d + t)) bytes, never O(n^2): packed points (fp32 and the bf16-split operands), packed V (fp32 and
    # split), one partial buffer
    assert 0 < kmm < n * (4 * (d + 5) + 320 + 4 * 6 * 33) + (1 << 22)
    mb = lib.egp_mbcg_ws_bytes(n, d, t, 100, 100)
    assert kmm < mb < 6 * n * t * 4 + kmm + (1 << 28)
    assert lib.egp_piv_chol_precond_ws_bytes(n, d, 100) > 0
    assert lib.egp_kmm_ws_bytes(0, d, t) == 0
    assert lib.egp_kmm_ws_bytes(n, 0, t) == 0
    assert lib.egp_kmm_ws_bytes(n, 400, t) == 0
    assert lib.egp_kmm_ws_bytes(4096, 399, t) > 4096 * 400 * 4
    assert lib.egp_kmm_grad_ws_bytes(n, 32, t) == 0          # the materialised derivative product stays at d <= 31
    assert lib.egp_mll_ws_bytes(4096, 90, 8, 10, 10) > 0
    assert lib.egp_kmm_grad_bilinear_ws_bytes(4096, 399, 17) > 0
    assert lib.egp_mll_ws_bytes(4096, 400, 8, 10, 10) == 0
    assert lib.egp_kmm_ws_bytes(n, d, 0) == 0
    assert lib.egp_mbcg_ws_bytes(n, d, 34, 0, 10) == 0


def test_argument_validation_without_device_work(lib):
    """Bad arguments are rejected before any HIP call is made."""
    from paper_1903_08114_amd.binding import _hyper
    h = _hyper(0, [1.0, 1.0], 1.0, 0.1)
    fake = C.c_void_p(0x1000)      # aligned, never dereferenced: validation fails first
    # NULL X
    assert lib.egp_kmm(None, 10, fake, 2, C.byref(h), fake, fake, 1 << 30, None) == -1
    assert b"X is NULL" in lib.egp_last_error()
    # misaligned V
    assert lib.egp_kmm(fake, 10, C.c_void_p(0x1004), 2, C.byref(h), fake, fake, 1 << 30, None) == -1
    # n < 1, n beyond 2^31 - 1 (the same bound in every entry point), t out of range
    assert lib.egp_kmm(fake, 0, fake, 2, C.byref(h), fake, fake, 1 << 30, None) == -1
    assert lib.egp_kmm(fake, 1 << 31, fake, 2, C.byref(h), C.c_void_p(0x3000), C.c_void_p(0x2000), 1 << 62, None) == -1
    assert b"2^31-1" in lib.egp_last_error()
    assert lib.egp_kmm(fake, 10, fake, 0, C.byref(h), fake, fake, 1 << 30, None) == -1
    assert lib.egp_kmm(fake, 10, fake, 5000, C.byref(h), fake, fake, 1 << 30, None) == -1
    # aliasing
    assert lib.egp_kmm(fake, 10, fake, 2, C.byref(h), fake, C.c_void_p(0x2000), 1 << 30, None) == -1
    # workspace too small
    assert lib.egp_kmm(fake, 10, fake, 2, C.byref(h), C.c_void_p(0x3000), C.c_void_p(0x2000), 16, None) == -2
    # bad hyper-parameters
    for bad in (_hyper(5, [1.0], 1.0, 0.1), _hyper(0, [0.0], 1.0, 0.1), _hyper(0, [1.0], 0.0, 0.1),
                _hyper(0, [1.0], 1.0, -1.0), _hyper(0, [float("nan")], 1.0, 0.1)):
        assert lib.egp_kmm(fake, 10, fake, 2, C.byref(bad), C.c_void_p(0x3000), C.c_void_p(0x2000), 1 << 30,
                           None) == -1
    assert lib.egp_kmm(fake, 10, fake, 2, None, C.c_void_p(0x3000), C.c_void_p(0x2000), 1 << 30, None) == -1
    # mbcg: t > 33, negative max_iter
    assert lib.egp_mbcg(fake, 10, fake, 34, C.byref(h), None, 5, 0.1, C.c_void_p(0x3000), None, None, None, None,
                        None, C.c_void_p(0x2000), 1 << 30, None) == -1
    assert lib.egp_mbcg(fake, 10, fake, 2, C.byref(h), None, -1, 0.1, C.c_void_p(0x3000), None, None, None, None,
                        None, C.c_void_p(0x2000), 1 << 30, None) == -1


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_1903_08114_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith(".py"):
                assert "paper_1903_08114_amd" not in open(os.path.join(dirpath, f)).read().replace(
                    "The product path (paper_1903_08114_amd)", "")


def test_tridiag_log_quadrature_host_helper(lib):
    """The library's own tridiagonal eigen-solver (used for the Lanczos quadrature) against numpy's eigh."""
    import numpy as np
    import paper_1903_08114_amd as egp
    rng = np.random.default_rng(0)
    for m in (1, 2, 3, 7, 40, 200):
        # a positive definite tridiagonal: Lanczos-like, from a Cholesky-style bidiagonal product
        dg = rng.uniform(0.5, 2.0, m)
        lo = rng.uniform(-1.0, 1.0, max(m - 1, 0))
        Bm = np.diag(dg) + (np.diag(lo, -1) if m > 1 else 0)
        T = Bm @ Bm.T
        lam, Q = np.linalg.eigh(T)
        want = float(np.sum(Q[0] ** 2 * np.log(lam)))
        got = egp.tridiag_logquad(np.diag(T).copy(), np.diag(T, 1).copy() if m > 1 else np.zeros(0))
        assert abs(got - want) <= 1e-10 * max(1.0, abs(want)), m
    # graded spectrum (what CG on an ill-conditioned system produces)
    m = 60
    dg = np.geomspace(1e-3, 1e3, m)
    lo = 0.3 * np.sqrt(dg[:-1] * dg[1:])
    T = np.diag(dg) + np.diag(lo, 1) + np.diag(lo, -1)
    lam, Q = np.linalg.eigh(T)
    assert abs(egp.tridiag_logquad(dg, lo) - np.sum(Q[0] ** 2 * np.log(lam))) < 1e-9
    # not positive definite -> error
    with pytest.raises(egp.EgpError):
        egp.tridiag_logquad(np.array([1.0, -2.0]), np.array([0.1]))


@pytest.mark.parametrize("n", [1, 17, 4096, 100000, 1 << 21])
@pytest.mark.parametrize("d", [1, 11, 31, 32, 90, 399])
def test_workspace_queries_cover_every_shape(lib, n, d):
    """Every in-range shape has a workspace size, sizes grow with the problem, out-of-range shapes report 0."""
    prev = 0
    for t in (1, 16, 17, 33, 64, 1024):
        b = lib.egp_kmm_ws_bytes(n, d, t)
        assert b > 0 and b >= prev
        prev = b
        assert lib.egp_kmm_cross_ws_bytes(7, n, d, t) > 0
    assert lib.egp_kmm_ws_bytes(n, d, 1025) == 0
    for rank in (1, 100, 1024):
        if rank > n:
            continue
        pc = lib.egp_piv_chol_precond_ws_bytes(n, d, rank)
        assert pc > 0
        mb = lib.egp_mbcg_ws_bytes(n, d, 17, rank, 50)
        assert mb > lib.egp_kmm_ws_bytes(n, d, 17)
        assert lib.egp_mll_ws_bytes(n, d, 16, rank, 50) > mb
        assert lib.egp_precond_apply_ws_bytes(n, 17, rank) > 0
        assert lib.egp_lanczos_ws_bytes(n, d, rank) > 0
        assert lib.egp_predict_ws_bytes(100, n, d, rank) > 0
    assert lib.egp_piv_chol_precond_ws_bytes(n, d, 1025) == 0
    assert lib.egp_mbcg_ws_bytes(n, d, 34, 0, 10) == 0
    assert lib.egp_block_lanczos_ws_bytes(n, d, 16, 4) > 0
    assert lib.egp_block_lanczos_ws_bytes(n, d, 33, 1) == 0
    assert lib.egp_block_lanczos_ws_bytes(n, d, 32, 33) == 0          # 32 * 33 > EGP_RANK_MAX
    assert lib.egp_kmm_grad_bilinear_ws_bytes(n, d, 36) > 0
    assert lib.egp_kmm_grad_bilinear_ws_bytes(n, d, 37) == 0
    assert (lib.egp_kmm_grad_ws_bytes(n, d, 16) > 0) == (d <= 31)
    # nothing is quadratic in n: a 2^21-point problem at rank 1024 stays far below the 288 GB of one MI355X
    assert lib.egp_mll_ws_bytes(1 << 21, d, 16, 1024, 100) < 40 * (1 << 30)


def _plan_splits(lib, rows, cols, d, t):
    used, sized = C.c_int32(-1), C.c_int32(-1)
    assert lib.egp_kmm_plan_splits(rows, cols, d, t, C.byref(used), C.byref(sized)) == 0
    return used.value, sized.value


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_partial_sum_buffer_holds_every_launch_plan(lib, mode):
    """No launch shape of any mode cuts the column points into more splits than the workspace holds partial
    sums for (host-side planning only). Sizes cover every padding class up to 2^15 rows and a few large ones,
    square and cross; d covers every k-step count and both sides of each launch-shape boundary."""
    ds = sorted(set(list(range(1, 36)) + list(range(36, 400, 4)) + [131, 132, 135, 136, 159, 160, 161, 399]))
    points = [1, 512, 513, 1025, 1537, 2047, 2500, 4096, 5000, 8192, 12345, 16384, 32767, 32768, 40000, 65536,
              100000, 1 << 18, 1 << 20, 1 << 21]
    assert lib.egp_set_kmm_mode(mode) == 0
    try:
        for rows in points:
            for cols in (rows, 1, 513, 2047, 40000, 1 << 20):
                for d in ds:
                    for t in (1, 2, 16, 17, 18, 32, 33, 34, 49, 50, 100):
                        used, sized = _plan_splits(lib, rows, cols, d, t)
                        assert 1 <= used <= sized <= 64, (rows, cols, d, t, mode, used, sized)
    finally:
        assert lib.egp_set_kmm_mode(0) == 0


def test_call_options_fix_the_mode_per_call(lib):
    """The *_ex entry points take the arithmetic mode per call: the launch plan of a call depends on the mode in its
    options alone, whatever the process-wide default is at that moment (and NULL / -1 take the default)."""
    from paper_1903_08114_amd.binding import _CallOpts
    shapes = [(40000, 40000, 11, 17), (1 << 20, 1 << 20, 11, 16), (5000, 5000, 25, 16), (2047, 2047, 159, 18),
              (70000, 70000, 90, 17), (1 << 18, 1 << 18, 11, 33), (33000, 33000, 31, 17), (40000, 40000, 20, 17)]

    def plan(opts, shape):
        used, sized = C.c_int32(-1), C.c_int32(-1)
        assert lib.egp_kmm_plan_splits_ex(*shape, opts, C.byref(used), C.byref(sized)) == 0
        return used.value, sized.value

    try:
        by_default = {}
        for mode in range(4):
            assert lib.egp_set_kmm_mode(mode) == 0
            by_default[mode] = [_plan_splits(lib, *s) for s in shapes]
            assert [plan(None, s) for s in shapes] == by_default[mode]
            assert [plan(C.byref(_CallOpts(-1, -1)), s) for s in shapes] == by_default[mode]
        # the symmetric, the one-sided and the all-bf16 plans differ on these shapes
        assert by_default[0] != by_default[3] and by_default[0] != by_default[2] and by_default[2] != by_default[3]
        for default in range(4):
            assert lib.egp_set_kmm_mode(default) == 0
            for mode in range(4):
                assert [plan(C.byref(_CallOpts(mode, -1)), s) for s in shapes] == by_default[mode]
                assert lib.egp_get_kmm_mode() == default      # a call's options never touch the default
    finally:
        assert lib.egp_set_kmm_mode(0) == 0
    # bad option values are refused before anything else is looked at
    used, sized = C.c_int32(), C.c_int32()
    assert lib.egp_kmm_plan_splits_ex(4096, 4096, 3, 1, C.byref(_CallOpts(7, -1)), C.byref(used), C.byref(sized)) == -1
    assert lib.egp_kmm_plan_splits_ex(4096, 4096, 3, 1, C.byref(_CallOpts(0, 5)), C.byref(used), C.byref(sized)) == -1
    fake = C.c_void_p(0x1000)
    from paper_1903_08114_amd.binding import _hyper
    h = _hyper(0, [1.0, 1.0], 1.0, 0.1)
    assert lib.egp_kmm_ex(fake, 10, fake, 2, C.byref(h), C.c_void_p(0x3000), C.c_void_p(0x2000), 1 << 30, None,
                          C.byref(_CallOpts(9, -1))) == -1
    assert b"kmm mode" in lib.egp_last_error()
    assert lib.egp_mbcg_ex(fake, 10, fake, 2, C.byref(h), None, 5, 0.1, C.c_void_p(0x3000), None, None, None, None,
                           None, C.c_void_p(0x2000), 1 << 30, None, C.byref(_CallOpts(-1, 2))) == -1


def test_no_mode_read_below_the_entry_points():
    """The process-wide defaults are read in csrc/api.hip only (once per call, by resolve_opts); no other source
    names them."""
    csrc = os.path.join(ROOT, "paper_1903_08114_amd", "csrc")
    for f in os.listdir(csrc):
        text = open(os.path.join(csrc, f)).read()
        if f != "api.hip":
            assert "g_kmm_mode" not in text and "g_mbcg_shrink" not in text and "kmm_mode()" not in text, f
    api = open(os.path.join(csrc, "api.hip")).read()
    body = api.split("static int resolve_opts", 1)[1]
    tail = body.split("\n}\n", 1)[1]
    # after resolve_opts only the setters and getters touch the atomics
    for line in tail.splitlines():
        if "g_kmm_mode" in line or "g_mbcg_shrink" in line:
            assert ".store(" in line or "egp_get_" in line, line


def test_plan_check_pins_a_shape_with_two_row_tiles_and_short_stages(lib):
    """2047 points at d = 159 (40 k-steps: two row tiles per wave, two column tiles per stage) take 64 splits; the
    workspace must hold them. This launch-shape class lies between the shapes a sampled bound would look at."""
    used, sized = _plan_splits(lib, 2047, 2047, 159, 18)
    assert used == 64 and sized >= 64
    assert lib.egp_kmm_plan_splits(0, 5, 3, 1, None, None) != 0


def test_python_mode_switch_by_name(lib):
    import paper_1903_08114_amd as egp
    prev = egp.set_kmm_mode("fp32_one_sided")
    try:
        assert lib.egp_get_kmm_mode() == 3
        assert egp.set_kmm_mode(prev) == 3
        with pytest.raises(egp.EgpError):
            egp.set_kmm_mode(9)
        with pytest.raises(KeyError):
            egp.set_kmm_mode("fp16")
    finally:
        lib.egp_set_kmm_mode(0)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on exactly one GPU: bench.py --gpus N with N > 1 exits with a message saying so."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in (res.stderr + res.stdout)
