"""egp_kmm_noalloc (the entry point for callers that cannot allocate: workspace in a device array built into the
library) against egp_kmm with a caller-provided workspace, through the C ABI: two calls in a row, the second with a
smaller input, so that whatever the first call left in the shared scratch array must not leak into the second."""
import ctypes as C

import numpy as np
import pytest

import oracle as orc

pytestmark = pytest.mark.gpu
KMM_TOL = 1e-4      # the fp32 bound of the multiply against the oracle; against egp_kmm the two entry points agree to the bit


@pytest.fixture(scope="module")
def egp():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1903_08114_amd as egp
    egp.lib()
    return egp


def _inputs(seed, n, d, t):
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    ls = np.exp(rng.uniform(np.log(0.3), np.log(3.0), d)).astype(np.float32)
    return X, V, ls


def test_noalloc_matches_workspace_entry_point_on_two_calls_in_a_row(egp):
    import torch
    # first call: n_pad >= 32768, so the default mode runs the symmetric kernel, whose int64 column-side slab lives in
    # the scratch array and must start at zero; second call: a smaller problem (one-sided kernel, other layout);
    # third call: d > 31 (the wide symmetric kernel: row operands in LDS, another workspace layout again)
    cases = [(7, 40000, 11, 17, orc.RBF), (8, 5000, 7, 16, orc.MATERN32), (9, 33000, 40, 16, orc.MATERN52)]
    dev = []
    for seed, n, d, t, kind in cases:
        X, V, ls = _inputs(seed, n, d, t)
        dev.append((torch.from_numpy(X).cuda(), torch.from_numpy(V).cuda(), X, V, ls, kind))
    want = [egp.kmm(Xd, Vd, ls, 1.3, 0.2, kind) for Xd, Vd, _, _, ls, kind in dev]
    torch.cuda.synchronize()
    outs = [torch.empty_like(Vd) for _, Vd, *_ in dev]
    before = torch.cuda.memory_allocated()
    got = []
    for (Xd, Vd, _, _, ls, kind), out in zip(dev, outs):      # back to back on one stream, no synchronisation between
        print("egp_kmm_noalloc n=%d d=%d t=%d kind=%d" % (Xd.shape[0], Xd.shape[1], Vd.shape[1], kind), flush=True)
        got.append(egp.kmm_noalloc(Xd, Vd, ls, 1.3, 0.2, kind, out=out))
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before      # the binding allocated nothing either (out was passed in)
    for g, wnt, (_, _, X, V, ls, kind) in zip(got, want, dev):
        assert torch.equal(g, wnt)      # same kernels, same launch plan: identical bits
        rows = np.random.default_rng(3).choice(X.shape[0], 64, replace=False)
        ref = orc.kmm_rows(X, V, orc.Hyper(kind, ls, 1.3, 0.2), rows)
        err = np.linalg.norm(g.cpu().numpy()[rows] - ref) / np.linalg.norm(ref)
        assert err <= KMM_TOL
    # and once more in the opposite order (small, then large): the large call finds the small call's leftovers
    again = [egp.kmm_noalloc(Xd, Vd, ls, 1.3, 0.2, kind) for Xd, Vd, _, _, ls, kind in reversed(dev)]
    torch.cuda.synchronize()
    for g, wnt in zip(again, reversed(want)):
        assert torch.equal(g, wnt)


def test_noalloc_rejects_sizes_beyond_the_scratch_array(egp):
    import torch
    L = egp.lib()
    X = torch.zeros((16, 11), dtype=torch.float32, device="cuda")
    V = torch.zeros((16, 17), dtype=torch.float32, device="cuda")
    from paper_1903_08114_amd.binding import _hyper
    h = _hyper(0, [1.0] * 11, 1.0, 0.1)
    # only the sizes are looked at before the refusal: n = 2^20 needs far more than the array holds
    rc = L.egp_kmm_noalloc(C.c_void_p(X.data_ptr()), 1 << 20, C.c_void_p(V.data_ptr()), 17, C.byref(h),
                           C.c_void_p(V.data_ptr()), None)
    assert rc == -1 and b"scratch" in L.egp_last_error()
    assert L.egp_kmm_noalloc(C.c_void_p(X.data_ptr()), 0, C.c_void_p(V.data_ptr()), 17, C.byref(h),
                             C.c_void_p(V.data_ptr()), None) == -1


def test_noalloc_under_hip_graph_capture(egp):
    """What the entry point is for: a caller that cannot allocate captures it into a HIP graph (after one call outside
    the capture, which looks up the scratch array's address). Every replay, with new right-hand sides and eager work
    in between, gives the bits of an eager egp_kmm call (symmetric kernel: its column-side slab in the scratch array is
    cleared by a fill kernel inside the graph, not by a memset node)."""
    import torch
    rng = np.random.default_rng(21)
    n, d, t = 33000, 11, 17
    X = torch.from_numpy(rng.uniform(0, 1, (n, d)).astype(np.float32)).cuda()
    V = torch.from_numpy(rng.standard_normal((n, t)).astype(np.float32)).cuda()
    ls = np.full(d, 0.8, np.float32)
    out = torch.empty_like(V)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        egp.kmm_noalloc(X, V, ls, 1.1, 0.2, orc.RBF, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        egp.kmm_noalloc(X, V, ls, 1.1, 0.2, orc.RBF, out=out)
    for _ in range(3):
        V.copy_(torch.from_numpy(rng.standard_normal((n, t)).astype(np.float32)).cuda())
        want = egp.kmm(X, V, ls, 1.1, 0.2, orc.RBF).clone()
        torch.cuda.synchronize()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want)
