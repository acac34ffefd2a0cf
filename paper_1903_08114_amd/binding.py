"""ctypes binding of libegp.so. Tensors are torch CUDA (ROCm) tensors used only as device buffers."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
EGP_RBF, EGP_MATERN32, EGP_MATERN52, EGP_MATERN12 = 0, 1, 2, 3

_lib = None


class EgpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libegp error {code}: {msg}")
        self.code = code


class _Hyper(C.Structure):
    _fields_ = [("kernel_type", C.c_int32), ("d", C.c_int32), ("lengthscales", C.POINTER(C.c_float)),
                ("outputscale", C.c_float), ("noise", C.c_float)]


class _MllResult(C.Structure):
    _fields_ = [("mll", C.c_double), ("logdet", C.c_double), ("quad", C.c_double), ("grad", C.c_double * 401),
                ("iters", C.c_int32), ("precond_rank", C.c_int32), ("rel_resid_max", C.c_float)]


class _Adam(C.Structure):
    _fields_ = [("steps", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("noise_floor", C.c_float)]


class _CallOpts(C.Structure):
    _fields_ = [("kmm_mode", C.c_int32), ("mbcg_shrink", C.c_int32)]


class _Precond(C.Structure):
    _fields_ = [("rank", C.c_int32), ("L", C.c_void_p), ("pivots", C.POINTER(C.c_int32)),
                ("small", C.POINTER(C.c_double)), ("small_dev", C.c_void_p)]


def lib_path() -> str:
    return os.path.join(HERE, "libegp.so")


def lib():
    """Load libegp.so (built in-tree by paper_1903_08114_amd.build). Fails loudly when absent."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_1903_08114_amd.build` first; "
                              "there is no CPU fallback")
        # torch first: it ships its own HIP runtime, and the device buffers this library works on are torch's. Loaded
        # the other way round, libegp.so binds the system runtime and then sees no device of torch's process state
        # ("no ROCm-capable device is detected" from the first launch).
        import torch  # noqa: F401
        L = C.CDLL(path)
        L.egp_last_error.restype = C.c_char_p
        L.egp_version.restype = C.c_char_p
        for name in ("egp_kmm_ws_bytes", "egp_piv_chol_precond_ws_bytes", "egp_mbcg_ws_bytes",
                     "egp_precond_apply_ws_bytes"):
            getattr(L, name).restype = C.c_size_t
        L.egp_piv_chol_precond_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.egp_mbcg_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.egp_precond_apply_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.egp_piv_chol_precond.restype = C.c_int
        L.egp_piv_chol_precond.argtypes = [C.c_void_p, C.c_int64, C.POINTER(_Hyper), C.c_float,
                                           C.POINTER(_Precond), C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_precond_apply.restype = C.c_int
        L.egp_precond_apply.argtypes = [C.POINTER(_Precond), C.c_int64, C.c_float, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_mbcg.restype = C.c_int
        L.egp_mbcg.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.POINTER(_Hyper),
                               C.POINTER(_Precond), C.c_int32, C.c_float, C.c_void_p,
                               C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int32),
                               C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_kmm_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.egp_kmm_grad_bilinear_ws_bytes.restype = C.c_size_t
        L.egp_kmm_grad_bilinear_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.egp_kmm_grad_bilinear.restype = C.c_int
        L.egp_kmm_grad_bilinear.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32,
                                            C.POINTER(C.c_float), C.POINTER(_Hyper), C.POINTER(C.c_double),
                                            C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_kmm_cross_ws_bytes.restype = C.c_size_t
        L.egp_kmm_cross_ws_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32]
        L.egp_kmm_plan_splits.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                          C.POINTER(C.c_int32)]
        L.egp_kmm_cross.restype = C.c_int
        L.egp_kmm_cross.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                    C.POINTER(_Hyper), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_lanczos_ws_bytes.restype = C.c_size_t
        L.egp_lanczos_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.egp_lanczos.restype = C.c_int
        L.egp_lanczos.argtypes = [C.c_void_p, C.c_int64, C.POINTER(_Hyper), C.c_void_p, C.c_int32, C.c_void_p,
                                  C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_void_p,
                                  C.c_size_t, C.c_void_p]
        L.egp_predict_ws_bytes.restype = C.c_size_t
        L.egp_predict_ws_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32]
        L.egp_predict.restype = C.c_int
        L.egp_predict.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.POINTER(_Hyper), C.c_void_p,
                                  C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_mll_ws_bytes.restype = C.c_size_t
        L.egp_mll_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.egp_mll.restype = C.c_int
        L.egp_mll.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                              C.POINTER(_Hyper), C.c_int32, C.c_int32, C.c_float, C.POINTER(_MllResult),
                              C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_train_adam.restype = C.c_int
        L.egp_train_adam.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                     C.c_int32, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float),
                                     C.POINTER(C.c_float), C.c_int32, C.c_int32, C.c_float, C.POINTER(_Adam),
                                     C.POINTER(_MllResult), C.POINTER(C.c_double), C.c_void_p, C.c_size_t,
                                     C.c_void_p]
        L.egp_block_lanczos.restype = C.c_int
        L.egp_block_lanczos.argtypes = [C.c_void_p, C.c_int64, C.POINTER(_Hyper), C.c_void_p, C.c_int32, C.c_int32,
                                        C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_void_p,
                                        C.c_size_t, C.c_void_p]
        L.egp_block_lanczos_ws_bytes.restype = C.c_size_t
        L.egp_block_lanczos_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32]
        L.egp_predict_dense.restype = C.c_int
        L.egp_predict_dense.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.POINTER(_Hyper), C.c_void_p,
                                        C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.c_int32, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_tridiag_logquad.restype = C.c_int
        L.egp_tridiag_logquad.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int32,
                                          C.POINTER(C.c_double)]
        L.egp_kmm_grad_ws_bytes.restype = C.c_size_t
        L.egp_kmm_grad_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.egp_kmm_grad.restype = C.c_int
        L.egp_kmm_grad.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.POINTER(_Hyper), C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]
        L.egp_kmm.restype = C.c_int
        L.egp_kmm.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.POINTER(_Hyper), C.c_void_p,
                              C.c_void_p, C.c_size_t, C.c_void_p]
        opts = [C.POINTER(_CallOpts)]
        L.egp_kmm_ex.restype = C.c_int
        L.egp_kmm_ex.argtypes = L.egp_kmm.argtypes + opts
        L.egp_mbcg_ex.restype = C.c_int
        L.egp_mbcg_ex.argtypes = L.egp_mbcg.argtypes + opts
        L.egp_mll_ex.restype = C.c_int
        L.egp_mll_ex.argtypes = L.egp_mll.argtypes + opts
        L.egp_train_adam_ex.restype = C.c_int
        L.egp_train_adam_ex.argtypes = L.egp_train_adam.argtypes + opts
        L.egp_kmm_plan_splits_ex.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.POINTER(_CallOpts),
                                             C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.egp_kmm_noalloc.restype = C.c_int
        L.egp_kmm_noalloc.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.POINTER(_Hyper), C.c_void_p,
                                      C.c_void_p]
        _lib = L
    return _lib


# Debug aid for tests: with a guard of G bytes set, every workspace this module allocates is followed by G bytes
# of a fill pattern, verified after the library call that used it. A kernel writing past its workspace then
# raises here instead of corrupting a neighbouring tensor.
_GUARD_FILL = 0x5A
_guard_bytes = int(os.environ.get("EGP_WS_GUARD_BYTES", "0"))
_guards = []


def set_workspace_guard(nbytes):
    """Set the number of guard bytes behind each workspace allocated by this module (0 switches the check off)."""
    global _guard_bytes
    _guard_bytes = max(int(nbytes), 0)
    _guards.clear()


def _verify_guards():
    import torch
    pending, _guards[:] = list(_guards), []
    for buf, used in pending:
        torch.cuda.synchronize(buf.device)
        if not bool((buf[used:] == _GUARD_FILL).all()):
            bad = int((buf[used:] != _GUARD_FILL).nonzero()[0])
            raise EgpError(-2, f"workspace overrun: byte {bad} behind a workspace of {used} bytes was overwritten")


def _check(rc):
    if _guards:
        _verify_guards()
    if rc != 0:
        raise EgpError(rc, lib().egp_last_error().decode())


KMM_MODES = {"fp32": 0, "split_bf16": 1, "split_bf16_all": 2, "fp32_one_sided": 3}


def set_kmm_mode(mode):
    """Select the arithmetic of the fused multiply for every later call in this process (egp_set_kmm_mode):
    "fp32" (default: fp32 throughout; large square products use every off-diagonal tile for both output sides),
    "fp32_one_sided" (fp32 with every tile formed: same results up to summation order, slower; for comparison),
    "split_bf16", "split_bf16_all" (contractions on the bf16 MFMA through exact bf16 splits). All modes are
    bit-reproducible. Accepts the name or the integer code; returns the previous code."""
    L = lib()
    code = KMM_MODES[mode] if isinstance(mode, str) else int(mode)
    prev = int(L.egp_get_kmm_mode())
    _check(L.egp_set_kmm_mode(C.c_int32(code)))
    return prev


def _opts(mode=None, shrink=None):
    """egp_call_opts_t for one call: the arithmetic mode (name, code or None = process default) and column shrinking
    (True, False or None = process default)."""
    code = -1 if mode is None else (KMM_MODES[mode] if isinstance(mode, str) else int(mode))
    return _CallOpts(code, -1 if shrink is None else (1 if shrink else 0))


def _hyper(kernel_type, lengthscales, outputscale, noise):
    ls = [float(v) for v in lengthscales]
    arr = (C.c_float * len(ls))(*ls)
    h = _Hyper(int(kernel_type), len(ls), C.cast(arr, C.POINTER(C.c_float)), float(outputscale), float(noise))
    h._keep = arr
    return h


def _dev(tensor, name):
    import torch
    if not (isinstance(tensor, torch.Tensor) and tensor.is_cuda and tensor.dtype == torch.float32
            and tensor.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous float32 tensor on the GPU")
    return C.c_void_p(tensor.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes, device):
    import torch
    nbytes = max(int(nbytes), 256)
    if _guard_bytes == 0:
        return torch.empty(nbytes, dtype=torch.uint8, device=device)
    used = (nbytes + 255) // 256 * 256
    buf = torch.empty(used + _guard_bytes, dtype=torch.uint8, device=device)
    buf[used:].fill_(_GUARD_FILL)
    _guards.append((buf, used))
    return buf[:nbytes]


class Precond:
    """Buffers of a rank-k pivoted-Cholesky preconditioner P = L L^T + noise I (filled by piv_chol_precond).

    L: (rank, n) float32 CUDA tensor (column m of the factor is row m here); pivots: numpy int32;
    chol_small: (rank, rank) float64 lower factor of noise I + L^T L; logdet: log|P|."""

    def __init__(self, n, capacity, device):
        import numpy as np
        import torch
        self.n, self.capacity, self.rank = int(n), int(capacity), 0
        self.L_buf = torch.empty((capacity, n), dtype=torch.float32, device=device)
        self.small_dev = torch.empty((capacity * capacity,), dtype=torch.float64, device=device)
        self._pivots = np.zeros(capacity, dtype=np.int32)
        self._small = np.zeros(capacity * capacity + 1, dtype=np.float64)
        self.noise = None

    def _struct(self, rank):
        return _Precond(int(rank), C.c_void_p(self.L_buf.data_ptr()),
                        self._pivots.ctypes.data_as(C.POINTER(C.c_int32)),
                        self._small.ctypes.data_as(C.POINTER(C.c_double)),
                        C.c_void_p(self.small_dev.data_ptr()))

    @property
    def L(self):
        return self.L_buf[:self.rank]

    @property
    def pivots(self):
        return self._pivots[:self.rank].copy()

    @property
    def chol_small(self):
        k = self.rank
        return self._small[:k * k].reshape(k, k).copy()

    @property
    def logdet(self):
        return float(self._small[self.capacity * self.capacity])


def kmm(X, V, lengthscales, outputscale, noise, kernel_type, out=None, ws=None, mode=None):
    """out = K(X,X) V + noise V on the GPU (egp_kmm_ex). X: (n,d), V: (n,t) float32 CUDA tensors.
    mode: arithmetic of this call (a KMM_MODES name or code); None takes the process default (set_kmm_mode)."""
    import torch
    L = lib()
    n, d = X.shape
    t = V.shape[1]
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    if out is None:
        out = torch.empty_like(V)
    need = L.egp_kmm_ws_bytes(n, d, t)
    if ws is None:
        ws = _workspace(need, X.device)
    o = _opts(mode)
    _check(L.egp_kmm_ex(_dev(X, "X"), n, _dev(V, "V"), t, C.byref(h), _dev(out, "out"),
                        C.c_void_p(ws.data_ptr()), ws.numel(), _stream(), C.byref(o)))
    return out


def kmm_noalloc(X, V, lengthscales, outputscale, noise, kernel_type, out=None):
    """egp_kmm_noalloc: the same product with the library's built-in scratch array as workspace (no workspace is
    allocated or passed; sizes beyond the array raise EgpError). `out` is still the caller's."""
    import torch
    L = lib()
    n, d = X.shape
    t = V.shape[1]
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    if out is None:
        out = torch.empty_like(V)
    _check(L.egp_kmm_noalloc(_dev(X, "X"), n, _dev(V, "V"), t, C.byref(h), _dev(out, "out"), _stream()))
    return out


def kmm_grad(X, V, lengthscales, outputscale, noise, kernel_type, out=None, ws=None):
    """out[k] = (dK/dl_k) V for every lengthscale (egp_kmm_grad). Returns a (d, n, t) tensor."""
    import torch
    L = lib()
    n, d = X.shape
    t = V.shape[1]
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    if out is None:
        out = torch.empty((d, n, t), dtype=torch.float32, device=X.device)
    need = L.egp_kmm_grad_ws_bytes(n, d, t)
    if ws is None:
        ws = _workspace(need, X.device)
    _check(L.egp_kmm_grad(_dev(X, "X"), n, _dev(V, "V"), t, C.byref(h), _dev(out, "dout"),
                          C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return out


def kmm_grad_bilinear(X, A, B, lengthscales, outputscale, noise, kernel_type, weights=None, ws=None):
    """sum_c w_c A[:,c]^T (dK/dl_k) B[:,c] for every lengthscale, then sum_c w_c A[:,c]^T K B[:,c] / outputscale
    (egp_kmm_grad_bilinear). Returns a float64 array of d + 1 values."""
    import numpy as np
    L = lib()
    n, d = X.shape
    t = A.shape[1]
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    need = L.egp_kmm_grad_bilinear_ws_bytes(n, d, t)
    if ws is None:
        ws = _workspace(need, X.device)
    out = np.zeros(d + 1, dtype=np.float64)
    wp = None
    if weights is not None:
        warr = (C.c_float * t)(*[float(v) for v in weights])
        wp = C.cast(warr, C.POINTER(C.c_float))
    _check(L.egp_kmm_grad_bilinear(_dev(X, "X"), n, _dev(A, "A"), _dev(B, "B"), t, wp, C.byref(h),
                                   out.ctypes.data_as(C.POINTER(C.c_double)), C.c_void_p(ws.data_ptr()),
                                   ws.numel(), _stream()))
    return out


def piv_chol_precond(X, lengthscales, outputscale, noise, kernel_type, rank, tol_abs=0.0, ws=None):
    """Rank-`rank` pivoted-Cholesky preconditioner of K(X,X) (egp_piv_chol_precond). Returns a Precond."""
    L = lib()
    n, d = X.shape
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    P = Precond(n, rank, X.device)
    st = P._struct(rank)
    need = L.egp_piv_chol_precond_ws_bytes(n, d, rank)
    if ws is None:
        ws = _workspace(need, X.device)
    _check(L.egp_piv_chol_precond(_dev(X, "X"), n, C.byref(h), float(tol_abs), C.byref(st),
                                  C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    P.rank = int(st.rank)
    P.noise = float(noise)
    return P


def precond_apply(P, R, noise=None, out=None, ws=None):
    """Z = P^{-1} R (egp_precond_apply)."""
    import torch
    L = lib()
    n, t = R.shape
    if out is None:
        out = torch.empty_like(R)
    need = L.egp_precond_apply_ws_bytes(n, t, max(P.rank, 1))
    if ws is None:
        ws = _workspace(need, R.device)
    st = P._struct(P.rank)
    _check(L.egp_precond_apply(C.byref(st), n, float(P.noise if noise is None else noise), _dev(R, "R"), t,
                               _dev(out, "Z"), C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return out


def mbcg(X, B, lengthscales, outputscale, noise, kernel_type, precond=None, max_iter=100, tol=1e-2, ws=None,
         shrink=None, mode=None):
    """Batched PCG solve of (K + noise I) U = B (egp_mbcg_ex).

    mode: arithmetic of the multiplies of this call (None = process default).
    shrink=True (a per-call option): trailing columns that have met the tolerance leave
    the iteration, so with B = [y | probes] and y the slowest column the late iterations run on fewer columns.
    Returns dict: U (n,t) tensor, iters, rel_resid (t,), alphas/betas (iters,t) float64, gamma0 (t,), col_iters (t,)
    = iterations each column took part in."""
    import numpy as np
    import torch
    L = lib()
    n, d = X.shape
    t = B.shape[1]
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    U = torch.empty_like(B)
    rank = precond.rank if precond is not None else 0
    need = L.egp_mbcg_ws_bytes(n, d, t, rank, max_iter)
    if ws is None:
        ws = _workspace(need, X.device)
    coef = np.zeros((max(max_iter, 1), 2, t), dtype=np.float64)
    gamma0 = np.zeros(t, dtype=np.float64)
    iters = C.c_int32(0)
    rel = np.zeros(t, dtype=np.float32)
    hist = np.zeros((max(max_iter, 1), t), dtype=np.float32)
    st = precond._struct(precond.rank) if precond is not None else None
    o = _opts(mode, shrink)
    _check(L.egp_mbcg_ex(_dev(X, "X"), n, _dev(B, "B"), t, C.byref(h), C.byref(st) if st is not None else None,
                         int(max_iter), float(tol), _dev(U, "U"), coef.ctypes.data_as(C.POINTER(C.c_double)),
                         gamma0.ctypes.data_as(C.POINTER(C.c_double)), C.byref(iters),
                         rel.ctypes.data_as(C.POINTER(C.c_float)), hist.ctypes.data_as(C.POINTER(C.c_float)),
                         C.c_void_p(ws.data_ptr()), ws.numel(), _stream(), C.byref(o)))
    m = int(iters.value)
    alphas = coef[:m, 0, :].copy()
    return {"U": U, "iters": m, "rel_resid": rel, "alphas": alphas,
            "betas": coef[:m, 1, :].copy(), "gamma0": gamma0, "resid_hist": hist[:m].copy(),
            "col_iters": (alphas != 0.0).sum(axis=0).astype(np.int64)}


def mll(X, y, W1, W2, lengthscales, outputscale, noise, kernel_type, rank=100, max_iter=100, tol=1.0, ws=None,
        shrink=None, mode=None):
    """Log marginal likelihood and gradient w.r.t. (lengthscales, outputscale, noise) (egp_mll_ex).
    shrink: as in mbcg (a probe's Lanczos tridiagonal then ends where the probe met the tolerance, which truncates
    the quadrature of the log-determinant: at loose tolerances the value shifts by several per cent); mode: as in kmm.

    y: (n,), W1: (rank, tp) and W2: (n, tp) Rademacher draws, all float32 CUDA tensors. Returns a dict."""
    import numpy as np
    L = lib()
    n, d = X.shape
    tp = W2.shape[1]
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    need = L.egp_mll_ws_bytes(n, d, tp, rank, max_iter)
    if ws is None:
        ws = _workspace(need, X.device)
    res = _MllResult()
    o = _opts(mode, shrink)
    _check(L.egp_mll_ex(_dev(X, "X"), n, _dev(y, "y"), _dev(W1, "W1") if rank > 0 else None, _dev(W2, "W2"), tp,
                        C.byref(h), int(rank), int(max_iter), float(tol), C.byref(res),
                        C.c_void_p(ws.data_ptr()), ws.numel(), _stream(), C.byref(o)))
    return {"mll": res.mll, "logdet": res.logdet, "quad": res.quad,
            "grad": np.array(res.grad[:d + 2], dtype=np.float64), "iters": res.iters,
            "rank": res.precond_rank, "rel_resid_max": res.rel_resid_max}


def tridiag_logquad(diag, off):
    """e1^T log(T) e1 for a symmetric positive definite tridiagonal T (host-only helper, egp_tridiag_logquad)."""
    import numpy as np
    diag = np.ascontiguousarray(diag, dtype=np.float64)
    off = np.ascontiguousarray(off, dtype=np.float64)
    out = C.c_double(0.0)
    _check(lib().egp_tridiag_logquad(diag.ctypes.data_as(C.POINTER(C.c_double)),
                                     off.ctypes.data_as(C.POINTER(C.c_double)) if len(off) else None,
                                     len(diag), C.byref(out)))
    return out.value


def kmm_cross(Xq, X, V, lengthscales, outputscale, kernel_type, out=None, ws=None):
    """out (nq x t) = K(Xq, X) V, no noise term (egp_kmm_cross)."""
    import torch
    L = lib()
    nq, d = Xq.shape
    n = X.shape[0]
    t = V.shape[1]
    h = _hyper(kernel_type, lengthscales, outputscale, 0.0)
    if out is None:
        out = torch.empty((nq, t), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = _workspace(L.egp_kmm_cross_ws_bytes(nq, n, d, t), X.device)
    _check(L.egp_kmm_cross(_dev(Xq, "Xq"), nq, _dev(X, "X"), n, _dev(V, "V"), t, C.byref(h), _dev(out, "out"),
                           C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return out


class LanczosCache:
    """Q (steps, n) float32 CUDA tensor with orthonormal rows and the tridiagonal T = Q Khat Q^T (alpha, beta)."""

    def __init__(self, Q, alpha, beta, steps):
        self.Q, self.alpha, self.beta, self.steps = Q, alpha, beta, steps


def lanczos(X, b, lengthscales, outputscale, noise, kernel_type, r, ws=None):
    """r Lanczos steps on K + noise I from the start vector b (egp_lanczos). Returns a LanczosCache."""
    import numpy as np
    import torch
    L = lib()
    n, d = X.shape
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    Q = torch.zeros((r, n), dtype=torch.float32, device=X.device)
    alpha = np.zeros(r, dtype=np.float64)
    beta = np.zeros(max(r - 1, 1), dtype=np.float64)
    steps = C.c_int32(0)
    if ws is None:
        ws = _workspace(L.egp_lanczos_ws_bytes(n, d, r), X.device)
    _check(L.egp_lanczos(_dev(X, "X"), n, C.byref(h), _dev(b, "b"), int(r), _dev(Q, "Q"),
                         alpha.ctypes.data_as(C.POINTER(C.c_double)), beta.ctypes.data_as(C.POINTER(C.c_double)),
                         C.byref(steps), C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    m = int(steps.value)
    return LanczosCache(Q[:m], alpha[:m].copy(), beta[:max(m - 1, 0)].copy(), m)


class BlockCache:
    """Q (rows, n) float32 CUDA tensor with orthonormal rows and the dense projected matrix T = Q Khat Q^T."""

    def __init__(self, Q, T, steps):
        self.Q, self.T, self.steps = Q, T, steps


def block_lanczos(X, B0, lengthscales, outputscale, noise, kernel_type, blocks, ws=None):
    """Variance cache from a block of start vectors B0 (n, b), b <= 32 (egp_block_lanczos). Returns a BlockCache with
    up to b * blocks basis vectors; one fused multiply per block."""
    import numpy as np
    import torch
    L = lib()
    n, d = X.shape
    b = B0.shape[1]
    rcap = b * int(blocks)
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    Q = torch.zeros((rcap, n), dtype=torch.float32, device=X.device)
    T = np.zeros((rcap, rcap), dtype=np.float64)
    rows = C.c_int32(0)
    if ws is None:
        ws = _workspace(L.egp_block_lanczos_ws_bytes(n, d, b, int(blocks)), X.device)
    _check(L.egp_block_lanczos(_dev(X, "X"), n, C.byref(h), _dev(B0, "B0"), b, int(blocks), _dev(Q, "Q"),
                               T.ctypes.data_as(C.POINTER(C.c_double)), C.byref(rows),
                               C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    m = int(rows.value)
    return BlockCache(Q[:m], np.ascontiguousarray(T[:m, :m]), m)


def predict(Xq, X, a, lengthscales, outputscale, noise, kernel_type, cache=None, ws=None):
    """Predictive mean K(Xq,X) a and, with a LanczosCache, the cached predictive variance (egp_predict).
    Returns (mean, var) float32 CUDA tensors of length nq (var is None without a cache)."""
    import numpy as np
    import torch
    L = lib()
    nq, d = Xq.shape
    n = X.shape[0]
    h = _hyper(kernel_type, lengthscales, outputscale, noise)
    mean = torch.empty(nq, dtype=torch.float32, device=X.device)
    r = cache.steps if cache is not None else 0
    var = torch.empty(nq, dtype=torch.float32, device=X.device) if cache is not None else None
    if ws is None:
        ws = _workspace(L.egp_predict_ws_bytes(nq, n, d, r), X.device)
    if isinstance(cache, BlockCache):
        Q = cache.Q.contiguous()
        T = np.ascontiguousarray(cache.T, dtype=np.float64)
        _check(L.egp_predict_dense(_dev(Xq, "Xq"), nq, _dev(X, "X"), n, C.byref(h), _dev(a, "a"), _dev(Q, "Q"), r,
                                   T.ctypes.data_as(C.POINTER(C.c_double)), r, _dev(mean, "mean"), _dev(var, "var"),
                                   C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    elif cache is not None:
        Q = cache.Q.contiguous()
        al = np.ascontiguousarray(cache.alpha, dtype=np.float64)
        be = np.ascontiguousarray(cache.beta if r > 1 else np.zeros(1), dtype=np.float64)
        _check(L.egp_predict(_dev(Xq, "Xq"), nq, _dev(X, "X"), n, C.byref(h), _dev(a, "a"), _dev(Q, "Q"), r,
                             al.ctypes.data_as(C.POINTER(C.c_double)), be.ctypes.data_as(C.POINTER(C.c_double)),
                             _dev(mean, "mean"), _dev(var, "var"), C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    else:
        _check(L.egp_predict(_dev(Xq, "Xq"), nq, _dev(X, "X"), n, C.byref(h), _dev(a, "a"), None, 0, None, None,
                             _dev(mean, "mean"), None, C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return mean, var


def train_adam(X, y, W1, W2, lengthscales, outputscale, noise, kernel_type, rank=100, max_iter=100, tol=1.0,
               steps=3, lr=0.1, noise_floor=0.0, beta1=0.9, beta2=0.999, eps=1e-8, ws=None, shrink=None, mode=None):
    """`steps` Adam ascent steps on the log marginal likelihood (egp_train_adam_ex). shrink, mode: as in mll.
    Returns dict: lengthscales, outputscale, noise (fitted), mll_history (steps + 1), last (final evaluation)."""
    import numpy as np
    L = lib()
    n, d = X.shape
    tp = W2.shape[1]
    ls = (C.c_float * d)(*[float(v) for v in lengthscales])
    s_io, n_io = C.c_float(float(outputscale)), C.c_float(float(noise))
    opt = _Adam(int(steps), float(lr), float(beta1), float(beta2), float(eps), float(noise_floor))
    res = _MllResult()
    hist = np.zeros(steps + 1, dtype=np.float64)
    if ws is None:
        ws = _workspace(L.egp_mll_ws_bytes(n, d, tp, rank, max_iter), X.device)
    o = _opts(mode, shrink)
    _check(L.egp_train_adam_ex(_dev(X, "X"), n, _dev(y, "y"), _dev(W1, "W1") if rank > 0 else None, _dev(W2, "W2"),
                               tp, int(kernel_type), d, ls, C.byref(s_io), C.byref(n_io), int(rank), int(max_iter),
                               float(tol), C.byref(opt), C.byref(res), hist.ctypes.data_as(C.POINTER(C.c_double)),
                               C.c_void_p(ws.data_ptr()), ws.numel(), _stream(), C.byref(o)))
    return {"lengthscales": np.array(list(ls), dtype=np.float64), "outputscale": float(s_io.value),
            "noise": float(n_io.value), "mll_history": hist,
            "last": {"mll": res.mll, "grad": np.array(res.grad[:d + 2]), "iters": res.iters}}
