"""ctypes binding of libegp.so. Tensors are torch CUDA (ROCm) tensors used only as device buffers."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
EGP_RBF, EGP_MATERN32, EGP_MATERN52 = 0, 1, 2

_lib = None


class EgpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libegp error {code}: {msg}")
        self.code = code


class _Hyper(C.Structure):
    _fields_ = [("kernel_type", C.c_int32), ("d", C.c_int32), ("lengthscales", C.POINTER(C.c_float)),
                ("outputscale", C.c_float), ("noise", C.c_float)]


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
        L = C.CDLL(path)
        L.egp_last_error.restype = C.c_char_p
        L.egp_version.restype = C.c_char_p
        for name in ("egp_kmm_ws_bytes",):
            getattr(L, name).restype = C.c_size_t
        L.egp_kmm_ws_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.egp_kmm.restype = C.c_int
        L.egp_kmm.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.POINTER(_Hyper), C.c_void_p,
                              C.c_void_p, C.c_size_t, C.c_void_p]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise EgpError(rc, lib().egp_last_error().decode())


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
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class Precond:
    """Buffers of a rank-k pivoted-Cholesky preconditioner (filled by piv_chol_precond)."""
    pass


def kmm(X, V, lengthscales, outputscale, noise, kernel_type, out=None, ws=None):
    """out = K(X,X) V + noise V on the GPU (egp_kmm). X: (n,d), V: (n,t) float32 CUDA tensors."""
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
    _check(L.egp_kmm(_dev(X, "X"), n, _dev(V, "V"), t, C.byref(h), _dev(out, "out"),
                     C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return out
