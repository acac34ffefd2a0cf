"""MI355X-native exact-GP hot path: fused kernel-matrix multiply, pivoted-Cholesky preconditioner, mBCG.

Thin ctypes binding over libegp.so (argument marshalling only; every step runs in HIP kernels).
"""
from .binding import (EGP_RBF, EGP_MATERN32, EGP_MATERN52, EGP_MATERN12, EgpError, Precond, kmm, kmm_noalloc, kmm_grad, kmm_grad_bilinear, piv_chol_precond,
                      precond_apply, mbcg, mll, tridiag_logquad, kmm_cross, lanczos, predict,
                      LanczosCache, BlockCache, block_lanczos, train_adam, lib, lib_path, set_workspace_guard, set_kmm_mode, KMM_MODES)

__all__ = ["EGP_RBF", "EGP_MATERN32", "EGP_MATERN52", "EGP_MATERN12", "EgpError", "Precond", "kmm", "kmm_noalloc", "kmm_grad", "kmm_grad_bilinear", "piv_chol_precond",
           "precond_apply", "mbcg", "mll", "tridiag_logquad", "kmm_cross", "lanczos",
           "predict", "LanczosCache", "BlockCache", "block_lanczos", "train_adam", "lib", "lib_path",
           "set_workspace_guard", "set_kmm_mode", "KMM_MODES"]
