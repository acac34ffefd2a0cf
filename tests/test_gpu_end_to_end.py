"""The whole path in one piece — fit, solve, cache, predict — on synthetic data small enough for the dense oracle:
the fitted model must predict as well as an exact GP with the same hyper-parameters, and must have learned."""
import numpy as np
import pytest

import oracle as orc

pytestmark = pytest.mark.gpu


def test_fit_solve_predict_matches_exact_gp():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1903_08114_amd.examples.train_predict import fit_and_predict, synthetic_regression
    n, nq, d = 3000, 400, 3
    X, y, f, noise_std = synthetic_regression(n + nq, d, seed=4)
    Xt, yt, Xq, yq = X[:n], y[:n], X[n:], y[n:]
    out = fit_and_predict(Xt, yt, Xq, kernel_type=orc.RBF, rank=40, probes=16, subset=1500, pre_steps=40,
                          full_steps=3, train_tol=1e-2, train_iters=200, solve_tol=1e-4, cache_rank=150,
                          noise_floor=1e-4, exact_var=32, verbose=False)
    h = orc.Hyper(orc.RBF, out["lengthscales"], out["outputscale"], out["noise"])
    mean_ref, var_ref = orc.predict_exact(Xt, yt, Xq, h)
    # same hyper-parameters, exact dense GP: means agree, cached variances sit just above the exact ones
    assert np.abs(out["mean"] - mean_ref).max() <= 5e-3 * max(1.0, np.abs(mean_ref).max())
    assert np.all(out["var"] >= var_ref - 5e-3)
    assert np.mean(out["var"] - var_ref) <= 0.05 * out["outputscale"]
    # variances from a solve with the columns k(X, x*): the exact ones up to the solve's tolerance
    assert out["var_exact"].shape == (32,)
    assert np.abs(out["var_exact"] - var_ref[:32]).max() <= 2e-3 * out["outputscale"]
    # it has learned: held-out error close to the noise level, far below predicting the mean (standardised y: 1.0)
    rmse = float(np.sqrt(np.mean((out["mean"] - yq) ** 2)))
    assert rmse <= 1.5 * noise_std + 0.05, (rmse, noise_std)
    assert rmse <= 0.6
    # and the fitted likelihood beats the start values'
    start = orc.Hyper(orc.RBF, np.full(d, 0.5 * np.sqrt(d)), 1.0, 0.5)
    assert orc.mll(Xt, yt, h) > orc.mll(Xt, yt, start)
