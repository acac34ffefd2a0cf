"""End-to-end exact-GP regression on synthetic data with the library's entry points only.

The procedure of the paper's Experiment details: hyper-parameters are first fitted with Adam on a random subset
("pre-training"), refined with a few Adam steps on all points, then K̂⁻¹y is computed once with a tight CG
tolerance, a Lanczos variance cache is built, and predictive means and variances cost O(n) per test point.

    python -m paper_1903_08114_amd.examples.train_predict --n 65536 --d 8

Everything numerical runs in libegp.so on the GPU; torch holds the device buffers, numpy draws the data.
"""
from __future__ import annotations

import argparse
import time

import numpy as np


def synthetic_regression(n, d, seed=0, noise_std=0.1):
    """Points in [0,1]^d, a smooth target (random Fourier features) plus Gaussian noise, standardised."""
    rng = np.random.default_rng(seed)
    X = rng.uniform(0.0, 1.0, (n, d))
    W = rng.standard_normal((d, 64)) * 3.0
    b = rng.uniform(0.0, 2.0 * np.pi, 64)
    a = rng.standard_normal(64) / 8.0
    f = np.cos(X @ W + b) @ a
    y = f + noise_std * rng.standard_normal(n)
    mu, sd = y.mean(), y.std()
    return X.astype(np.float32), ((y - mu) / sd).astype(np.float32), ((f - mu) / sd).astype(np.float32), noise_std / sd


def rademacher(rng, shape):
    return (2.0 * rng.integers(0, 2, size=shape) - 1.0).astype(np.float32)


def fit_and_predict(X, y, Xq, kernel_type=0, rank=512, probes=16, subset=10000, pre_steps=30, full_steps=3, lr=0.1,
                    noise_floor=0.1, train_tol=1.0, train_iters=100, solve_tol=1e-2, solve_iters=1000,
                    cache_rank=256, exact_var=0, seed=0, verbose=True):
    """Returns dict with the fitted hyper-parameters, predictive mean and variance (numpy) and timings.
    exact_var > 0 (at most 32): the first exact_var test points also get their variance from a solve with the
    columns k(X, x*), returned as "var_exact" (the cached variance is an upper bound of it)."""
    import torch
    import paper_1903_08114_amd as egp
    rng = np.random.default_rng(seed)
    dev = torch.device("cuda:0")
    n, d = X.shape
    say = (lambda *a: print(*a, flush=True)) if verbose else (lambda *a: None)
    times = {}

    def cuda(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)

    ls = np.full(d, 0.5 * np.sqrt(d), np.float32)
    s, noise = 1.0, 0.5
    # ---- pre-training on a subset ----
    m = min(subset, n)
    idx = rng.choice(n, m, replace=False)
    r_sub = min(rank, m // 4)
    t0 = time.perf_counter()
    fit = egp.train_adam(cuda(X[idx]), cuda(y[idx]), cuda(rademacher(rng, (max(r_sub, 1), probes))),
                         cuda(rademacher(rng, (m, probes))), ls, s, noise, kernel_type, rank=r_sub,
                         max_iter=train_iters, tol=train_tol, steps=pre_steps, lr=lr, noise_floor=noise_floor)
    times["pretrain_s"] = time.perf_counter() - t0
    ls, s, noise = fit["lengthscales"].astype(np.float32), fit["outputscale"], fit["noise"]
    say(f"pre-training on {m} points: L/n {fit['mll_history'][0] / m:.4f} -> {fit['mll_history'][-1] / m:.4f}")
    # ---- a few steps on all points ----
    Xd, yd = cuda(X), cuda(y)
    if full_steps > 0 and n > m:
        t0 = time.perf_counter()
        fit = egp.train_adam(Xd, yd, cuda(rademacher(rng, (rank, probes))), cuda(rademacher(rng, (n, probes))), ls, s,
                             noise, kernel_type, rank=rank, max_iter=train_iters, tol=train_tol, steps=full_steps,
                             lr=lr, noise_floor=noise_floor)
        times["full_steps_s"] = time.perf_counter() - t0
        ls, s, noise = fit["lengthscales"].astype(np.float32), fit["outputscale"], fit["noise"]
        say(f"{full_steps} steps on all {n} points: L/n {fit['mll_history'][0] / n:.4f} -> {fit['mll_history'][-1] / n:.4f}")
    # ---- the one-time solve and the variance cache ----
    t0 = time.perf_counter()
    P = egp.piv_chol_precond(Xd, ls, s, noise, kernel_type, min(rank, n // 4))
    sol = egp.mbcg(Xd, yd[:, None].contiguous(), ls, s, noise, kernel_type, precond=P, max_iter=solve_iters,
                   tol=solve_tol)
    a = sol["U"][:, 0].contiguous()
    times["solve_s"] = time.perf_counter() - t0
    say(f"solve: {sol['iters']} iterations, relative residual {float(sol['rel_resid'].max()):.3g}")
    t0 = time.perf_counter()
    # variance cache: block Krylov space of [y | 15 random sign vectors] (one fused multiply per 16 basis vectors)
    B0 = np.concatenate([y[:, None], rademacher(rng, (n, 15))], axis=1)
    cache = egp.block_lanczos(Xd, cuda(B0), ls, s, noise, kernel_type, max(1, min(cache_rank, n) // 16))
    times["cache_s"] = time.perf_counter() - t0
    # ---- predictions ----
    Xqd = cuda(Xq)
    egp.predict(Xqd, Xd, a, ls, s, noise, kernel_type, cache=cache)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    mean, var = egp.predict(Xqd, Xd, a, ls, s, noise, kernel_type, cache=cache)
    torch.cuda.synchronize()
    times["predict_s"] = time.perf_counter() - t0
    out = {"lengthscales": ls, "outputscale": s, "noise": noise, "mean": mean.cpu().numpy(),
           "var": var.cpu().numpy(), "alpha": a, "solve_iters": sol["iters"], "times": times}
    if exact_var > 0:
        # s - k*^T Khat^{-1} k* with the solve done for real: the columns k(X, x*) come from a cross product with the
        # identity, the solve is the same preconditioned batched CG
        m = min(int(exact_var), 32, Xq.shape[0])
        t0 = time.perf_counter()
        Kq = egp.kmm_cross(Xd, Xqd[:m].contiguous(), torch.eye(m, dtype=torch.float32, device=dev), ls, s,
                           kernel_type)
        Uq = egp.mbcg(Xd, Kq, ls, s, noise, kernel_type, precond=P, max_iter=solve_iters, tol=solve_tol)["U"]
        out["var_exact"] = (s - (Kq * Uq).sum(dim=0)).cpu().numpy()
        times["exact_var_s"] = time.perf_counter() - t0
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=65536)
    ap.add_argument("--d", type=int, default=8)
    ap.add_argument("--nq", type=int, default=1000)
    ap.add_argument("--kernel", type=int, default=0, help="0 RBF, 1 Matern-3/2, 2 Matern-5/2, 3 Matern-1/2")
    ap.add_argument("--kmm-mode", default="fp32", choices=["fp32", "fp32_one_sided", "split_bf16", "split_bf16_all"],
                    help="arithmetic of the fused multiply: fp32 (default), fp32_one_sided (no use of the symmetry), "
                         "split_bf16, split_bf16_all")
    ap.add_argument("--rank", type=int, default=512,
                    help="preconditioner rank (the paper uses 100; here an iteration costs far more than applying the "
                         "preconditioner, so a higher rank pays)")
    ap.add_argument("--noise-floor", type=float, default=0.1,
                    help="lower bound of the learned noise variance (the paper keeps it at 0.1 on its largest sets)")
    ap.add_argument("--exact-var", type=int, default=32,
                    help="number of test points (at most 32) whose variance is also computed by a solve, to show how "
                         "far above it the cached upper bound sits")
    args = ap.parse_args()
    X, y, f, noise_std = synthetic_regression(args.n + args.nq, args.d)
    Xt, yt = X[:args.n], y[:args.n]
    Xq, yq, fq = X[args.n:], y[args.n:], f[args.n:]
    import paper_1903_08114_amd as egp
    egp.set_kmm_mode(args.kmm_mode)
    out = fit_and_predict(Xt, yt, Xq, kernel_type=args.kernel, rank=args.rank, noise_floor=args.noise_floor,
                          exact_var=args.exact_var)
    rmse = float(np.sqrt(np.mean((out["mean"] - yq) ** 2)))
    rmse_f = float(np.sqrt(np.mean((out["mean"] - fq) ** 2)))
    v = np.maximum(out["var"], 0.0) + out["noise"]
    nll = float(np.mean(0.5 * np.log(2 * np.pi * v) + 0.5 * (yq - out["mean"]) ** 2 / v))
    print(f"held-out RMSE {rmse:.4f} (noise level {noise_std:.4f}), RMSE against the noise-free target {rmse_f:.4f}, "
          f"NLL {nll:.4f}")
    if "var_exact" in out:
        m = len(out["var_exact"])
        ve = np.maximum(out["var_exact"], 0.0) + out["noise"]
        nll_e = float(np.mean(0.5 * np.log(2 * np.pi * ve) + 0.5 * (yq[:m] - out["mean"][:m]) ** 2 / ve))
        nll_c = float(np.mean(0.5 * np.log(2 * np.pi * v[:m]) + 0.5 * (yq[:m] - out["mean"][:m]) ** 2 / v[:m]))
        print(f"first {m} test points: mean latent variance {out['var_exact'].mean():.4f} by solve, "
              f"{out['var'][:m].mean():.4f} from the cache (an upper bound); NLL {nll_e:.4f} against {nll_c:.4f}")
    print("fitted noise", round(out["noise"], 4), "outputscale", round(out["outputscale"], 4))
    print("timings (s):", {k: round(v, 3) for k, v in out["times"].items()})


if __name__ == "__main__":
    main()
