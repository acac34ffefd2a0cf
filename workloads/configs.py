"""Generators for the five benchmark configurations (C1..C5) and small test inputs."""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

RBF, MATERN32, MATERN52, MATERN12 = 0, 1, 2, 3
CONFIG_NAMES = ("C1", "C2", "C3", "C4", "C5")


def base_seed(index: int) -> int:
    """Seed of configuration `index` (1..5)."""
    return 190308114 * 10 + index


@dataclass
class Workload:
    name: str
    X: np.ndarray                 # (n, d) float32
    y: np.ndarray | None          # (n,) float32 or None
    V: np.ndarray                 # (n, t) float32 right-hand sides / multiplicand
    kernel_type: int
    lengthscales: np.ndarray      # (d,) float32
    outputscale: float
    noise: float                  # sigma^2, the value added to the diagonal
    rank: int                     # preconditioner rank the config asks for
    tol: float
    max_iter: int
    notes: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return self.X.shape[0]

    @property
    def d(self) -> int:
        return self.X.shape[1]

    @property
    def t(self) -> int:
        return self.V.shape[1]


def rademacher(rng: np.random.Generator, shape) -> np.ndarray:
    return (2.0 * rng.integers(0, 2, size=shape) - 1.0).astype(np.float32)


def _standardise(a: np.ndarray) -> np.ndarray:
    return (a - a.mean(axis=0)) / a.std(axis=0)


def _log_uniform(rng, lo, hi, size):
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=size))


def _mixture_points(rng, n, d, components=32):
    """Clustered sensor-style inputs: equal-weight isotropic Gaussian mixture clipped to [0,1]^d."""
    means = rng.uniform(0.15, 0.85, size=(components, d))
    stds = rng.uniform(0.03, 0.10, size=components)
    comp = rng.integers(0, components, size=n)
    X = means[comp] + stds[comp, None] * rng.standard_normal((n, d))
    return np.clip(X, 0.0, 1.0)


def _fourier_target(rng, X, features=512, omega_std=4.0, noise_std=0.1, chunk=65536):
    d = X.shape[1]
    omega = omega_std * rng.standard_normal((d, features))
    phase = rng.uniform(0.0, 2.0 * np.pi, size=features)
    amp = rng.standard_normal(features)
    out = np.empty(X.shape[0])
    for s in range(0, X.shape[0], chunk):
        out[s:s + chunk] = np.cos(X[s:s + chunk] @ omega + phase) @ amp
    out *= np.sqrt(2.0 / features)
    out += noise_std * rng.standard_normal(X.shape[0])
    return _standardise(out)


def make_workload(name: str, n: int | None = None, with_targets: bool = True) -> Workload:
    """Build configuration `name` in {"C1".."C5"}; `n` overrides the point count (same recipe)."""
    idx = CONFIG_NAMES.index(name) + 1
    rng = np.random.default_rng(base_seed(idx))
    if name == "C1":
        n = n or 4096
        d = 8
        X = rng.uniform(0.0, 1.0, size=(n, d))
        y = np.sin(3.0 * X).sum(axis=1) + 0.1 * rng.standard_normal(n)
        V = np.concatenate([y[:, None].astype(np.float32), rademacher(rng, (n, 15))], axis=1)
        return Workload(name, X.astype(np.float32), y.astype(np.float32), V, RBF,
                        np.full(d, 0.5, np.float32), 1.0, 0.01, rank=5, tol=0.0, max_iter=20)
    if name == "C2":
        n = n or 65536
        d = 18
        X = _standardise(rng.standard_normal((n, d)))
        a = rng.standard_normal(d) / np.sqrt(d)
        b = rng.standard_normal(d) / np.sqrt(d)
        y = _standardise(X @ a + 0.5 * np.sin(X @ b) + 0.05 * rng.standard_normal(n))
        ls = _log_uniform(rng, 0.3, 3.0, d)
        V = np.concatenate([y[:, None].astype(np.float32), rademacher(rng, (n, 16))], axis=1)
        return Workload(name, X.astype(np.float32), y.astype(np.float32), V, MATERN52,
                        ls.astype(np.float32), 1.0, 0.01, rank=20, tol=1e-2, max_iter=500)
    if name == "C3":
        n = n or 262144
        d = 25
        X = rng.uniform(-1.0, 1.0, size=(n, d))
        ls = _log_uniform(rng, 0.5, 5.0, d)
        V = rng.standard_normal((n, 16)).astype(np.float32)
        return Workload(name, X.astype(np.float32), None, V, RBF,
                        ls.astype(np.float32), 1.0, 0.1, rank=0, tol=0.0, max_iter=0)
    if name in ("C4", "C5"):
        n = n or (1048576 if name == "C4" else 2097152)
        d = 11
        X = _mixture_points(rng, n, d)
        ls = _log_uniform(rng, 0.3, 3.0, d)
        if with_targets:
            y = _fourier_target(rng, X)
        else:
            y = rng.standard_normal(n)
        V = np.concatenate([y[:, None].astype(np.float32), rademacher(rng, (n, 16))], axis=1)
        return Workload(name, X.astype(np.float32), y.astype(np.float32), V,
                        RBF if name == "C4" else MATERN32,
                        ls.astype(np.float32), 1.0, 0.1, rank=100, tol=1.0, max_iter=100)
    raise ValueError(name)


def well_separated_points(seed: int, n: int, d: int) -> np.ndarray:
    """Small point set on a jittered lattice: no duplicates and no near-coincident pairs,
    so that successive pivoted-Cholesky diagonal maxima are not near-ties."""
    rng = np.random.default_rng(seed)
    side = int(np.ceil(n ** (1.0 / d)))
    grid = np.stack(np.meshgrid(*[np.arange(side)] * d, indexing="ij"), axis=-1).reshape(-1, d)
    pick = rng.permutation(grid.shape[0])[:n]
    pts = (grid[pick] + rng.uniform(0.2, 0.8, size=(n, d))) / side
    return pts.astype(np.float32)
