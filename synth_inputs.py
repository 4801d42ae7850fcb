"""Seeded synthetic inputs for the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper).

This module only draws random numbers and names the workloads.  It holds none of the
method's arithmetic (no TCSC construction, no products), so the CPU oracle and the HIP
path can both take their inputs from it without sharing any code of the method.

The paper does not say how its random test matrices were drawn (Sec. 4, "Results"); the
recipe here is: one numpy PCG64 generator per workload, seeded with the workload's seed,
drawn in the order W, X, b.
  W : u = rng.random((K, N));  W = +1 where u < d/2,  -1 where d/2 <= u < d,  0 elsewhere
      (d = fraction of non-zeros, what the paper calls "sparsity" s in its cost analysis).
  X : float32, "uniform" = U[-1, 1), "normal" = N(0, 1), "int8" = integers in [-8, 8].
  b : float32, same family as X.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    K: int
    N: int
    density: float
    dist: str  # "uniform" | "normal" | "int8"
    seed: int

    @property
    def expected_nnz(self) -> float:
        return self.density * self.K * self.N


# The benchmark configurations.  C2 is the one the headline metric is quoted on.
WORKLOADS = {
    w.name: w
    for w in [
        Workload("C1", 64, 512, 512, 0.5, "uniform", 1001),
        Workload("C2", 256, 4096, 4096, 0.5, "uniform", 1002),
        Workload("C3a", 256, 4096, 4096, 0.25, "normal", 1003),
        Workload("C3b", 256, 4096, 4096, 0.125, "normal", 1004),
        Workload("C4-1", 1, 4096, 11008, 0.5, "normal", 1005),
        Workload("C4-8", 8, 4096, 11008, 0.5, "normal", 1005),
        Workload("C5a", 4096, 8192, 8192, 0.5, "uniform", 1006),
        Workload("C5b", 4096, 8192, 8192, 0.25, "uniform", 1007),
        Workload("C5c", 4096, 8192, 8192, 0.0625, "uniform", 1008),
    ]
}


def draw_ternary(rng: np.random.Generator, K: int, N: int, density: float) -> np.ndarray:
    """Dense ternary W (int8, K x N, row-major) with P(+1) = P(-1) = density / 2."""
    W = np.zeros((K, N), dtype=np.int8)
    # Drawn in row slabs so that the float64 uniforms never occupy more than ~64 MiB.
    slab = max(1, (8 << 20) // max(N, 1))
    for k0 in range(0, K, slab):
        u = rng.random((min(slab, K - k0), N))
        w = W[k0:k0 + u.shape[0]]
        w[u < density] = -1
        w[u < density / 2] = 1
    return W


def draw_dense(rng: np.random.Generator, shape, dist: str) -> np.ndarray:
    if dist == "uniform":
        return (rng.random(shape, dtype=np.float32) * np.float32(2) - np.float32(1)).astype(np.float32)
    if dist == "normal":
        return rng.standard_normal(shape, dtype=np.float32)
    if dist == "int8":
        return rng.integers(-8, 9, size=shape).astype(np.float32)
    raise ValueError(f"unknown distribution {dist!r}")


def make_inputs(M: int, K: int, N: int, density: float, dist: str, seed: int):
    """Return (W int8 [K,N], X float32 [M,K], b float32 [N]); draw order W, X, b."""
    rng = np.random.Generator(np.random.PCG64(seed))
    W = draw_ternary(rng, K, N, density)
    X = draw_dense(rng, (M, K), dist)
    b = draw_dense(rng, (N,), dist)
    return W, X, b


def workload(name: str) -> Workload:
    """A benchmark configuration by name, or an ad-hoc one spelled "M<m>-K<k>-N<n>-d<density>" (uniform X and b,
    seed derived from the shape): the shapes of the paper's own sweeps (Sec. 4) are named that way."""
    if name in WORKLOADS:
        return WORKLOADS[name]
    try:
        parts = dict((p[0], p[1:]) for p in name.split("-"))
        M, K, N, d = int(parts["M"]), int(parts["K"]), int(parts["N"]), float(parts["d"])
    except (KeyError, ValueError, IndexError):
        raise KeyError(f"unknown workload {name!r}") from None
    if min(M, K, N) < 1 or not 0.0 <= d <= 1.0:
        raise KeyError(f"bad workload {name!r}")
    return Workload(name, M, K, N, d, "uniform", 2000 + (M * 31 + K * 17 + N * 7 + int(d * 4096)) % 100000)


def make_workload(name: str, dist: str | None = None, M: int | None = None):
    """Inputs of a named workload; `dist` / `M` override the distribution / row count."""
    w = workload(name)
    return make_inputs(M if M is not None else w.M, w.K, w.N, w.density, dist or w.dist, w.seed)
