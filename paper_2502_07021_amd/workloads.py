"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and casts them; it contains none of the
method's arithmetic (no cost, no Gibbs kernel, no iteration), so both the GPU
path and the CPU oracle can be fed from it without sharing any of the method.

Recipe: NumPy ``default_rng(seed)`` (PCG64), draws in the order x, y, a, b in
fp64, marginals normalised to sum 1 in fp64, then everything cast to the
configuration's storage dtype.  Seed for configuration k is ``SEED_BASE*10 + k``.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 20250207


@dataclass
class Workload:
    name: str
    n: int
    d: int
    dtype: np.dtype
    eps: float
    mode: str                 # "dense" | "log" | "batched"
    normalise_by_max: bool
    iters: int
    c: int = 1
    m: int = 1                # histograms in a batch
    tol: float = 0.0          # > 0: tolerance mode (L1 row-marginal error)
    x: np.ndarray = field(default=None, repr=False)
    y: np.ndarray = field(default=None, repr=False)
    a: np.ndarray = field(default=None, repr=False)
    b: np.ndarray = field(default=None, repr=False)


def _normalised(w: np.ndarray) -> np.ndarray:
    return w / w.sum(axis=0, keepdims=True)


def make(config: int, n: int | None = None, m: int | None = None, seed: int | None = None) -> Workload:
    """Inputs of configuration ``config`` (1..5); ``n`` / ``m`` override the size while
    keeping the distribution (used by tests that need a smaller instance of the same law)."""
    rng = np.random.default_rng(SEED_BASE * 10 + config if seed is None else seed)
    if config == 1:
        n = 512 if n is None else n
        w = Workload("cfg1_n512_f64_dense", n, 2, np.dtype(np.float64), 0.05, "dense", False, 200)
        x = rng.uniform(0.0, 1.0, (n, 2)); y = rng.uniform(0.0, 1.0, (n, 2))
        a = np.full(n, 1.0 / n); b = np.full(n, 1.0 / n)
    elif config == 2:
        n = 8192 if n is None else n
        w = Workload("cfg2_n8192_f32_dense", n, 3, np.dtype(np.float32), 0.1, "dense", True, 500)
        x = rng.standard_normal((n, 3)); y = rng.standard_normal((n, 3))
        a = _normalised(rng.uniform(0.5, 1.5, n)); b = _normalised(rng.uniform(0.5, 1.5, n))
    elif config == 3:
        n = 32768 if n is None else n
        w = Workload("cfg3_n32768_f32_dense_c8", n, 8, np.dtype(np.float32), 0.05, "dense", True,
                     1000, c=8)
        x = rng.standard_normal((n, 8)); y = 0.5 + rng.standard_normal((n, 8))
        a = _normalised(rng.uniform(0.5, 1.5, n)); b = _normalised(rng.uniform(0.5, 1.5, n))
    elif config == 4:
        n = 65536 if n is None else n
        w = Workload("cfg4_n65536_f32_log", n, 16, np.dtype(np.float32), 0.01, "log", False, 2000,
                     tol=1e-6)
        x = rng.uniform(0.0, 1.0, (n, 16)); y = rng.uniform(0.0, 1.0, (n, 16))
        a = np.full(n, 1.0 / n); b = np.full(n, 1.0 / n)
    elif config == 5:
        n = 16384 if n is None else n
        m = 64 if m is None else m
        w = Workload("cfg5_n16384_m64_f32_batched", n, 2, np.dtype(np.float32), 0.05, "batched",
                     False, 300, m=m)
        x = rng.uniform(0.0, 1.0, (n, 2)); y = rng.uniform(0.0, 1.0, (n, 2))
        # Dirichlet(1) over n entries, one independent draw per column
        a = _normalised(rng.exponential(1.0, (n, m))); b = _normalised(rng.exponential(1.0, (n, m)))
    else:
        raise ValueError("config must be 1..5")
    w.x = np.ascontiguousarray(x.astype(w.dtype)); w.y = np.ascontiguousarray(y.astype(w.dtype))
    w.a = np.ascontiguousarray(a.astype(w.dtype)); w.b = np.ascontiguousarray(b.astype(w.dtype))
    return w
