"""Seeded synthetic path generators shared by the tests, the benchmark and the smoke check.

This module holds no signature arithmetic: it only draws Brownian-like sample paths
(cumulative sums of i.i.d. Gaussian increments) with the shapes of the benchmark
workloads, so that the CPU oracle and the HIP path are fed bit-identical fp32 arrays.
It imports neither of them.

The paper's benchmark fixes only shapes (batch 32, length 128, channels 2-7, depth 2-9;
section "Benchmark performance") and does not state the input values; the recipe here
stands in for them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

SEED_BASE = 200100706


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration (shape of a `sig_forward` call)."""

    index: int          # 1-based configuration number
    B: int              # batch: number of paths
    L: int              # points per path
    d: int              # channels
    N: int              # signature depth
    stream: bool        # emit every prefix signature
    basepoint: bool     # prepend the origin as an extra first point

    @property
    def name(self) -> str:
        mode = "stream" if self.stream else "final"
        tag = f"cfg{self.index}" if self.index > 0 else "custom"
        return f"{tag}:B{self.B}xL{self.L}xd{self.d},N{self.N},{mode}"

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def n_inc(self) -> int:
        return self.L if self.basepoint else self.L - 1

    @property
    def channels(self) -> int:
        return sum(self.d ** k for k in range(1, self.N + 1))


WORKLOADS = (
    Workload(1, B=32, L=16, d=2, N=4, stream=False, basepoint=False),
    Workload(2, B=1024, L=128, d=4, N=6, stream=False, basepoint=False),
    Workload(3, B=32, L=128, d=8, N=5, stream=False, basepoint=False),
    Workload(4, B=128, L=256, d=4, N=5, stream=True, basepoint=False),
    Workload(5, B=256, L=1024, d=16, N=4, stream=False, basepoint=False),
)


def workload(index: int) -> Workload:
    return WORKLOADS[index - 1]


def brownian_paths(B: int, L: int, d: int, seed: int) -> np.ndarray:
    """`[B, L, d]` float32 paths: x_1 = 0, x_{l+1} = x_l + xi_l, xi_l ~ N(0, 1/L) i.i.d.

    Drawn and accumulated in float64, rounded once to float32.  That float32 array is
    *the* input: the oracle widens it back to float64, the GPU reads it as is.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    x = np.zeros((B, L, d), dtype=np.float64)
    if L > 1:
        xi = rng.standard_normal((B, L - 1, d)) / math.sqrt(L)
        x[:, 1:, :] = np.cumsum(xi, axis=1)
    return x.astype(np.float32)


def uniform_paths(B: int, L: int, d: int, seed: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """`[B, L, d]` float32 paths with i.i.d. uniform points (rough paths; used by edge-case tests)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.uniform(lo, hi, size=(B, L, d)).astype(np.float32)


def workload_paths(w: Workload) -> np.ndarray:
    return brownian_paths(w.B, w.L, w.d, w.seed)
