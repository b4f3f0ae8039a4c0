"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

Holds no arithmetic of the emulation method: it only draws matrices with the
distribution of the paper's experiments (Section 5): entries
(rand - 0.5) * exp(phi * randn) with rand uniform in (0, 1] and randn standard
normal; phi = 0.5 is the spread the paper likens to HPL.  The paper drew them
with a GPU random-number library; here numpy's PCG64 stands in, one stream per
matrix, so every run of the same (shape, phi, seed) sees the same bits.
"""
from __future__ import annotations

import numpy as np


def matrix(rows: int, cols: int, phi: float, seed: int, dtype=np.float64) -> np.ndarray:
    """Row-major rows x cols matrix of (U - 0.5) * exp(phi * Z), drawn in FP64."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = np.empty((rows, cols), np.float64)
    # Row blocks keep the temporary memory small at the 16384-class sizes.
    step = max(1, (1 << 22) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        u = 1.0 - rng.random((r1 - r0, cols))          # (0, 1]
        z = rng.standard_normal((r1 - r0, cols))
        out[r0:r1] = (u - 0.5) * np.exp(phi * z)
    return out.astype(dtype, copy=False)


def gemm_inputs(m: int, n: int, k: int, phi: float = 0.5, seed: int = 0,
                dtype=np.float64):
    """A (m x k) from `seed`, B (k x n) from `seed + 1`."""
    return matrix(m, k, phi, seed, dtype), matrix(k, n, phi, seed + 1, dtype)
