"""Seeded synthetic test matrices (no arithmetic of the method lives here).

The paper's experiments use random matrices a_ij = (U_ij - 0.5) * exp(phi * N_ij)
with U uniform on (0,1) and N standard normal, B built the same way (caption
of the first accuracy figure and Section 4.1).  The paper names neither the
generator nor a seed; this module fixes both: numpy's PCG64 stream seeded with
`seed`, drawing U_A, N_A, U_B, N_B in that order, all in FP64 on the host.
Both the GPU path and the CPU oracle are fed from the arrays returned here.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def phi_matrix(rng: np.random.Generator, rows: int, cols: int, phi: float) -> np.ndarray:
    """(U - 0.5) * exp(phi * N), rows x cols, FP64."""
    u = rng.random((rows, cols))
    nrm = rng.standard_normal((rows, cols))
    nrm *= phi
    np.exp(nrm, out=nrm)
    u -= 0.5
    u *= nrm
    return u


def phi_pair(m: int, n: int, p: int, phi: float, seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """A (m x n) and B (n x p) for one benchmark / test case."""
    rng = np.random.Generator(np.random.PCG64(seed))
    A = phi_matrix(rng, m, n, phi)
    B = phi_matrix(rng, n, p, phi)
    return A, B


def small_int_pair(m: int, n: int, p: int, bound: int, seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Integer-valued FP64 matrices with entries in [-bound, bound]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    A = rng.integers(-bound, bound + 1, size=(m, n)).astype(np.float64)
    B = rng.integers(-bound, bound + 1, size=(n, p)).astype(np.float64)
    return A, B


def sample_indices(size: int, count: int, seed: int) -> np.ndarray:
    """Sorted sample of `count` distinct indices in [0, size), always holding
    the first and last index (so tile edges and ragged tails are covered)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    count = min(count, size)
    idx = set([0, size - 1]) if size > 0 else set()
    while len(idx) < count:
        idx.add(int(rng.integers(0, size)))
    return np.array(sorted(idx), dtype=np.int64)


def band_indices(size: int, band: int, seed: int) -> np.ndarray:
    """Sorted sample with one index in every block of `band` consecutive indices
    (a random position inside the block), plus the first and the last index:
    every tile row / tile column of an output is then represented."""
    rng = np.random.Generator(np.random.PCG64(seed))
    idx = set([0, size - 1]) if size > 0 else set()
    for lo in range(0, size, band):
        hi = min(lo + band, size)
        idx.add(int(rng.integers(lo, hi)))
    return np.array(sorted(idx), dtype=np.int64)
