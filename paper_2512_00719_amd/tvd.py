"""Total-variation instrument for the sampler's output distribution (measurement aid, host side).

The paper checks that speculative hot-vocab sampling leaves the output distribution unchanged by
the cumulative mean total-variation distance (TVD) between the token distributions of the SHVS
sampler and of the baseline sampler over many iterations (section 7, exactness of SHVS: below 1 %).
Here both samplers are the HIP library (with and without a hot set); the draws of one logits row,
replicated over the batch so that every copy has its own random numbers, are accumulated over
steps.  Only counting and the TVD formula live here; no sampling arithmetic.
"""
from __future__ import annotations

import numpy as np


def tvd(p: np.ndarray, q: np.ndarray) -> float:
    """Total-variation distance of two distributions (any non-negative vectors, normalised here)."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    return 0.5 * float(np.abs(p / p.sum() - q / q.sum()).sum())


def expected_tvd_of_sampling(p: np.ndarray, n: int) -> float:
    """Mean TVD between a distribution and the empirical distribution of n of its own draws
    (normal approximation per cell): what sampling noise alone produces."""
    p = np.asarray(p, dtype=np.float64)
    p = p[p > 0] / p.sum()
    return 0.5 * float(np.sqrt(2.0 * p * (1.0 - p) / (np.pi * n)).sum())


class CumulativeTvd:
    """Accumulates the ids drawn by two samplers step by step and reports, after each step, the TVD
    between their cumulative empirical distributions and its running mean over the steps so far."""

    def __init__(self, V: int):
        self.a = np.zeros(V, dtype=np.int64)
        self.b = np.zeros(V, dtype=np.int64)
        self.history: list[float] = []

    def add(self, ids_a: np.ndarray, ids_b: np.ndarray) -> float:
        self.a += np.bincount(ids_a, minlength=self.a.size)
        self.b += np.bincount(ids_b, minlength=self.b.size)
        self.history.append(tvd(self.a, self.b))
        return self.history[-1]

    @property
    def mean(self) -> float:
        return float(np.mean(self.history)) if self.history else 0.0
