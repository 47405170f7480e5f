"""Hot-vocabulary sizing model (paper section 5.4), host side: offline tooling, no sampling arithmetic.

The paper chooses the hot-set size H from two ingredients: an affine cost of a single-pass scan,
``T(H) = c * H + c0`` (fitted by least squares from a few measured points, section 7 "sizing model
validation"), and the hit ratio ``alpha_bar(H)`` (mean hot mass, measured from traces).  Their
composition is the expected decision cost of Eq. (cpu-time),

    F(H) = c0 + c * (alpha_bar(H) * H + (1 - alpha_bar(H)) * (V - H)),

whose derivative is ``c * (-1 + 2 alpha_bar + (2 H - V) alpha_bar')`` (Eq. first-derivative) and whose
stationary point satisfies ``2 alpha_bar(H*) + (2 H* - V) alpha_bar'(H*) = 1`` (Eq. stationary-h);
H being discrete, the deployed choice is ``argmin_H F(H)`` by enumeration.
"""
from __future__ import annotations

from typing import Callable, Sequence

import numpy as np


def fit_affine_cost(H: Sequence[float], t: Sequence[float]) -> tuple[float, float]:
    """Least-squares fit of ``t = c * H + c0``; returns ``(c, c0)``."""
    H = np.asarray(H, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    A = np.stack([H, np.ones_like(H)], axis=1)
    (c, c0), *_ = np.linalg.lstsq(A, t, rcond=None)
    return float(c), float(c0)


def expected_cost(H, alpha_bar, c: float, c0: float, V: int):
    """F(H) of Eq. (cpu-time): the hot path costs c*H + c0, a rejected draw visits the V - H others."""
    H = np.asarray(H, dtype=np.float64)
    a = np.asarray(alpha_bar, dtype=np.float64)
    return c0 + c * (a * H + (1.0 - a) * (V - H))


def stationary_residual(H, alpha_bar, d_alpha_bar, V: int):
    """``2 alpha_bar + (2 H - V) alpha_bar' - 1``: zero at the continuous optimum, dF/dH = c * residual."""
    H = np.asarray(H, dtype=np.float64)
    return 2.0 * np.asarray(alpha_bar, dtype=np.float64) + (2.0 * H - V) * np.asarray(d_alpha_bar, dtype=np.float64) - 1.0


def best_hot_size(alpha_bar_of: Callable[[np.ndarray], np.ndarray], c: float, c0: float, V: int,
                  candidates: Sequence[int] | None = None) -> tuple[int, float]:
    """``argmin_H F(H)`` by enumeration over ``candidates`` (default: every H in 1..V); returns (H, F(H))."""
    Hs = np.arange(1, V + 1) if candidates is None else np.asarray(candidates)
    F = expected_cost(Hs, alpha_bar_of(Hs), c, c0, V)
    i = int(np.argmin(F))
    return int(Hs[i]), float(F[i])


def interpolate_hit_ratio(H_points: Sequence[float], alpha_points: Sequence[float]) -> Callable[[np.ndarray], np.ndarray]:
    """``alpha_bar(H)`` between measured points: linear in log H (the curve is Zipf-like), clamped to
    the end points outside them."""
    lh = np.log(np.asarray(H_points, dtype=np.float64))
    a = np.asarray(alpha_points, dtype=np.float64)
    order = np.argsort(lh)
    lh, a = lh[order], a[order]
    return lambda H: np.interp(np.log(np.asarray(H, dtype=np.float64)), lh, a)


def summarize_sweep(H: Sequence[int], seconds_per_row: Sequence[float], alpha_bar: Sequence[float], V: int,
                    reference: tuple[float, float] | None = None) -> dict:
    """What a measured sweep over H says: the affine fit of the measured cost, how much of the cost
    varies with H at all, F(H) at the measured points with the fitted constants and (optionally)
    with reference constants such as the paper's CPU fit, and the best measured H under each."""
    c, c0 = fit_affine_cost(H, seconds_per_row)
    t = np.asarray(seconds_per_row, dtype=np.float64)
    out = {"H": [int(h) for h in H], "alpha_bar": [float(a) for a in alpha_bar], "seconds_per_row": [float(x) for x in t],
           "fit": {"c": c, "c0": c0}, "relative_spread_of_cost": float((t.max() - t.min()) / t.mean())}
    F = expected_cost(H, alpha_bar, c, c0, V)
    out["F_fitted"] = [float(x) for x in F]
    out["best_H_fitted"] = int(np.asarray(H)[int(np.argmin(F))])
    if reference is not None:
        Fr = expected_cost(H, alpha_bar, reference[0], reference[1], V)
        out["F_reference"] = [float(x) for x in Fr]
        out["best_H_reference"] = int(np.asarray(H)[int(np.argmin(Fr))])
    return out
