"""The hot-vocabulary sizing model (paper section 5.4) against what the mathematics fixes: the fit
recovers an affine cost exactly, the printed derivative is the derivative of F, and the enumerated
argmin of F sits where the stationary condition changes sign, for the closed-form hit ratio of a
Zipf profile."""
import numpy as np

from paper_2512_00719_amd import sizing


def _zipf_alpha(V, s):
    mass = np.cumsum(np.arange(1, V + 1, dtype=np.float64) ** -s)
    return lambda H: mass[np.asarray(H, dtype=np.int64) - 1] / mass[-1]


def test_fit_recovers_an_affine_cost():
    H = np.array([1024, 4096, 16384, 65536])
    c, c0 = sizing.fit_affine_cost(H, 1.06e-8 * H + 8.55e-6)   # the constants the paper reports for its CPU fit
    assert abs(c - 1.06e-8) < 1e-15 and abs(c0 - 8.55e-6) < 1e-12


def test_derivative_and_stationary_condition_match_the_enumerated_optimum():
    V, s, c, c0 = 151_936, 1.1, 1.06e-8, 8.55e-6
    alpha = _zipf_alpha(V, s)
    Hs = np.arange(1, V + 1)
    a = alpha(Hs)
    F = sizing.expected_cost(Hs, a, c, c0, V)
    # Eq. (first-derivative) against a central difference of F itself (alpha' by central difference too)
    da = np.gradient(a, Hs)
    dF = c * sizing.stationary_residual(Hs, a, da, V)
    num = np.gradient(F, Hs)
    inner = slice(10, V - 10)
    assert np.allclose(dF[inner], num[inner], rtol=1e-3, atol=1e-14)
    # the enumerated argmin is interior and the stationary residual changes sign there (Eq. stationary-h)
    H_star, F_star = sizing.best_hot_size(alpha, c, c0, V)
    assert 1 < H_star < V and F_star == F.min()
    res = sizing.stationary_residual(Hs, a, da, V)
    assert res[H_star - 30] < 0 < res[H_star + 30]
    # more covered mass per hot column (a steeper profile) moves the optimum to a smaller hot set
    H_steep, _ = sizing.best_hot_size(_zipf_alpha(V, 1.4), c, c0, V)
    assert H_steep < H_star
    # c scales F - c0 and leaves the optimum where it is; c = 0 leaves nothing to choose
    assert sizing.best_hot_size(alpha, 5 * c, c0, V)[0] == H_star
    assert np.ptp(sizing.expected_cost(Hs, a, 0.0, c0, V)) == 0.0


def test_sweep_summary_and_interpolation():
    V = 201_088
    H = [4096, 8192, 16384, 32768]
    alpha = [0.940, 0.965, 0.984, 0.994]
    flat = sizing.summarize_sweep(H, [0.68e-6] * 4, alpha, V, reference=(1.06e-8, 8.55e-6))
    assert abs(flat["fit"]["c"]) < 1e-18 and flat["relative_spread_of_cost"] == 0.0
    assert flat["best_H_reference"] == 8192   # with the paper's CPU constants this hit-ratio curve puts the optimum there
    f = sizing.interpolate_hit_ratio(H, alpha)
    assert abs(float(f(8192)) - 0.965) < 1e-12 and 0.940 < float(f(6000)) < 0.965 and float(f(10 ** 6)) == 0.994
