"""Pins of the oracle's quantisation sensitivity (Background: Definition "Quantization
Sensitivity", Eq. 1, and the theorem quoted there).  Pinned by the paper's own statement that for
the uniform distribution the optimal step is (max - min)/(2^k - 1), a brute-force scan of the MSE written
in numpy on a grid of its own, the textbook optimal step of a Gaussian source, and a hand-built sample whose
error has two separate minima (a coarse search that only refines around its first guess fails it)."""
import numpy as np
import pytest

import oracle


def _mse(y, s, L=7):
    q = np.clip(np.rint(y / s), -L, L)
    return float(((y - q * s) ** 2).mean())


def test_uniform_optimum_is_the_range_over_levels():
    rng = np.random.default_rng(0)
    y = rng.uniform(-1, 1, 400000).astype(np.float32)
    for bits in (3, 4, 5):
        o = oracle.quant_sensitivity(y, [0.1], bits=bits)
        levels = 2 ** bits - 1                      # symmetric grid: -L..L, 2L + 1 = 2^bits - 1 levels
        assert abs(o["s_opt"] - 2.0 / levels) < 0.01 * 2.0 / levels
        assert abs(o["mse_opt"] - o["s_opt"] ** 2 / 12) < 0.02 * o["mse_opt"]


@pytest.mark.parametrize("dist", ["normal", "laplace", "outliers"])
def test_optimum_against_a_dense_scan(dist):
    rng = np.random.default_rng(1)
    y = {"normal": rng.standard_normal(100000), "laplace": rng.laplace(size=100000),
         "outliers": np.concatenate([rng.standard_normal(99000), 40 * rng.standard_normal(1000)])}[dist].astype(np.float32)
    o = oracle.quant_sensitivity(y, [0.05, 0.1, 0.2])
    yd = y.astype(np.float64)
    smax = np.abs(yd).max() / 7
    grid = smax * np.exp(np.linspace(np.log(1 / 250), 0, 4000))
    scan = np.array([_mse(yd, s) for s in grid])
    assert o["mse_opt"] <= scan.min() * (1 + 1e-3)          # as good as the dense scan
    assert abs(o["mse_opt"] - _mse(yd, o["s_opt"])) < 1e-6 * o["mse_opt"]
    for a, g in zip([0.05, 0.1, 0.2], o["gamma"]):
        assert abs(g - abs(_mse(yd, o["s_opt"] * (1 + np.float32(a))) - o["mse_opt"])) < 1e-5 * o["mse_opt"] + 1e-3 * g
    assert o["gamma"][0] < o["gamma"][1] < o["gamma"][2]
    if dist == "normal":                                   # 15-level uniform quantiser of a Gaussian: step ~ 0.35 sigma
        assert 0.33 < o["s_opt"] < 0.38


def test_gamma_vanishes_at_zero_and_is_quadratic_at_a_smooth_minimum():
    rng = np.random.default_rng(2)
    yn = rng.standard_normal(400000).astype(np.float32)
    o = oracle.quant_sensitivity(yn, [0.0, 0.05, 0.1])
    assert o["gamma"][0] <= 1e-12 * o["mse_opt"]     # same step again (the parallel sum may reorder)
    # a Gaussian source has a smooth MSE minimum in the step: Gamma grows with the square of the offset
    assert 3.0 < o["gamma"][2] / o["gamma"][1] < 5.5


def test_mse_is_eq_1_on_hand_values():
    # step 1, levels -7..7: 0.4 -> 0, 2.6 -> 3, 9 -> 7 (clipped), -0.5 -> -0 (half to even), 1.5 -> 2
    y = np.array([0.4, 2.6, 9.0, -0.5, 1.5], dtype=np.float32)
    want = np.mean(np.array([0.4, 0.4, 2.0, 0.5, 0.5], dtype=np.float32).astype(np.float64) ** 2)
    assert abs(oracle.quant_mse(y, 1.0) - want) < 1e-7
    assert abs(oracle.quant_mse(y, 1.0, bits=3) - np.mean([0.4 ** 2, 0.4 ** 2, 36.0, 0.25, 0.25])) < 1e-6


def test_two_minima_the_deeper_one_is_found():
    # Half the sample sits exactly on +-1, the other half on +-7.3.  With 3 bits (levels -3..3) the error vanishes
    # on neither cluster at one step, and MSE(s) has separate valleys: s near 7.3/3 (big cluster exact, small one
    # rounds to 0 or 1 step) and s near 1 (small cluster exact, big one clipped at 3).  The definition asks for
    # the global minimum over s; brute force in numpy on an independent linear grid says where it is.
    y = np.concatenate([np.full(5000, 1.0), np.full(5000, -1.0), np.full(300, 7.3), np.full(300, -7.3)]).astype(np.float32)
    o = oracle.quant_sensitivity(y, [0.1], bits=3)
    yd = y.astype(np.float64)
    grid = np.linspace(0.01, 7.3 / 3, 20000)
    scan = np.array([_mse(yd, s, L=3) for s in grid])
    assert o["mse_opt"] <= scan.min() * (1 + 1e-3)
    assert abs(o["s_opt"] - grid[scan.argmin()]) < 2e-3 * o["s_opt"]
    # and the other valley is a strict local minimum that is worse
    far = np.abs(grid - grid[scan.argmin()]) > 0.5
    assert scan[far].min() > 1.2 * scan.min()
    lo, hi = o["flat"]
    assert lo <= o["s_opt"] <= hi and hi - lo < 0.05 * o["s_opt"]


def test_flat_region_brackets_the_optimum():
    rng = np.random.default_rng(3)
    y = rng.standard_normal(200000).astype(np.float32)
    o = oracle.quant_sensitivity(y, [0.1], flat_tol=1e-3)
    lo, hi = o["flat"]
    assert lo < o["s_opt"] < hi
    assert oracle.quant_mse(y, lo) <= (1 + 1e-3) * o["mse_opt"] and oracle.quant_mse(y, hi) <= (1 + 1e-3) * o["mse_opt"]
    # a smooth minimum: MSE rises by 1e-3 over a few per cent of the step
    assert 0.01 < (hi - lo) / o["s_opt"] < 0.2
