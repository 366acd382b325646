"""Pins of the oracle's per-token quantisation-quality figures: the max-value "success" count of
the paper's "Evaluation ... on Channel Outliers" paragraph, symmetric int4 with the scale clipped
at a row quantile (Setup appendix: quantile 0.98), asymmetric int4 (Background, "Uniform
Quantization for k-bit Precision": b = min, s = (max - min)/(2^k - 1); Setup: KV caches).
Pinned by numpy's quantile, rows built from exact multiples of the step, a brute-force search of
the nearest level, the half-step bound, the s^2/12 law and constructed success / no-success cases."""
import numpy as np
import pytest
import scipy.linalg

import oracle


def test_threshold_is_numpys_linear_quantile():
    rng = np.random.default_rng(0)
    for d, q in [(16, 0.9), (128, 0.98), (100, 0.5), (64, 0.999)]:
        X = rng.standard_normal((7, d)) * 3
        o = oracle.quant_metrics(X, np.eye(d), q)
        ref = np.quantile(np.abs(X.astype(np.float32)).astype(np.float64), q, axis=1)
        assert np.abs(o["thr"] - ref).max() <= 2e-7 * ref.max()
    o = oracle.quant_metrics(X, np.eye(d), 1.0)
    assert np.array_equal(o["thr"], np.abs(X.astype(np.float32)).max(1))
    assert np.array_equal(o["thr"], o["amax"][:, 1])


def test_symmetric_exact_multiples_and_clipping():
    # row = k * s with k in [-7, 7] and max |k| = 7: codes reproduce the row exactly (quantile 1)
    s = 0.25
    k = np.array([[-7, -3, 0, 1, 2, 5, 7, 4], [7, 7, -7, 0, 0, 1, -1, 3]], dtype=np.float64)
    o = oracle.quant_metrics(k * s, np.eye(8), 1.0)
    assert np.abs(o["err_sym"][:, 0]).max() == 0.0
    assert np.allclose(o["err_sym"][:, 1], ((k * s) ** 2).sum(1))
    # one huge entry, quantile below it: the step follows the bulk, the outlier is clipped to 7 s
    row = np.concatenate([np.linspace(-1, 1, 99), [100.0]])[None]
    o = oracle.quant_metrics(row, np.eye(100), 0.98)
    t = np.quantile(np.abs(row[0].astype(np.float32)).astype(np.float64), 0.98)
    assert abs(o["thr"][0] - t) < 1e-6
    bulk_bound = 99 * (t / 7 / 2) ** 2
    assert abs(o["err_sym"][0, 0] - (100.0 - t) ** 2) <= bulk_bound + 1e-3


def test_asymmetric_brute_force_nearest_level():
    rng = np.random.default_rng(3)
    Y = rng.standard_normal((6, 40)) * 2 + 1.5          # not centred: the asymmetric grid pays off
    o = oracle.quant_metrics(Y, np.eye(40), 1.0)
    Yf = Y.astype(np.float32).astype(np.float64)
    for i in range(6):
        mn, mx = Yf[i].min(), Yf[i].max()
        s = (mx - mn) / 15
        levels = mn + s * np.arange(16)
        nearest = levels[np.abs(Yf[i][:, None] - levels[None]).argmin(1)]
        e = ((Y[i] - nearest) ** 2).sum()
        assert abs(o["err_asym"][i, 0] - e) <= 1e-5 * e
        assert np.abs(Y[i] - nearest).max() <= s / 2 * (1 + 1e-6)
    # an off-centre row is quantised better by the asymmetric grid (16 levels over max - min) than by
    # the symmetric one (15 levels over 2 max|y|)
    assert (o["err_asym"][:, 0] < o["err_sym"][:, 0]).all()


def test_uniform_data_follow_the_s2_over_12_law():
    rng = np.random.default_rng(4)
    Y = rng.uniform(-1, 1, (64, 4096))
    o = oracle.quant_metrics(Y, np.eye(4096), 1.0)
    s_sym = o["amax"][:, 1] / 7
    assert np.abs(o["err_sym"][:, 0] / 4096 / (s_sym ** 2 / 12) - 1).max() < 0.1
    s_asym = (Y.max(1) - Y.min(1)) / 15
    assert np.abs(o["err_asym"][:, 0] / 4096 / (s_asym ** 2 / 12) - 1).max() < 0.1


def test_success_counts_on_constructed_rotations():
    d = 64
    H = scipy.linalg.hadamard(d) / np.sqrt(d)
    X = np.eye(d)[:10] * 5.0                      # one-hot rows: the worst case for a token's max
    o = oracle.quant_metrics(X, H, 1.0)
    assert o["success"] == 10                     # max drops from 5 to 5/sqrt(d)
    assert np.allclose(o["amax"][:, 0], 5.0) and np.allclose(o["amax"][:, 1], 5.0 / np.sqrt(d))
    assert oracle.quant_metrics(X, np.eye(d), 1.0)["success"] == 0     # equal is not smaller
    Xf = np.ones((4, d))                          # flat rows: the Hadamard rotation concentrates them
    assert oracle.quant_metrics(Xf, H, 1.0)["success"] == 0
