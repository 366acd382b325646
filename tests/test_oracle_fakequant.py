"""Pins for the oracle's per-token symmetric int4 fake quantiser (CPU only).

Follows 'Uniform Quantization for k-bit Precision' with k = 4, b = 0 and one scale
per token row (Setup), and the MSE of Eq. 1.
"""
import json
import os

import numpy as np
import pytest

import oracle


def test_levels_come_from_paper_formula(golden_dir):
    with open(os.path.join(golden_dir, "paper_facts.json")) as f:
        levels = json.load(f)["symmetric_levels_k4"]["value"]
    assert levels == 2 ** (4 - 1) - 1
    X = np.array([[0.5, -3.25, 1.0, 2.0]])
    out = oracle.fakequant_int4(X, np.eye(4))
    assert out["scales"][0] == np.float32(np.float32(3.25) / np.float32(levels))
    assert np.abs(out["codes"]).max() == levels


def test_exact_multiples_have_zero_error():
    rng = np.random.default_rng(0)
    n, d = 64, 32
    s = 2.0 ** rng.integers(-6, 6, size=(n, 1))
    k = rng.integers(-7, 8, size=(n, d))
    k[:, 0] = 7 * rng.choice([-1, 1], size=n)  # max |k| = 7 in every row
    X = k * s
    out = oracle.fakequant_int4(X, np.eye(d))
    assert np.array_equal(out["codes"], k.astype(np.int8))
    assert np.allclose(out["scales"], s[:, 0], rtol=1e-6)
    assert np.all(out["err"][:, 0] <= 1e-10 * out["err"][:, 1])


def test_bounds_and_half_step_error():
    rng = np.random.default_rng(1)
    n, d = 128, 96
    X = rng.standard_t(3, size=(n, d))
    Q, _ = np.linalg.qr(rng.standard_normal((d, d)))
    out = oracle.fakequant_int4(X, Q)
    Y = X @ Q
    s = out["scales"].astype(np.float64)[:, None]
    assert np.allclose(s[:, 0], np.abs(Y).max(1) / 7, rtol=1e-6)
    assert out["codes"].min() >= -7 and out["codes"].max() <= 7
    assert np.all(np.abs(out["codes"]).max(1) == 7)
    assert np.all(np.abs(Y - out["codes"] * s) <= 0.5 * s * (1 + 1e-5))
    # err = {sum (y - yhat)^2, sum y^2}
    assert np.allclose(out["err"][:, 0], ((Y - out["codes"] * s) ** 2).sum(1), rtol=1e-9)
    assert np.allclose(out["err"][:, 1], (Y ** 2).sum(1), rtol=1e-12)
    # nearest level: brute force over the 15 levels
    levels = np.arange(-7, 8)[None, None, :] * s[:, :, None]
    nearest = np.abs(Y[:, :, None] - levels).argmin(-1) - 7
    boundary = np.abs(np.abs(Y / s) % 1.0 - 0.5) < 1e-5
    assert np.array_equal(out["codes"][~boundary], nearest[~boundary].astype(np.int8))


def test_round_half_to_even_and_clipping():
    # s = 1 exactly: 7 -> amax; halves round to even
    X = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 6.5]])
    out = oracle.fakequant_int4(X, np.eye(8))
    assert out["scales"][0] == 1.0
    assert out["codes"][0].tolist() == [7, 0, 2, 2, 0, -2, -2, 6]
    # clip ratio 0.5 halves the scale and saturates the large entries at +-7
    out = oracle.fakequant_int4(X, np.eye(8), clip=0.5)
    assert out["scales"][0] == 0.5
    assert out["codes"][0].tolist() == [7, 1, 3, 5, -1, -3, -5, 7]
    # given scales are used verbatim
    out = oracle.fakequant_int4(X, np.eye(8), scales_in=[2.0])
    assert out["scales"][0] == 2.0
    assert out["codes"][0].tolist() == [4, 0, 1, 1, 0, -1, -1, 3]  # 3.5->4, .25->0, .75->1, 1.25->1, 3.25->3


def test_dense_uniform_mse_is_s2_over_12():
    rng = np.random.default_rng(2)
    n, d = 8, 65536
    X = rng.uniform(-1, 1, size=(n, d))
    X[:, 0] = 1.0
    # rotation by identity is implied; use a tiny d x d only through a block trick:
    # quantise rows directly with R = I on a thin problem is too big (d^2), so fold rows
    Xs = X.reshape(n * 1024, 64)
    Xs[:, 0] = np.where(np.abs(Xs).max(1) < 1.0, 1.0, Xs[:, 0])
    out = oracle.fakequant_int4(Xs, np.eye(64))
    s = out["scales"].astype(np.float64)
    mse = out["err"][:, 0].sum() / Xs.size
    assert mse == pytest.approx((s ** 2).mean() / 12.0, rel=0.02)


def test_zero_row():
    out = oracle.fakequant_int4(np.zeros((2, 8)), np.eye(8))
    assert np.all(out["scales"] == 0) and np.all(out["codes"] == 0) and np.all(out["err"] == 0)
