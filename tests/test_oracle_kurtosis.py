"""Pins for the oracle's rotation + per-row kurtosis + loss (CPU only).

The oracle follows Eq. 3 (population moments about the mean, not excess) and the
kurtosis loss of the 'Kurtosis' paragraph in its per-token-row reading.  Nothing
here re-types the oracle's own loops: the checks are closed forms, library
routines the oracle does not use, and values the paper prints.
"""
import json
import os

import numpy as np
import pytest
import scipy.linalg
import scipy.stats

import oracle


def _facts(golden_dir):
    with open(os.path.join(golden_dir, "paper_facts.json")) as f:
        return json.load(f)


def test_rotate_matches_blas():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((37, 24))
    R = rng.standard_normal((24, 24))
    assert np.allclose(oracle.rotate(X, R), X @ R, rtol=0, atol=1e-12)
    # a non-symmetric R catches a transposed operand
    assert not np.allclose(oracle.rotate(X, R), X @ R.T, atol=1e-3)


def test_worked_row_1234():
    mu, m2, m3, m4, kappa, deg = oracle.row_moments([1, 2, 3, 4])
    assert (mu, m2, m3, m4) == (2.5, 1.25, 0.0, 2.5625)
    assert kappa == pytest.approx(1.64, abs=1e-15)
    assert not deg


@pytest.mark.parametrize("m", [2, 3, 4, 7, 16, 101])
def test_discrete_uniform_closed_form(m):
    # discrete uniform on 1..m: kappa = (3/5)(3m^2-7)/(m^2-1)
    kappa = oracle.row_moments(np.arange(1, m + 1))[4]
    assert kappa == pytest.approx(0.6 * (3 * m * m - 7) / (m * m - 1), rel=1e-13)


@pytest.mark.parametrize("d", [4, 16, 256])
def test_one_hot_identity(d):
    # a one-hot row is Bernoulli(1/d): kappa = d - 2 + 1/(d-1)
    X = np.zeros((3, d))
    X[0, 0] = 1.0
    X[1, d // 2] = -3.5
    X[2, d - 1] = 1e-3
    out = oracle.loss_grad(X, np.eye(d), want_dR=False)
    expect = d - 2 + 1.0 / (d - 1)
    assert np.allclose(out["row_kurt"], expect, rtol=1e-12)
    assert out["loss"] == pytest.approx(expect, rel=1e-12)


def test_one_hot_hadamard_is_global_minimum():
    d = 16
    H = scipy.linalg.hadamard(d) / np.sqrt(d)
    X = np.eye(d)[1:]  # rows e_1..e_{d-1}; e_0 would give the constant row
    out = oracle.loss_grad(X, H, want_G=True)
    assert np.allclose(out["row_kurt"], 1.0, atol=1e-13)
    assert np.allclose(out["G"], 0.0, atol=1e-13)
    assert np.allclose(out["dR"], 0.0, atol=1e-13)


def test_constant_row_is_degenerate():
    d = 16
    H = scipy.linalg.hadamard(d) / np.sqrt(d)
    X = np.zeros((2, d))
    X[0, 0] = 1.0  # -> constant row 1/sqrt(d)
    X[1, 3] = 2.0
    out = oracle.loss_grad(X, H, want_G=True)
    assert out["row_kurt"][0] == 0.0
    assert np.all(out["G"][0] == 0.0)
    assert out["row_kurt"][1] == pytest.approx(1.0, abs=1e-13)
    # the degenerate row still counts in 1/n
    assert out["loss"] == pytest.approx(0.5, abs=1e-13)
    # an all-zero row too
    out = oracle.loss_grad(np.zeros((1, d)), H, want_G=True)
    assert out["row_kurt"][0] == 0.0 and np.all(out["G"] == 0.0)


def test_identity_rotation_equals_scipy_kurtosis():
    rng = np.random.default_rng(2)
    X = rng.standard_t(3, size=(64, 96)) * 5 + rng.standard_normal((64, 1))
    out = oracle.loss_grad(X, np.eye(96), want_dR=False)
    ref = scipy.stats.kurtosis(X, axis=1, fisher=False, bias=True)
    assert np.allclose(out["row_kurt"], ref, rtol=1e-12)
    assert out["loss"] == pytest.approx(ref.mean(), rel=1e-12)


def test_rotated_equals_scipy_kurtosis_of_blas_product():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((40, 32))
    X[:, 5] *= 40
    Q, _ = np.linalg.qr(rng.standard_normal((32, 32)))
    out = oracle.loss_grad(X, Q, want_dR=False)
    ref = scipy.stats.kurtosis(X @ Q, axis=1, fisher=False, bias=True)
    assert np.allclose(out["row_kurt"], ref, rtol=1e-11)


def test_gaussian_rows_match_paper_value(golden_dir):
    k_normal = _facts(golden_dir)["kurtosis_of_normal"]["value"]
    n, d = 4096, 256
    rng = np.random.default_rng(4)
    X = rng.standard_normal((n, d))
    out = oracle.loss_grad(X, np.eye(d), want_dR=False)
    # finite-sample mean of the biased estimator: 3(d-1)/(d+1); s.d. of a row ~ sqrt(24/d)
    expect = k_normal * (d - 1) / (d + 1)
    assert abs(out["loss"] - expect) < 3 * np.sqrt(24.0 / d) / np.sqrt(n)
    assert abs(out["loss"] - k_normal) < 0.05


def test_tail_ordering(golden_dir):
    order = _facts(golden_dir)["kurtosis_ordering"]["value"]
    assert order == ["laplace", "normal", "uniform"]
    n, d = 512, 2048
    rng = np.random.default_rng(5)
    eye = np.eye(d)
    k_lap = oracle.loss_grad(rng.laplace(size=(n, d)), eye, want_dR=False)["loss"]
    k_nor = oracle.loss_grad(rng.standard_normal((n, d)), eye, want_dR=False)["loss"]
    k_uni = oracle.loss_grad(rng.uniform(-1, 1, size=(n, d)), eye, want_dR=False)["loss"]
    assert k_lap == pytest.approx(6.0, abs=0.15)
    assert k_nor == pytest.approx(3.0, abs=0.05)
    assert k_uni == pytest.approx(1.8, abs=0.02)
    assert k_lap > k_nor > k_uni


def test_target_loss_is_mean_abs_deviation():
    rng = np.random.default_rng(6)
    X = rng.standard_normal((50, 64))
    X[::2] = rng.uniform(-1, 1, size=(25, 64))  # kappa below and above the target
    out0 = oracle.loss_grad(X, np.eye(64), want_dR=False)
    out = oracle.loss_grad(X, np.eye(64), kappa_target=2.4, want_dR=False)
    assert (out0["row_kurt"] > 2.4).any() and (out0["row_kurt"] < 2.4).any()
    assert out["loss"] == pytest.approx(np.abs(out0["row_kurt"] - 2.4).mean(), rel=1e-13)


def test_invariances_of_loss():
    rng = np.random.default_rng(7)
    n, d = 30, 24
    X = rng.standard_t(4, size=(n, d))
    Q, _ = np.linalg.qr(rng.standard_normal((d, d)))
    base = oracle.loss_grad(X, Q, want_dR=False)
    # row permutation of X permutes the per-row kurtosis, loss unchanged
    p = rng.permutation(n)
    perm = oracle.loss_grad(X[p], Q, want_dR=False)
    assert np.allclose(perm["row_kurt"], base["row_kurt"][p], rtol=1e-13)
    assert perm["loss"] == pytest.approx(base["loss"], rel=1e-13)
    # global sign flip and column permutation of R leave kappa unchanged
    assert np.allclose(oracle.loss_grad(X, -Q, want_dR=False)["row_kurt"], base["row_kurt"], rtol=1e-13)
    cp = rng.permutation(d)
    assert np.allclose(oracle.loss_grad(X, Q[:, cp], want_dR=False)["row_kurt"], base["row_kurt"], rtol=1e-12)
    # positive row scaling leaves kappa unchanged
    a = rng.uniform(0.1, 10, size=(n, 1))
    assert np.allclose(oracle.loss_grad(a * X, Q, want_dR=False)["row_kurt"], base["row_kurt"], rtol=1e-12)
    # flipping a subset of columns keeps sum y^2 and sum y^4 but not the centred kurtosis
    s = np.ones(d)
    s[: d // 3] = -1
    Y, Ys = oracle.rotate(X, Q), oracle.rotate(X, Q * s)
    assert np.allclose((Y ** 2).sum(1), (Ys ** 2).sum(1), rtol=1e-13)
    assert np.allclose((Y ** 4).sum(1), (Ys ** 4).sum(1), rtol=1e-13)
    # kappa >= 1 always (Jensen)
    assert (base["row_kurt"] >= 1.0).all()
