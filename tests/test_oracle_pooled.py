"""Pins of the oracle's pooled loss: the loss exactly as the paper writes it (loss equation of
the "Kurtosis" paragraph: kurtosis of the concatenation of all tokens' activations, distance to
the kurtosis of the uniform distribution) on the output of the small network of "Learning the
Rotations" (linear layer + RMSNorm).  Pinned by scipy's kurtosis on the flattened activations,
the textbook values for uniform / normal / Laplace samples, central finite differences on every
entry of R, and the structure the RMSNorm forces on the gradient."""
import numpy as np
import pytest
import scipy.stats

import oracle


def _rand_orth(d, seed):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((d, d)))
    return q * np.sign(np.diag(r))


def _z(X, R, eps=0.0):
    Y = X @ R
    return Y / np.sqrt((Y ** 2).mean(1, keepdims=True) + eps)


@pytest.mark.parametrize("n,d,eps", [(64, 8, 0.0), (300, 16, 1e-5), (128, 32, 1e-2)])
def test_loss_is_scipy_kurtosis_of_the_flattened_rmsnormed_activations(n, d, eps):
    rng = np.random.default_rng(n + d)
    X = rng.standard_normal((n, d)) * rng.lognormal(0, 1, size=(1, d))
    R = _rand_orth(d, 3)
    o = oracle.pooled_loss_grad(X, R, kappa_target=1.8, rms_eps=eps, want_dR=False)
    k = scipy.stats.kurtosis(_z(X, R, eps).ravel(), fisher=False, bias=True)
    assert abs(o["kappa"] - k) < 1e-11 * k
    assert abs(o["loss"] - abs(k - 1.8)) < 1e-11
    assert oracle.pooled_loss_grad(X, R, kappa_target=0.0, rms_eps=eps, want_dR=False)["loss"] == pytest.approx(k, rel=1e-12)


def test_textbook_values():
    rng = np.random.default_rng(0)
    n, d = 4096, 64
    I = np.eye(d)
    # A normal row after RMSNorm is a uniform point on the sphere of radius sqrt(d): its entries have
    # E z^2 = 1 and E z^4 = 3 d / (d + 2) exactly, so the pooled kurtosis is 3 d / (d + 2).
    # For large d the RMSNorm scale of a row of iid entries is nearly constant and the pooled
    # kurtosis approaches that of the entry distribution: uniform 9/5, the target of the loss.
    ku = oracle.pooled_loss_grad(rng.uniform(-1, 1, (n, d)), I, want_dR=False)["kappa"]
    kn = oracle.pooled_loss_grad(rng.standard_normal((n, d)), I, want_dR=False)["kappa"]
    kl = oracle.pooled_loss_grad(rng.laplace(size=(n, d)), I, want_dR=False)["kappa"]
    assert abs(ku - 1.8) < 0.02
    assert abs(kn - 3.0 * d / (d + 2)) < 0.03
    assert kn + 1.0 < kl < 6.0          # heavier tails than the normal; the row scale damps the largest entries
    assert oracle.pooled_loss_grad(rng.uniform(-1, 1, (n, d)), I, want_dR=False)["loss"] < 0.02


@pytest.mark.parametrize("n,d,eps,kt", [(16, 8, 0.0, 1.8), (40, 6, 1e-3, 1.8), (24, 8, 0.0, 0.0), (16, 8, 0.0, 50.0)])
def test_gradient_by_central_differences(n, d, eps, kt):
    rng = np.random.default_rng(5 + n)
    X = rng.standard_normal((n, d))
    X[:, 1] *= 8.0
    R = _rand_orth(d, 11) + 0.05 * rng.standard_normal((d, d))   # R is a free matrix for this gradient
    o = oracle.pooled_loss_grad(X, R, kappa_target=kt, rms_eps=eps, want_G=True)
    h = 1e-6
    num = np.zeros((d, d))
    for k in range(d):
        for l in range(d):
            Rp, Rm = R.copy(), R.copy()
            Rp[k, l] += h
            Rm[k, l] -= h
            num[k, l] = (oracle.pooled_loss_grad(X, Rp, kt, eps, want_dR=False)["loss"]
                         - oracle.pooled_loss_grad(X, Rm, kt, eps, want_dR=False)["loss"]) / (2 * h)
    assert np.abs(num - o["dR"]).max() <= 2e-6 * np.abs(o["dR"]).max()
    assert np.abs(X.T @ o["G"] - o["dR"]).max() < 1e-12 * max(1.0, np.abs(o["dR"]).max())


def test_structure_forced_by_the_rmsnorm():
    rng = np.random.default_rng(2)
    n, d = 50, 12
    X = rng.standard_normal((n, d)) * rng.lognormal(0, 1.5, size=(n, 1))   # very different row norms
    R = _rand_orth(d, 4)
    o = oracle.pooled_loss_grad(X, R, want_G=True)
    Y = X @ R
    # RMSNorm output is invariant to the scale of its input row: every row of dL/dY is orthogonal to y_i
    assert np.abs((o["G"] * Y).sum(1)).max() < 1e-12 * np.abs(o["G"]).max() * np.abs(Y).max() * d
    # scaling token rows does not change anything (eps = 0)
    o2 = oracle.pooled_loss_grad(X * rng.uniform(0.5, 2.0, size=(n, 1)), R)
    assert abs(o2["loss"] - o["loss"]) < 1e-12
    # for orthogonal R the row norms do not depend on R: the skew part of dR R^T (what a Cayley
    # step uses) equals the one computed with the RMSNorm scales held constant
    rho = np.sqrt((Y ** 2).mean(1, keepdims=True))
    Z = Y / rho
    N = n * d
    mu = Z.mean(); c = Z - mu; m2 = (c ** 2).mean(); m3 = (c ** 3).mean(); kap = (c ** 4).mean() / m2 ** 2
    gz = np.sign(kap - 1.8) * 4.0 / (N * m2 ** 2) * (c ** 3 - m3 - kap * m2 * c)
    dR_const = X.T @ (gz / rho)
    A1 = o["dR"] @ R.T - R @ o["dR"].T
    A2 = dR_const @ R.T - R @ dR_const.T
    assert np.abs(A1 - A2).max() < 1e-12 * np.abs(A1).max()
    assert np.abs(o["dR"] - dR_const).max() > 1e-3 * np.abs(o["dR"]).max()   # the Jacobian term itself is not small


def test_zero_rows_and_degenerate_input():
    X = np.zeros((8, 4))
    X[0] = [1.0, -1.0, 1.0, -1.0]
    X[3] = [2.0, 0.0, 0.0, 0.0]
    o = oracle.pooled_loss_grad(X, np.eye(4), want_G=True)
    assert np.isfinite(o["loss"]) and np.isfinite(o["dR"]).all()
    assert np.abs(o["G"][1]).max() == 0.0           # zero rows carry no gradient
