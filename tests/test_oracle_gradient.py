"""Pins for the oracle's gradient dL/dR = X^T (dL/dY) (CPU only).

The paper prints no gradient formula (it relies on automatic differentiation of
Eq. 3), so the oracle's closed form is pinned by central finite differences on
every entry of R, by reverse-mode autodiff of the definition written with library
ops, and by the invariants shift / scale invariance imply.
"""
import numpy as np
import pytest
import torch

import oracle


def _problem(n, d, seed, heavy=True):
    rng = np.random.default_rng(seed)
    X = rng.standard_t(3, size=(n, d)) if heavy else rng.standard_normal((n, d))
    X[:, 1] *= 20.0
    Q, _ = np.linalg.qr(rng.standard_normal((d, d)))
    return X, Q


@pytest.mark.parametrize("n,d,kt", [(16, 8, 0.0), (64, 16, 0.0), (16, 8, 2.6)])
def test_finite_differences(n, d, kt):
    X, R = _problem(n, d, 10 + d)
    out = oracle.loss_grad(X, R, kappa_target=kt)
    fd = np.zeros((d, d))
    h = 1e-6
    for k in range(d):
        for l in range(d):
            Rp, Rm = R.copy(), R.copy()
            Rp[k, l] += h
            Rm[k, l] -= h
            lp = oracle.loss_grad(X, Rp, kappa_target=kt, want_dR=False)["loss"]
            lm = oracle.loss_grad(X, Rm, kappa_target=kt, want_dR=False)["loss"]
            fd[k, l] = (lp - lm) / (2 * h)
    rel = np.linalg.norm(fd - out["dR"]) / np.linalg.norm(fd)
    assert rel < 1e-6


@pytest.mark.parametrize("kt", [0.0, 1.8, 3.2])
def test_autodiff_of_definition(kt):
    n, d = 48, 20
    X, R = _problem(n, d, 20)
    Xt = torch.tensor(X, dtype=torch.float64)
    Rt = torch.tensor(R, dtype=torch.float64, requires_grad=True)
    Y = Xt @ Rt
    Y.retain_grad()
    c = Y - Y.mean(dim=1, keepdim=True)
    kappa = (c ** 4).mean(dim=1) / (c ** 2).mean(dim=1) ** 2
    loss = kappa.mean() if kt == 0.0 else (kappa - kt).abs().mean()
    loss.backward()
    out = oracle.loss_grad(X, R, kappa_target=kt, want_G=True)
    assert out["loss"] == pytest.approx(loss.item(), rel=1e-13)
    assert np.allclose(out["G"], Y.grad.numpy(), rtol=1e-9, atol=1e-14)
    assert np.allclose(out["dR"], Rt.grad.numpy(), rtol=1e-9, atol=1e-13)


def test_gradient_invariants():
    n, d = 200, 48
    X, R = _problem(n, d, 30)
    out = oracle.loss_grad(X, R, want_G=True)
    G, dR = out["G"], out["dR"]
    Y = X @ R
    scale = np.abs(G).sum(1)
    # each row: sum_j G_ij = 0 (shift invariance) and sum_j G_ij y_ij = 0 (scale invariance)
    assert np.all(np.abs(G.sum(1)) <= 1e-12 * scale)
    assert np.all(np.abs((G * Y).sum(1)) <= 1e-12 * (np.abs(G) * np.abs(Y)).sum(1))
    # globally: <dR, R>_F = 0 for any R; dR 1 = 0
    nrm = np.linalg.norm(dR)
    assert abs((dR * R).sum()) < 1e-12 * nrm * np.linalg.norm(R)
    assert np.linalg.norm(dR.sum(1)) < 1e-12 * nrm * np.sqrt(d)


def test_gradient_equivariances():
    n, d = 60, 16
    X, R = _problem(n, d, 40)
    rng = np.random.default_rng(41)
    base = oracle.loss_grad(X, R)["dR"]
    p = rng.permutation(n)
    assert np.allclose(oracle.loss_grad(X[p], R)["dR"], base, rtol=1e-11, atol=1e-14)
    cp = rng.permutation(d)
    assert np.allclose(oracle.loss_grad(X, R[:, cp])["dR"], base[:, cp], rtol=1e-11, atol=1e-14)
    assert np.allclose(oracle.loss_grad(X, -R)["dR"], -base, rtol=1e-11, atol=1e-14)


def test_chunk_additivity():
    n, d = 96, 24
    X, R = _problem(n, d, 50)
    full = oracle.loss_grad(X, R)
    acc_dR = np.zeros((d, d))
    acc_loss = 0.0
    for lo, hi in [(0, 10), (10, 64), (64, 96)]:
        part = oracle.loss_grad(X[lo:hi], R)
        acc_dR += (hi - lo) * part["dR"]
        acc_loss += (hi - lo) * part["loss"]
    assert np.allclose(n * full["dR"], acc_dR, rtol=1e-11, atol=1e-13)
    assert n * full["loss"] == pytest.approx(acc_loss, rel=1e-13)


def test_descent_direction():
    # a small step along -dR lowers the loss to first order
    n, d = 128, 16
    X, R = _problem(n, d, 60)
    out = oracle.loss_grad(X, R)
    eps = 1e-5 / np.linalg.norm(out["dR"])
    l1 = oracle.loss_grad(X, R - eps * out["dR"], want_dR=False)["loss"]
    predicted = -eps * np.linalg.norm(out["dR"]) ** 2
    assert (l1 - out["loss"]) == pytest.approx(predicted, rel=1e-3)
