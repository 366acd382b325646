"""Pins for the oracle's Cayley retraction (CPU only).

'Optimization in the Orthogonal Space' names Cayley SGD on the Stiefel manifold
without printing a formula; the oracle takes the closed-form Cayley transform of
the skew matrix A = G R^T - R G^T with an exact solve.  Pinned by the 2x2 closed
form, orthogonality, determinant, fixed points, first-order behaviour, the
equivalent right-hand form and a library solve the oracle does not use.
"""
import numpy as np
import pytest

import oracle


def _rot(t):
    return np.array([[np.cos(t), -np.sin(t)], [np.sin(t), np.cos(t)]])


@pytest.mark.parametrize("theta,lr", [(0.3, 0.1), (-1.2, 0.7), (2.0, 3.0)])
def test_2x2_closed_form(theta, lr):
    R = _rot(theta)
    G = np.array([[0.4, -1.3], [0.9, 0.2]])
    M = G @ R.T
    a = M[0, 1] - M[1, 0]  # A = [[0, a], [-a, 0]]
    Rn, A = oracle.cayley_step(R, G, lr, want_A=True)
    assert np.allclose(A, [[0, a], [-a, 0]], atol=1e-15)
    # with t = lr a / 2: (I + tJ)^-1 (I - tJ), J = [[0,1],[-1,0]], equals
    # [[1-t^2, -2t], [2t, 1-t^2]] / (1+t^2), the rotation by phi = 2 atan(t)
    phi = 2 * np.arctan(lr * a / 2)
    assert np.allclose(Rn, _rot(phi) @ R, atol=1e-14)


@pytest.mark.parametrize("d,lr", [(8, 0.01), (64, 0.5), (96, 5.0)])
def test_orthogonality_det_and_library_solve(d, lr):
    rng = np.random.default_rng(d)
    R, _ = np.linalg.qr(rng.standard_normal((d, d)))
    G = rng.standard_normal((d, d))
    Rn, A = oracle.cayley_step(R, G, lr, want_A=True)
    assert np.allclose(A, -A.T, atol=1e-14)
    assert np.linalg.norm(Rn.T @ Rn - np.eye(d)) < 1e-6   # the bar the method needs
    assert np.linalg.norm(Rn.T @ Rn - np.eye(d)) < 1e-12  # what fp64 delivers
    assert np.linalg.det(Rn) == pytest.approx(np.linalg.det(R), rel=1e-10)
    A_ref = G @ R.T - R @ G.T
    ref = np.linalg.solve(np.eye(d) + 0.5 * lr * A_ref, (np.eye(d) - 0.5 * lr * A_ref) @ R)
    assert np.allclose(Rn, ref, atol=1e-12)


def test_fixed_point_when_gradient_is_radial():
    d = 12
    rng = np.random.default_rng(1)
    R, _ = np.linalg.qr(rng.standard_normal((d, d)))
    S = rng.standard_normal((d, d))
    S = S + S.T
    # G = R S with S symmetric gives A = R S R^T - R S^T R^T = 0
    Rn, A = oracle.cayley_step(R, R @ S, 0.3, want_A=True)
    assert np.allclose(A, 0, atol=1e-13)
    assert np.allclose(Rn, R, atol=1e-13)


def test_first_order_expansion():
    d = 10
    rng = np.random.default_rng(2)
    R, _ = np.linalg.qr(rng.standard_normal((d, d)))
    G = rng.standard_normal((d, d))
    A = G @ R.T - R @ G.T
    errs = []
    for lr in (1e-2, 5e-3):
        Rn = oracle.cayley_step(R, G, lr)
        errs.append(np.linalg.norm(Rn - (R - lr * A @ R)))
    # the remainder is O(lr^2): halving lr quarters it
    assert errs[0] / errs[1] == pytest.approx(4.0, rel=0.05)
    # <G, A R> = 1/2 ||A||_F^2 >= 0: the step is a descent direction for any G
    assert (G * (A @ R)).sum() == pytest.approx(0.5 * np.linalg.norm(A) ** 2, rel=1e-12)


def test_left_and_right_forms_agree():
    d = 20
    rng = np.random.default_rng(3)
    R, _ = np.linalg.qr(rng.standard_normal((d, d)))
    G = rng.standard_normal((d, d))
    assert np.allclose(oracle.cayley_step(R, G, 0.2), oracle.cayley_step_right(R, G, 0.2), atol=1e-12)


def test_step_lowers_kurtosis_loss():
    # qualitative claim of the method: rotating by the learned step lowers the kurtosis
    rng = np.random.default_rng(4)
    n, d = 256, 16
    X = rng.standard_normal((n, d))
    X[:, 3] *= 30.0
    R = np.eye(d)
    losses = []
    for _ in range(5):
        out = oracle.loss_grad(X, R)
        losses.append(out["loss"])
        R = oracle.cayley_step(R, out["dR"], 2e-2)
    assert all(b < a for a, b in zip(losses, losses[1:]))
    assert np.linalg.norm(R.T @ R - np.eye(d)) < 1e-12
    # small-step decrease ~ lr * 1/2 ||A||_F^2
    out = oracle.loss_grad(X, np.eye(d))
    lr = 1e-6
    Rn, A = oracle.cayley_step(np.eye(d), out["dR"], lr, want_A=True)
    l1 = oracle.loss_grad(X, Rn, want_dR=False)["loss"]
    assert (out["loss"] - l1) == pytest.approx(lr * 0.5 * np.linalg.norm(A) ** 2, rel=1e-3)
