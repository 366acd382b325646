"""Pins of the oracle's Cayley Adam step (the optimiser the paper names in "Learning the
Rotations" and in its Setup appendix and defers to the cited work on Stiefel-manifold
optimisation for).  The paper prints no formula, so there are no printed values to compare with;
the step is pinned by what the mathematics fixes: its reduction to the Cayley SGD step, the 2x2
closed form, numpy's solver on the same transform, the orthogonal-group invariants, the
tangent-space projection written independently, and the scalar recurrences worked by hand."""
import numpy as np
import pytest

import oracle


def _rand_orth(d, seed):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((d, d)))
    return q * np.sign(np.diag(r))


def test_beta1_zero_first_step_is_a_cayley_sgd_step():
    # beta1 = 0, k = 1: M1 = G, r = sqrt(v1/(1-beta2) + eps), W = (G R^T - R G^T)/(2 r) for orthogonal R,
    # so the step equals the SGD retraction with lr_eff = alpha / (2 r)
    d, lr, b2, eps = 12, 0.03, 0.99, 1e-8
    rng = np.random.default_rng(1)
    R, G = _rand_orth(d, 1), rng.standard_normal((d, d))
    o = oracle.cayley_adam_step(R, G, np.zeros((d, d)), 1.0, 1, lr, beta1=0.0, beta2=b2, eps=eps, q=0.5)
    v1 = b2 * 1.0 + (1 - b2) * (G ** 2).sum()
    r = np.sqrt(v1 / (1 - b2) + eps)
    assert abs(o["v"] - v1) < 1e-12 * v1 and abs(o["r"] - r) < 1e-12 * r
    wn = np.linalg.norm(G @ R.T - R @ G.T) / (2 * r)
    assert abs(o["w_norm"] - wn) < 1e-10 * wn
    alpha = min(lr, 2 * 0.5 / (wn + eps))
    assert abs(o["alpha"] - alpha) < 1e-12
    ref = oracle.cayley_step(R, G, alpha / (2 * r))
    assert np.abs(o["R"] - ref).max() < 1e-12


def test_two_by_two_closed_form():
    # d = 2: W = [[0, w], [-w, 0]] and the transform is a rotation by phi = 2 atan(alpha w / 2)
    th = 0.4
    R = np.array([[np.cos(th), -np.sin(th)], [np.sin(th), np.cos(th)]])
    G = np.array([[0.3, -1.1], [0.7, 0.2]])
    M0 = np.array([[0.1, 0.2], [-0.3, 0.05]])
    b1, b2, eps, lr, k, v0 = 0.9, 0.99, 1e-8, 0.5, 3, 2.0
    o = oracle.cayley_adam_step(R, G, M0, v0, k, lr, beta1=b1, beta2=b2, eps=eps, q=0.5)
    M1 = b1 * M0 + (1 - b1) * G
    v1 = b2 * v0 + (1 - b2) * (G ** 2).sum()
    r = (1 - b1 ** k) * np.sqrt(v1 / (1 - b2 ** k) + eps)
    Wh = 0.5 * M1 @ R.T
    w = (Wh[0, 1] - Wh[1, 0]) / r
    alpha = min(lr, 1.0 / (abs(w) * np.sqrt(2) + eps))
    phi = 2 * np.arctan(alpha * w / 2)
    # (I + a/2 W)^-1 (I - a/2 W) with W = w J, J = [[0,1],[-1,0]], is the rotation [[c, -s], [s, c]] by phi
    rot = np.array([[np.cos(phi), -np.sin(phi)], [np.sin(phi), np.cos(phi)]])
    assert np.abs(o["R"] - rot @ R).max() < 1e-13
    assert abs(o["alpha"] - alpha) < 1e-14


@pytest.mark.parametrize("d,k,lr", [(8, 1, 0.01), (16, 5, 0.1), (24, 40, 3.0)])
def test_invariants_and_numpy_solve(d, k, lr):
    rng = np.random.default_rng(d + k)
    R, G, M0 = _rand_orth(d, d), rng.standard_normal((d, d)), 0.1 * rng.standard_normal((d, d))
    b1, b2, eps, q, v0 = 0.9, 0.99, 1e-8, 0.5, 1.3
    o = oracle.cayley_adam_step(R, G, M0, v0, k, lr, beta1=b1, beta2=b2, eps=eps, q=q)
    Rn, Mn = o["R"], o["M"]
    # stays on the orthogonal group, same component
    assert np.abs(Rn.T @ Rn - np.eye(d)).max() < 1e-12
    assert abs(np.linalg.det(Rn) - np.linalg.det(R)) < 1e-10
    # momentum after the step is tangent at R (R^T M skew) and is the canonical-metric projection
    # of M1, which for orthogonal R is (M1 - R M1^T R) / 2
    M1 = b1 * M0 + (1 - b1) * G
    assert np.abs(R.T @ Mn + Mn.T @ R).max() < 1e-12
    assert np.abs(Mn - 0.5 * (M1 - R @ M1.T @ R)).max() < 1e-12
    # the transform itself, rebuilt with numpy's solver from W = M+ R^T / r
    W = Mn @ R.T / o["r"]
    assert np.abs(W + W.T).max() < 1e-12
    assert abs(np.linalg.norm(W) - o["w_norm"]) < 1e-12 * max(1.0, o["w_norm"])
    a = o["alpha"]
    assert a == pytest.approx(min(lr, 2 * q / (o["w_norm"] + eps)), rel=1e-14)
    ref = np.linalg.solve(np.eye(d) + 0.5 * a * W, (np.eye(d) - 0.5 * a * W) @ R)
    assert np.abs(Rn - ref).max() < 1e-12
    # the clamp bounds the rotation: alpha ||W||_F <= 2 q
    assert a * o["w_norm"] <= 2 * q + 1e-12


def test_scalar_recurrences_by_hand():
    # G = diag(3, 4) on R = I: ||G||^2 = 25; M0 = 0, v0 = 1, k = 2, beta1 = 0.5, beta2 = 0.75
    R, G = np.eye(2), np.diag([3.0, 4.0])
    o = oracle.cayley_adam_step(R, G, np.zeros((2, 2)), 1.0, 2, 0.1, beta1=0.5, beta2=0.75, eps=0.0, q=0.5)
    assert o["v"] == pytest.approx(0.75 + 0.25 * 25.0)              # 7.0
    assert o["r"] == pytest.approx((1 - 0.25) * np.sqrt(7.0 / (1 - 0.5625)))  # 0.75 * 4 = 3.0
    # symmetric M1 R^T: no rotation at all, momentum projected to zero
    assert np.abs(o["R"] - R).max() < 1e-15 and np.abs(o["M"]).max() < 1e-15 and o["w_norm"] == 0.0


def test_descends_on_a_small_kurtosis_problem():
    rng = np.random.default_rng(0)
    n, d = 256, 16
    X = rng.standard_normal((n, d))
    X[:, 3] *= 30.0
    R = _rand_orth(d, 7)
    M, v = np.zeros((d, d)), 1.0
    losses = []
    for k in range(1, 31):
        lg = oracle.loss_grad(X, R)
        losses.append(lg["loss"])
        o = oracle.cayley_adam_step(R, lg["dR"], M, v, k, 0.05)
        R, M, v = o["R"], o["M"], o["v"]
    assert oracle.loss_grad(X, R, want_dR=False)["loss"] < 0.8 * losses[0]
    assert np.abs(R.T @ R - np.eye(d)).max() < 1e-11
