"""Pins of the oracle's "apply the rotation" functions ("Placement of the Rotations": online random
Hadamard rotations R3-R5, fusible rotations merged into the weights).  Pinned by scipy's Hadamard
matrix (a routine the oracle does not use), the Sylvester recursion written out in numpy,
orthogonality / involution, one-hot rows, numpy matmul, and the computational-invariance identity
the paper relies on."""
import numpy as np
import pytest
import scipy.linalg

import oracle


@pytest.mark.parametrize("d", [2, 8, 64, 256])
def test_hadamard_is_scipys_and_the_recursion(d):
    rng = np.random.default_rng(d)
    X = rng.standard_normal((5, d))
    s = rng.choice([-1.0, 1.0], size=d)
    Y = oracle.hadamard_rows(X, s)
    H = scipy.linalg.hadamard(d).astype(np.float64)
    assert np.abs(Y - (X * s) @ H / np.sqrt(d)).max() < 1e-12
    Hr = np.array([[1.0]])
    while Hr.shape[0] < d:
        Hr = np.block([[Hr, Hr], [Hr, -Hr]])
    assert np.array_equal(Hr, H)
    # orthogonal: norms preserved; without signs the transform is its own inverse
    assert np.allclose((Y ** 2).sum(1), (X ** 2).sum(1), rtol=1e-12)
    assert np.abs(oracle.hadamard_rows(oracle.hadamard_rows(X)) - X).max() < 1e-12


def test_hadamard_spreads_a_one_hot_row():
    d = 128
    X = np.eye(d)[[3, 77]] * 9.0
    Y = oracle.hadamard_rows(X)
    assert np.allclose(np.abs(Y), 9.0 / np.sqrt(d))
    assert np.array_equal(np.sign(Y[0]), scipy.linalg.hadamard(d)[3])


def test_fuse_rotation_is_matmul_and_keeps_the_layer_output():
    rng = np.random.default_rng(1)
    d, k, n = 24, 40, 9
    q, r = np.linalg.qr(rng.standard_normal((d, d)))
    R = q * np.sign(np.diag(r))
    Wd = rng.standard_normal((k, d))          # a weight whose output feeds the residual stream: W R
    Wu = rng.standard_normal((d, k))          # a weight that reads the residual stream: R^T W
    assert np.abs(oracle.fuse_rotation(Wd, R, 0) - Wd @ R).max() < 1e-12
    assert np.abs(oracle.fuse_rotation(Wu, R, 1) - R.T @ Wu).max() < 1e-12
    # computational invariance: rotated activations times the fused weight give the original output
    X = rng.standard_normal((n, d))
    assert np.abs((X @ R) @ oracle.fuse_rotation(Wu, R, 1) - X @ Wu).max() < 1e-12
    H = rng.standard_normal((n, k))
    assert np.abs(H @ oracle.fuse_rotation(Wd, R, 0) - (H @ Wd) @ R).max() < 1e-12
