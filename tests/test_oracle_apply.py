"""Pins of the oracle's "apply the rotation" functions ("Placement of the Rotations": online random
Hadamard rotations R3-R5, fusible rotations merged into the weights).  Pinned by scipy's Hadamard
matrix (a routine the oracle does not use), the Sylvester recursion written out in numpy,
orthogonality / involution, one-hot rows, numpy matmul, and the computational-invariance identity
the paper relies on.  The Paley factors used for sizes that are not powers of two are pinned by the
definition of a Hadamard matrix (H H^T = m I), their textbook symmetry types, Euler's criterion for
the quadratic character and a dense Kronecker product built with numpy."""
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


def _supported_orders():
    out = []
    for r in range(3, 64, 2):
        f = oracle.hadamard_factor(r * 4096)
        if f is not None:
            out.append(f)
    return out


def test_every_paley_factor_is_a_hadamard_matrix():
    """H H^T = m I with entries +-1 is the whole definition of a Hadamard matrix; Paley's first
    construction gives a skew-type matrix (H + H^T = 2 I), the second a symmetric one."""
    fs = _supported_orders()
    assert {(28, 2), (12, 1), (20, 1), (108, 1), (36, 2), (44, 1)} <= {(m, kind) for m, _, kind in fs}
    for m, p2, kind in fs:
        H = oracle.hadamard_matrix(m, kind).astype(np.int64)
        assert set(np.unique(H)) == {-1, 1}, (m, kind)
        assert np.array_equal(H @ H.T, m * np.eye(m, dtype=np.int64)), (m, kind)
        if kind == 1:
            assert np.array_equal(H + H.T, 2 * np.eye(m, dtype=np.int64))
        else:
            assert np.array_equal(H, H.T)


def test_quadratic_character_through_eulers_criterion():
    """Row 1 of the Paley I matrix holds chi(1 - j): compare with x^((q-1)/2) mod q."""
    for m in (12, 20, 44, 108):
        q = m - 1
        H = oracle.hadamard_matrix(m, 1)
        for j in range(2, m):
            x = (1 - j) % q
            e = pow(x, (q - 1) // 2, q)
            assert H[1, j] == (1 if e == 1 else -1), (m, j)
    for m in (28, 36):                       # Paley II: block (0, 0) is C + I, C[1][v] = chi(1 - v)
        q = m // 2 - 1
        H = oracle.hadamard_matrix(m, 2)
        for v in range(2, q + 1):
            e = pow((1 - v) % q, (q - 1) // 2, q)
            assert H[1, v] == (1 if e == 1 else -1), (m, v)


def test_how_model_sizes_split():
    """Hidden and FFN sizes of the model families in the Setup."""
    assert oracle.hadamard_factor(4096) == (1, 4096, 0)
    assert oracle.hadamard_factor(8192) == (4, 2048, 0)
    assert oracle.hadamard_factor(14336) == (28, 512, 2)     # 7 * 2^11
    assert oracle.hadamard_factor(28672) == (28, 1024, 2)
    assert oracle.hadamard_factor(13824) == (108, 128, 1)    # 27 * 2^9
    assert oracle.hadamard_factor(5120) == (20, 256, 1)
    assert oracle.hadamard_factor(6144) == (12, 512, 1)
    assert oracle.hadamard_factor(11008) is None             # 43 * 2^8: no Paley order up to 256


@pytest.mark.parametrize("d", [96, 160, 224, 288, 8192])
def test_general_hadamard_rows_against_a_dense_kronecker_product(d):
    m, p2, kind = oracle.hadamard_factor(d)
    rng = np.random.default_rng(d)
    n = 3 if d < 1000 else 2
    X = rng.standard_normal((n, d))
    s = rng.choice([-1.0, 1.0], size=d)
    Y = oracle.hadamard_rows(X, s)
    Hm = oracle.hadamard_matrix(m, kind).astype(np.float64)
    Hd = np.kron(Hm, scipy.linalg.hadamard(p2).astype(np.float64))
    if kind == 0:
        assert np.array_equal(Hd, scipy.linalg.hadamard(d))          # Sylvester (x) Sylvester = Sylvester
    assert np.abs(Y - (X * s) @ Hd / np.sqrt(d)).max() < 1e-11
    assert np.allclose((Y ** 2).sum(1), (X ** 2).sum(1), rtol=1e-12)
    assert np.abs((Y @ Hd.T / np.sqrt(d)) * s - X).max() < 1e-11     # the transposed matrix undoes it


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
