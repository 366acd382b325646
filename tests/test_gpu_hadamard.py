"""GPU parity of kt_hadamard_rows against the oracle's O(d^2) definition.
fp32: the transform adds d values with fp32 rounding in a tree of depth log2 d: 1e-5 of the row
norm per output.  bf16: the same fp32 result rounded to nearest even: at most one bf16 ulp
(2^-8 relative) from the oracle value rounded the same way, plus the fp32 term.  Sizes m 2^k with
m > 1 run as two factors with the intermediate z (the Sylvester transform of each of the m segments
of a row) stored in the output buffer: in bf16 that intermediate is rounded too, by at most 2^-8 |z|
each (the unit roundoff of an 8-bit significand), and an output is +-1/sqrt(m) times the sum of the m
intermediates of its column: the bound adds 2^-8 sum_j |z_j| / sqrt(m), with z from the oracle."""
import numpy as np
import pytest
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,d,dtype,use_signs", [(37, 128, "f32", False), (1000, 128, "bf16", True), (33, 256, "f32", True),
                                                  (515, 512, "bf16", False), (70, 1024, "f32", True), (9, 2048, "bf16", True),
                                                  (130, 4096, "bf16", False), (5, 4096, "f32", True)])
def test_against_oracle(n, d, dtype, use_signs):
    X = ktgen.make_x(n, d, seed=n + d, outlier_cols=3, outlier_scale=40.0, t_frac=0.02, dtype=dtype)
    g = torch.Generator().manual_seed(d)
    signs = (torch.randint(0, 2, (d,), generator=g) * 2 - 1).to(torch.int8) if use_signs else None
    Y = kt.kt_hadamard_rows(X.cuda(), signs=None if signs is None else signs.cuda())
    torch.cuda.synchronize()
    ref = oracle.hadamard_rows(ktgen.to_f64(X), None if signs is None else signs.numpy().astype(np.float64))
    got = Y.float().cpu().numpy().astype(np.float64)
    rown = np.linalg.norm(ref, axis=1, keepdims=True)
    tol = 1e-5 * rown + (np.abs(ref) * 2.0 ** -8 if dtype == "bf16" else 0.0)
    assert (np.abs(got - ref) <= tol).all(), float((np.abs(got - ref) / rown).max())


def _intermediate_rounding_bound(Xs, m, p2):
    """2^-8 sum_j |z_j| / sqrt(m) per output, z = the normalised Sylvester transform of the segments."""
    n, d = Xs.shape
    z = oracle.hadamard_rows(np.ascontiguousarray(Xs.reshape(n * m, p2)))
    colsum = np.abs(z).reshape(n, m, p2).sum(axis=1) / np.sqrt(m)
    return 2.0 ** -8 * 1.01 * np.tile(colsum, (1, m))


# d = m 2^k: Paley I (12, 20, 44, 108), Paley II (28, 36), Sylvester factor for powers of two > 4096;
# the cases with hundreds of rows reach the tail of the rounding-error distribution
@pytest.mark.parametrize("n,d,dtype,use_signs", [(40, 1536, "f32", True), (300, 3072, "bf16", True), (17, 5120, "f32", False),
                                                  (9, 4608, "bf16", True), (6, 5632, "f32", True), (5, 13824, "bf16", True),
                                                  (6, 14336, "bf16", True), (4, 14336, "f32", False), (3, 28672, "bf16", True),
                                                  (6, 8192, "f32", True), (3, 16384, "bf16", False), (329, 8192, "bf16", True)])
def test_sizes_that_are_not_powers_of_two_against_oracle(n, d, dtype, use_signs):
    m, p2, kind = oracle.hadamard_factor(d)
    assert m > 1
    X = ktgen.make_x(n, d, seed=n + d, outlier_cols=3, outlier_scale=40.0, t_frac=0.02, dtype=dtype)
    g = torch.Generator().manual_seed(d)
    signs = (torch.randint(0, 2, (d,), generator=g) * 2 - 1).to(torch.int8) if use_signs else None
    Y = kt.kt_hadamard_rows(X.cuda(), signs=None if signs is None else signs.cuda())
    torch.cuda.synchronize()
    sg = None if signs is None else signs.numpy().astype(np.float64)
    ref = oracle.hadamard_rows(ktgen.to_f64(X), sg)
    got = Y.float().cpu().numpy().astype(np.float64)
    rown = np.linalg.norm(ref, axis=1, keepdims=True)
    tol = 1e-5 * rown
    if dtype == "bf16":
        Xs = ktgen.to_f64(X) if sg is None else ktgen.to_f64(X) * sg[None, :]
        tol = tol + np.abs(ref) * 2.0 ** -8 + _intermediate_rounding_bound(Xs, m, p2)
    assert (np.abs(got - ref) <= tol).all(), float((np.abs(got - ref) / tol).max())
    assert np.allclose(np.linalg.norm(got, axis=1), np.linalg.norm(ktgen.to_f64(X), axis=1), rtol=3e-3)


def test_general_size_in_place_with_row_stride():
    n, d = 50, 3072
    buf = torch.randn(n, d + 64, device="cuda")
    X = buf[:, :d]
    ref = oracle.hadamard_rows(X.cpu().numpy().astype(np.float64))
    guard = buf[:, d:].clone()
    kt.kt_hadamard_rows(X, out=X)
    torch.cuda.synchronize()
    assert np.abs(X.cpu().numpy() - ref).max() < 1e-4
    assert torch.equal(buf[:, d:], guard)


def test_in_place_strided_and_involution():
    n, d = 300, 256
    buf = torch.randn(n, d + 64, device="cuda")
    X = buf[:, :d]                                   # row stride d + 64
    ref = oracle.hadamard_rows(X.cpu().numpy().astype(np.float64))
    guard = buf[:, d:].clone()
    kt.kt_hadamard_rows(X, out=X)
    torch.cuda.synchronize()
    assert np.abs(X.cpu().numpy() - ref).max() < 1e-4
    assert torch.equal(buf[:, d:], guard)            # nothing written past the d columns
    kt.kt_hadamard_rows(X, out=X)                    # H/sqrt(d) is its own inverse
    torch.cuda.synchronize()
    assert np.abs(oracle.hadamard_rows(ref) - X.cpu().numpy()).max() < 1e-4


def test_bad_shapes_are_refused():
    X = torch.zeros(4, 96, device="cuda")
    with pytest.raises(Exception):
        kt.kt_hadamard_rows(X)
    with pytest.raises(Exception):
        kt.kt_hadamard_rows(torch.zeros(4, 11008, device="cuda"))      # 43 * 2^8: no Paley order
    with pytest.raises(Exception):
        kt.kt_hadamard_rows(torch.zeros(4, 768, device="cuda"))        # 12 * 64: the power-of-two part is too short
