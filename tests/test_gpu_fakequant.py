"""GPU parity: kt_rotate_fakequant_int4 through the C ABI against the oracle.

Codes are integer work: they must be bit-exact whenever the rotated activations are exactly
representable (so that fp32 and fp64 accumulation agree bit for bit), and with the oracle's
scales handed in they may differ from the oracle's only where y/s sits on a rounding boundary
within the fp32 accumulation error, and then by one code."""
import numpy as np
import pytest
import scipy.linalg
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt

pytestmark = pytest.mark.gpu


def _run(X, R, clip=1.0, scales_in=None):
    Xd, Rd = X.cuda(), R.cuda()
    if Xd.dim() == 2:
        Xd, Rd = Xd.unsqueeze(0), Rd.unsqueeze(0)
    b, n, d = Xd.shape
    so = torch.full((b, n), float("nan"), device="cuda")
    codes = torch.full((b, n, d), 99, dtype=torch.int8, device="cuda")
    err = torch.full((b, n, 2), float("nan"), device="cuda")
    sin = None if scales_in is None else torch.as_tensor(scales_in, dtype=torch.float32).reshape(b, n).cuda()
    kt.kt_rotate_fakequant_int4(Xd, Rd, clip_ratio=clip, scales_in=sin, scales_out=so, codes=codes, err=err)
    torch.cuda.synchronize()
    return so.cpu().numpy(), codes.cpu().numpy(), err.cpu().numpy()


def _oracle(X, R, clip=1.0, scales_in=None, bf16=True):
    Rr = ktgen.bf16_round(R) if bf16 else R
    return oracle.fakequant_int4(ktgen.to_f64(X), ktgen.to_f64(Rr), clip=clip, scales_in=scales_in)


@pytest.mark.parametrize("n,d", [(300, 128), (1000, 256), (257, 384)])
def test_bit_exact_identity_rotation(n, d):
    # Y = X exactly, heavy-tailed values: scales and codes must match bit for bit
    X = ktgen.make_x(n, d, seed=n, base="t4", outlier_cols=2, outlier_scale=50.0, dtype="bf16")
    R = torch.eye(d)
    s, c, e = _run(X, R)
    o = _oracle(X, R)
    assert np.array_equal(s[0], o["scales"])
    assert np.array_equal(c[0], o["codes"])
    assert np.allclose(e[0], o["err"], rtol=1e-4, atol=1e-30)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_bit_exact_hadamard_of_small_integers(dtype):
    # integers times +-1/16: every partial sum is exact in fp32, whatever the order
    n, d = 700, 256
    g = torch.Generator().manual_seed(3)
    X = torch.randint(-8, 9, (n, d), generator=g).to(torch.bfloat16 if dtype == "bf16" else torch.float32)
    X[:, 7] *= 6
    H = torch.tensor(scipy.linalg.hadamard(d) / 16.0, dtype=torch.float32)
    for clip in (1.0, 0.6):
        s, c, e = _run(X, H, clip=clip)
        o = _oracle(X, H, clip=clip, bf16=(dtype == "bf16"))
        assert np.array_equal(s[0], o["scales"])
        assert np.array_equal(c[0], o["codes"])
        assert np.allclose(e[0], o["err"], rtol=1e-4, atol=1e-30)


@pytest.mark.parametrize("dtype,n,d,batch", [("bf16", 600, 256, 1), ("bf16", 200, 128, 2), ("bf16", 5000, 128, 3), ("bf16", 300, 512, 1),
                                              ("f32", 500, 256, 1)])
def test_general_rotation_with_given_scales(dtype, n, d, batch):
    for b in range(batch):
        X = ktgen.make_x(n, d, seed=40 + b, outlier_cols=4, outlier_scale=50.0, t_frac=0.05, dtype=dtype)
        R = ktgen.random_orthogonal(d, seed=41 + b)
        o = _oracle(X, R, bf16=(dtype == "bf16"))
        # own scales: equal up to the fp32 accumulation error of the row maximum
        s, c, e = _run(X, R)
        assert np.allclose(s[0], o["scales"], rtol=1e-5)
        # oracle's scales handed in: codes may differ only on rounding boundaries, by one
        s2, c2, e2 = _run(X, R, scales_in=o["scales"])
        assert np.array_equal(s2[0], o["scales"])
        Rr = ktgen.bf16_round(R) if dtype == "bf16" else R
        Y = ktgen.to_f64(X) @ ktgen.to_f64(Rr)
        t = Y / o["scales"].astype(np.float64)[:, None]
        diff = c2[0].astype(np.int32) - o["codes"].astype(np.int32)
        bad = diff != 0
        assert np.abs(diff).max() <= 1
        assert np.all(np.abs(np.abs(t[bad]) % 1.0 - 0.5) < 1e-3)
        assert bad.mean() < 1e-3
        assert np.allclose(e2[0], o["err"], rtol=1e-3)
        assert c2.min() >= -7 and c2.max() <= 7


def test_scales_only_and_zero_rows():
    n, d = 130, 128
    X = ktgen.make_x(n, d, seed=8, dtype="bf16")
    X[5] = 0
    R = torch.eye(d)
    s, c, e = _run(X, R)
    assert s[0, 5] == 0 and np.all(c[0, 5] == 0) and np.all(e[0, 5] == 0)
    so = torch.empty((1, n), device="cuda")
    kt.kt_rotate_fakequant_int4(X.cuda(), R.cuda(), scales_out=so)
    torch.cuda.synchronize()
    assert np.array_equal(so.cpu().numpy(), s)


def test_single_pass_d128_batched_with_row_stride_matches_the_contiguous_call():
    n, d, batch = 700, 128, 3
    Xfull = ktgen.make_x(n * batch, 192, seed=17, outlier_cols=3, outlier_scale=30.0, dtype="bf16").reshape(batch, n, 192).cuda()
    Xv, Xc = Xfull[:, :, :d], Xfull[:, :, :d].contiguous()
    R = torch.stack([ktgen.random_orthogonal(d, seed=50 + b) for b in range(batch)]).cuda()
    outs = []
    for X in (Xv, Xc):
        codes = torch.empty((batch, n, d), dtype=torch.int8, device="cuda")
        scales = torch.empty((batch, n), device="cuda")
        err = torch.empty((batch, n, 2), device="cuda")
        kt.kt_rotate_fakequant_int4(X, R, scales_out=scales, codes=codes, err=err)
        torch.cuda.synchronize()
        outs.append((codes.cpu(), scales.cpu(), err.cpu()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    ref = oracle.fakequant_int4(ktgen.to_f64(Xc[1].cpu()), ktgen.to_f64(ktgen.bf16_round(R[1].cpu())))
    assert np.allclose(outs[0][1][1].numpy(), ref["scales"], rtol=1e-2)
