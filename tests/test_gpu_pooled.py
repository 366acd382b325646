"""GPU parity of kt_pooled_kurtosis_loss_grad (the loss as the paper writes it: pooled kurtosis of
the RMSNorm-ed rotated activations) against the fp64 oracle.  Tolerances as for the per-row loss:
fp32 path 1e-4, bf16 path 2e-2 (loss and kappa relative, dR Frobenius relative)."""
import numpy as np
import pytest
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt
from parity_util import rel_fro

pytestmark = pytest.mark.gpu


def _gpu(X, R, kt_, eps, want_dR=True):
    Xd, Rd = X.cuda(), R.cuda()
    b, n, d = Xd.shape
    loss = torch.zeros(b, device="cuda")
    kap = torch.zeros(b, device="cuda")
    dR = torch.empty((b, d, d), device="cuda") if want_dR else None
    kt.kt_pooled_kurtosis_loss_grad(Xd, Rd, kappa_target=kt_, rms_eps=eps, loss=loss, kappa=kap, dR=dR)
    torch.cuda.synchronize()
    return loss.cpu().numpy(), kap.cpu().numpy(), None if dR is None else dR.cpu().numpy()


def _check(X, R, kt_, eps, tol, bf16):
    loss, kap, dR = _gpu(X, R, kt_, eps)
    for b in range(X.shape[0]):
        Rb = ktgen.bf16_round(R[b]) if bf16 else R[b]
        o = oracle.pooled_loss_grad(ktgen.to_f64(X[b]), ktgen.to_f64(Rb), kappa_target=kt_, rms_eps=float(np.float32(eps)))
        assert abs(kap[b] - o["kappa"]) <= tol * o["kappa"], (kap[b], o["kappa"])
        assert abs(loss[b] - o["loss"]) <= tol * max(o["loss"], o["kappa"] * 1e-2), (loss[b], o["loss"])
        assert rel_fro(dR[b], o["dR"]) <= tol, rel_fro(dR[b], o["dR"])
    l2, k2, _ = _gpu(X, R, kt_, eps, want_dR=False)
    assert np.array_equal(l2, loss) and np.array_equal(k2, kap)


@pytest.mark.parametrize("n,d,batch,kt_,eps", [(2048, 256, 1, 1.8, 0.0), (700, 128, 2, 1.8, 1e-5), (1000, 384, 1, 0.0, 0.0)])
def test_fp32_against_oracle(n, d, batch, kt_, eps):
    X, R, cfg = ktgen.make_problem("C1", seed=n, n=n, batch=batch) if d == 256 else (None, None, None)
    if X is None:
        X = ktgen.make_x(n * batch, d, seed=n, outlier_cols=4, outlier_scale=30.0, dtype="f32").reshape(batch, n, d)
        R = torch.stack([ktgen.random_orthogonal(d, seed=b) for b in range(batch)])
    _check(X, R, kt_, eps, 1e-4, bf16=False)


@pytest.mark.parametrize("n,d,batch,kt_,eps", [(3000, 256, 1, 1.8, 0.0), (1500, 128, 3, 1.8, 1e-6), (1200, 512, 1, 1.8, 0.0),
                                                (9000, 256, 1, 0.0, 0.0)])
def test_bf16_against_oracle(n, d, batch, kt_, eps):
    X = ktgen.make_x(n * batch, d, seed=d + n, outlier_cols=8, outlier_scale=40.0, t_frac=0.05,
                     dtype="bf16").reshape(batch, n, d)
    R = torch.stack([ktgen.random_orthogonal(d, seed=20 + b) for b in range(batch)])
    _check(X, R, kt_, eps, 2e-2, bf16=True)


def test_row_scaling_invariance_and_zero_rows():
    n, d = 1024, 256
    X = ktgen.make_x(n, d, seed=1, outlier_cols=4, outlier_scale=20.0, dtype="f32").reshape(1, n, d)
    R = ktgen.random_orthogonal(d, seed=2).unsqueeze(0)
    l0, k0, g0 = _gpu(X, R, 1.8, 0.0)
    X2 = X.clone()
    X2[0, ::2] *= 8.0          # RMSNorm removes any per-token scale (powers of two: exactly)
    l1, k1, g1 = _gpu(X2, R, 1.8, 0.0)
    assert abs(k1[0] - k0[0]) <= 1e-5 * k0[0]
    X3 = X.clone()
    X3[0, 5] = 0.0             # a token of zeros: z = 0, no gradient, still counted in N
    l3, k3, g3 = _gpu(X3, R, 1.8, 0.0)
    o = oracle.pooled_loss_grad(ktgen.to_f64(X3[0]), ktgen.to_f64(R[0]))
    assert np.isfinite(g3).all() and abs(k3[0] - o["kappa"]) <= 1e-4 * o["kappa"]
    assert rel_fro(g3[0], o["dR"]) <= 1e-4
