"""GPU parity: kt_cayley_step through the C ABI against the oracle's exact (LU) Cayley step."""
import numpy as np
import pytest
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt
from parity_util import rel_fro

pytestmark = pytest.mark.gpu


def _run(R, G, lr, want_lowp=True):
    Rd = R.clone().cuda().contiguous()
    Gd = G.cuda().contiguous()
    b, d = Rd.shape[0], Rd.shape[-1]
    lowp = torch.zeros((b, d, d), dtype=torch.bfloat16, device="cuda") if want_lowp else None
    oe = torch.full((b,), float("nan"), device="cuda")
    info = torch.zeros((b,), dtype=torch.int32, device="cuda")
    kt.kt_cayley_step(Rd, Gd, lr, R_lowp=lowp, ortho_err=oe, info=info)
    torch.cuda.synchronize()
    return Rd.cpu(), None if lowp is None else lowp.cpu(), oe.cpu().numpy(), info.cpu().numpy()


@pytest.mark.parametrize("d,batch,lr,gscale", [(128, 1, 1e-2, 1.0), (128, 3, 0.05, 1.0), (128, 40, 0.02, 2.0), (256, 1, 1e-2, 3.0),
                                                (384, 2, 1e-3, 10.0), (512, 1, 1e-2, 1.0)])
def test_against_oracle(d, batch, lr, gscale):
    g = torch.Generator().manual_seed(d + batch)
    R = torch.stack([ktgen.random_orthogonal(d, seed=b) for b in range(batch)])
    G = torch.randn((batch, d, d), generator=g) * gscale / np.sqrt(d)
    Rn, lowp, oe, info = _run(R, G, lr)
    for b in range(batch):
        ref = oracle.cayley_step(ktgen.to_f64(R[b]), ktgen.to_f64(G[b]), lr)
        step = ref - ktgen.to_f64(R[b])
        assert rel_fro(Rn[b].numpy().astype(np.float64) - ktgen.to_f64(R[b]), step) <= 1e-4
        RtR = Rn[b].double().T @ Rn[b].double()
        assert float((RtR - torch.eye(d, dtype=torch.float64)).abs().max()) < 1e-6
        # the library's own figure is an fp32 GEMM: true value plus a few ulp of 1
        assert oe[b] < 1e-6 and abs(oe[b] - float((RtR - torch.eye(d, dtype=torch.float64)).abs().max())) < 6e-7
        assert 1 <= info[b] <= 32
    assert torch.equal(lowp, Rn.to(torch.bfloat16))


@pytest.mark.parametrize("d,lr,gscale", [(1024, 1e-2, 1.0), (1024, 0.2, 2.0), (2048, 1e-2, 1.0)])
def test_large_d_three_term_bf16_path(d, lr, gscale):
    # d >= 1024 runs its GEMMs as three-term bf16 products; same bars as the fp32 path
    g = torch.Generator().manual_seed(d)
    R = ktgen.random_orthogonal(d, seed=3).unsqueeze(0)
    G = torch.randn((1, d, d), generator=g) * gscale / np.sqrt(d)
    Rn, lowp, oe, info = _run(R, G, lr)
    ref = oracle.cayley_step(ktgen.to_f64(R[0]), ktgen.to_f64(G[0]), lr)
    assert rel_fro(Rn[0].numpy().astype(np.float64) - ktgen.to_f64(R[0]), ref - ktgen.to_f64(R[0])) <= 1e-4
    RtR = Rn[0].double().T @ Rn[0].double()
    assert float((RtR - torch.eye(d, dtype=torch.float64)).abs().max()) < 1e-6
    assert oe[0] < 1e-6 and 1 <= info[0] <= 32
    if lr >= 0.2:
        assert info[0] > 8          # long enough to run the late, single-launch form of an iteration too
    assert torch.equal(lowp, Rn.to(torch.bfloat16))


def _spectral_norm(A, iters=60):
    """Largest singular value by power iteration on A^T A (host, fp64)."""
    v = np.random.default_rng(0).standard_normal(A.shape[0])
    for _ in range(iters):
        v = A.T @ (A @ v)
        v /= np.linalg.norm(v)
    return float(np.linalg.norm(A @ v))


def test_d4096_headline_tiles_against_oracle():
    """The retraction as the benchmark's configuration runs it (d = 4096: 256 x 256 tiles, three-term bf16
    products), against the oracle's exact LU solve ("Optimization in the Orthogonal Space").  R is C3's rotation,
    the gradient is the oracle's own dR on a 512-row chunk of C3's activations (rounded to fp32 for both
    sides).  Two steps: lr = 1e-2 (converges in a few iterations) and a step sized so that
    (lr/2) ||A||_2 = 0.4, which needs more than eight iterations and so runs the late, single-launch form of
    an iteration as well."""
    X, R, cfg = ktgen.make_problem("C3", seed=0, n=512)
    d = cfg["d"]
    assert d == 4096
    Ro = ktgen.to_f64(R[0])
    dRo = oracle.loss_grad(ktgen.to_f64(X[0]), ktgen.to_f64(ktgen.bf16_round(R[0])))["dR"]
    G = torch.tensor(dRo, dtype=torch.float32).unsqueeze(0)
    Go = ktgen.to_f64(G[0])
    A = Go @ Ro.T
    A = A - A.T
    lr_big = 2 * 0.4 / _spectral_norm(A)
    for lr, long_run in ((1e-2, False), (float(np.float32(lr_big)), True)):
        Rn, lowp, oe, info = _run(R, G, lr)
        ref = oracle.cayley_step(Ro, Go, lr)
        rel = rel_fro(Rn[0].numpy().astype(np.float64) - Ro, ref - Ro)
        assert rel <= 1e-4, (lr, rel)
        RtR = Rn[0].double().T @ Rn[0].double()
        assert float((RtR - torch.eye(d, dtype=torch.float64)).abs().max()) < 1e-6
        assert oe[0] < 1e-6 and 1 <= info[0] <= 32
        if long_run:
            assert info[0] > 8, info
        assert torch.equal(lowp, Rn.to(torch.bfloat16))


def test_zero_step_and_radial_gradient():
    d = 128
    R = ktgen.random_orthogonal(d, seed=4).unsqueeze(0)
    G = torch.randn((1, d, d), generator=torch.Generator().manual_seed(1))
    Rn, _, _, info = _run(R, G, 0.0)
    assert torch.equal(Rn, R) and info[0] == 1
    S = G[0] + G[0].T
    Rn, _, _, _ = _run(R, (R[0] @ S).unsqueeze(0), 0.01)     # A = R S R^T - R S R^T = 0
    assert float((Rn - R).abs().max()) < 1e-6


@pytest.mark.parametrize("d", [128, 256, 1024])   # single-workgroup kernel, fp32 GEMM path, three-term bf16 path
def test_divergent_step_is_flagged_and_rejected(d):
    # (lr/2)||A|| >> 1: the fixed point does not contract; the library must say so, and R (with its
    # bf16 copy) must come back as it went in rather than as the last, meaningless iterate
    R = ktgen.random_orthogonal(d, seed=4).unsqueeze(0)
    G = torch.randn((1, d, d), generator=torch.Generator().manual_seed(2))
    Rn, lowp, _, info = _run(R, G, 10.0)
    assert info[0] == -1
    assert torch.equal(Rn, R)
    assert torch.equal(lowp, R.to(torch.bfloat16))


def test_teacher_forced_steps_c1():
    # three consecutive loss+grad+Cayley steps on the Tiny config; at every step the GPU starts
    # from the oracle's R so that chaotic drift cannot build up
    X, R, cfg = ktgen.make_problem("C1", seed=0, n=1024)
    Xd = X.cuda()
    Xo = ktgen.to_f64(X[0])
    Ro = ktgen.to_f64(R[0])
    losses = []
    for _ in range(3):
        o = oracle.loss_grad(Xo, Ro)
        Rd = torch.tensor(Ro, dtype=torch.float32).unsqueeze(0).cuda()
        dR = torch.empty_like(Rd)
        loss = kt.kt_kurtosis_loss_grad(Xd, Rd, dR=dR)
        kt.kt_cayley_step(Rd, dR, cfg["lr"] * 50)
        torch.cuda.synchronize()
        Rnext = oracle.cayley_step(Ro, o["dR"], cfg["lr"] * 50)
        assert abs(loss.item() - o["loss"]) <= 1e-4 * o["loss"]
        assert rel_fro(dR[0].cpu().numpy(), o["dR"]) <= 1e-4
        assert rel_fro(Rd[0].cpu().numpy().astype(np.float64) - Ro, Rnext - Ro) <= 2e-4
        losses.append(o["loss"])
        Ro = Rnext
    assert losses[2] < losses[0]


@pytest.mark.parametrize("d", [128, 256, 1024])
def test_non_finite_gradient_never_reaches_the_rotation(d):
    # a NaN in the gradient (say, from a NaN activation): the fixed point cannot converge on it, the call reports
    # -1 and leaves R untouched, so a training loop stalls visibly instead of filling R with NaNs
    R = ktgen.random_orthogonal(d, seed=7).unsqueeze(0)
    G = torch.randn((1, d, d), generator=torch.Generator().manual_seed(3)) * 0.1
    G[0, 5, 9] = float("nan")
    Rn, lowp, _, info = _run(R, G, 0.01)
    assert info[0] == -1 and torch.equal(Rn, R) and torch.equal(lowp, R.to(torch.bfloat16))
