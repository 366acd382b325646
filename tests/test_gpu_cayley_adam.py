"""GPU parity of kt_cayley_adam_step against the fp64 oracle (exact Cayley transform).
Tolerance as for the SGD step: the step R+ - R to 1e-4 relative (Frobenius), the momentum to
1e-4, scalars to 1e-5, orthogonality max|R^T R - I| < 1e-6."""
import numpy as np
import pytest
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt
from parity_util import rel_fro

pytestmark = pytest.mark.gpu

# the ABI takes fp32 hyper-parameters: the oracle gets the same rounded values
F = lambda x: float(np.float32(x))
HP = dict(beta1=F(0.9), beta2=F(0.99), eps=F(1e-8), q=0.5)


def _gpu_step(R, G, M, v, k, lr, **kw):
    Rd, Gd, Md, vd = R.clone().cuda(), G.cuda().contiguous(), M.clone().cuda(), v.clone().cuda()
    b, d = Rd.shape[0], Rd.shape[-1]
    lowp = torch.empty((b, d, d), dtype=torch.bfloat16, device="cuda")
    oe = torch.zeros(b, device="cuda")
    info = torch.zeros(b, dtype=torch.int32, device="cuda")
    sc = torch.zeros((b, 3), device="cuda")
    kt.kt_cayley_adam_step(Rd, Gd, Md, vd, k, lr, R_lowp=lowp, ortho_err=oe, info=info, scalars=sc, **kw)
    torch.cuda.synchronize()
    return Rd.cpu(), Md.cpu(), vd.cpu(), lowp.cpu(), oe.cpu().numpy(), info.cpu().numpy(), sc.cpu().numpy()


@pytest.mark.parametrize("d,batch,k,lr,gscale", [(128, 1, 1, 1e-2, 1.0), (128, 3, 7, 0.5, 1.0), (256, 2, 2, 0.1, 5.0),
                                                   (512, 1, 30, 5.0, 1.0), (1024, 1, 3, 0.05, 1.0)])
def test_single_step_against_oracle(d, batch, k, lr, gscale):
    g = torch.Generator().manual_seed(d + batch + k)
    R = torch.stack([ktgen.random_orthogonal(d, seed=10 + b) for b in range(batch)])
    G = torch.randn((batch, d, d), generator=g) * gscale / np.sqrt(d)
    M = 0.3 * torch.randn((batch, d, d), generator=g) / np.sqrt(d)
    v = torch.rand(batch, generator=g) + 0.5
    Rn, Mn, vn, lowp, oe, info, sc = _gpu_step(R, G, M, v, k, lr)
    for b in range(batch):
        o = oracle.cayley_adam_step(ktgen.to_f64(R[b]), ktgen.to_f64(G[b]), ktgen.to_f64(M[b]), float(v[b]), k, F(lr), **HP)
        assert abs(vn[b].item() - o["v"]) <= 1e-6 * o["v"]
        assert abs(sc[b, 0] - o["r"]) <= 1e-5 * o["r"]
        assert abs(sc[b, 1] - o["alpha"]) <= 1e-5 * o["alpha"]
        assert abs(sc[b, 2] - o["w_norm"]) <= 1e-5 * o["w_norm"]
        step = o["R"] - ktgen.to_f64(R[b])
        assert rel_fro(Rn[b].numpy().astype(np.float64) - ktgen.to_f64(R[b]), step) <= 1e-4
        assert rel_fro(Mn[b].numpy().astype(np.float64), o["M"]) <= 1e-4
        RtR = Rn[b].double().T @ Rn[b].double()
        assert float((RtR - torch.eye(d, dtype=torch.float64)).abs().max()) < 1e-6
        assert oe[b] < 1e-6 and 1 <= info[b] <= 32
    assert torch.equal(lowp, Rn.to(torch.bfloat16))


def test_d4096_headline_tiles_against_oracle():
    """Cayley Adam on the tile path the benchmark's configuration takes (d = 4096: 256 x 256 tiles, three-term bf16
    products for the momentum products and the fixed point), against the oracle's exact solve."""
    d = 4096
    g = torch.Generator().manual_seed(d)
    R = ktgen.random_orthogonal(d, seed=2).unsqueeze(0)
    G = torch.randn((1, d, d), generator=g) / np.sqrt(d)
    M = 0.3 * torch.randn((1, d, d), generator=g) / np.sqrt(d)
    v = torch.tensor([0.8])
    k, lr = 3, 0.05
    Rn, Mn, vn, lowp, oe, info, sc = _gpu_step(R, G, M, v, k, lr)
    o = oracle.cayley_adam_step(ktgen.to_f64(R[0]), ktgen.to_f64(G[0]), ktgen.to_f64(M[0]), float(v[0]), k, F(lr), **HP)
    assert abs(vn[0].item() - o["v"]) <= 1e-6 * o["v"]
    for i, key in enumerate(("r", "alpha", "w_norm")):
        assert abs(sc[0, i] - o[key]) <= 1e-5 * o[key], key
    assert rel_fro(Rn[0].numpy().astype(np.float64) - ktgen.to_f64(R[0]), o["R"] - ktgen.to_f64(R[0])) <= 1e-4
    assert rel_fro(Mn[0].numpy().astype(np.float64), o["M"]) <= 1e-4
    RtR = Rn[0].double().T @ Rn[0].double()
    assert float((RtR - torch.eye(d, dtype=torch.float64)).abs().max()) < 1e-6
    assert oe[0] < 1e-6 and 1 <= info[0] <= 32
    assert torch.equal(lowp, Rn.to(torch.bfloat16))


def test_clamp_engages_for_a_huge_learning_rate():
    d = 128
    R = ktgen.random_orthogonal(d, seed=1).unsqueeze(0)
    G = torch.randn((1, d, d), generator=torch.Generator().manual_seed(2))
    Rn, Mn, vn, lowp, oe, info, sc = _gpu_step(R, G, torch.zeros(1, d, d), torch.ones(1), 1, 1e6)
    assert sc[0, 1] < 1e6 and abs(sc[0, 1] * sc[0, 2] - 1.0) < 1e-4       # alpha ||W|| = 2 q
    assert 1 <= info[0] <= 32 and oe[0] < 1e-6


def test_low_rank_step_at_the_clamp_needs_many_iterations():
    # a rank-one gradient makes ||W||_2 ~ ||W||_F / sqrt(2): with the clamp engaged the fixed point contracts
    # by ~0.35 per iteration, long enough to reach the single-launch form of the late iterations (d >= 1024)
    d = 1024
    g = torch.Generator().manual_seed(5)
    R = ktgen.random_orthogonal(d, seed=6).unsqueeze(0)
    u, w = torch.randn(d, generator=g), torch.randn(d, generator=g)
    G = (torch.outer(u, w) / d).unsqueeze(0)
    M, v = torch.zeros(1, d, d), torch.ones(1)
    Rn, Mn, vn, lowp, oe, info, sc = _gpu_step(R, G, M, v, 1, 1e3)
    o = oracle.cayley_adam_step(ktgen.to_f64(R[0]), ktgen.to_f64(G[0]), ktgen.to_f64(M[0]), 1.0, 1, F(1e3), **HP)
    assert abs(sc[0, 1] * sc[0, 2] - 1.0) < 1e-4 and 6 < info[0] <= 32
    step = o["R"] - ktgen.to_f64(R[0])
    assert rel_fro(Rn[0].numpy().astype(np.float64) - ktgen.to_f64(R[0]), step) <= 1e-4
    assert rel_fro(Mn[0].numpy().astype(np.float64), o["M"]) <= 1e-4
    assert oe[0] < 1e-6


def test_zero_gradient_and_momentum_leave_r_unchanged():
    d = 256
    R = ktgen.random_orthogonal(d, seed=3).unsqueeze(0)
    Rn, Mn, vn, lowp, oe, info, sc = _gpu_step(R, torch.zeros(1, d, d), torch.zeros(1, d, d), torch.ones(1), 4, 0.1)
    assert torch.equal(Rn, R) and float(Mn.abs().max()) == 0.0 and sc[0, 2] == 0.0
    assert abs(vn.item() - 0.99) < 1e-7


def test_teacher_forced_optimisation_descends():
    # 12 steps on a small outlier-channel problem; at each step the GPU starts from the oracle's state
    X, R, cfg = ktgen.make_problem("C1", seed=0, n=1024)
    d = R.shape[-1]
    Xd = X.cuda()
    Ro, Mo, vo = ktgen.to_f64(R[0]), np.zeros((d, d)), 1.0
    first = last = None
    for k in range(1, 13):
        lg = oracle.loss_grad(ktgen.to_f64(X[0]), Ro)
        first = lg["loss"] if first is None else first
        last = lg["loss"]
        Rd = torch.tensor(Ro, dtype=torch.float32).unsqueeze(0).cuda()
        dR = torch.empty((1, d, d), device="cuda")
        kt.kt_kurtosis_loss_grad(Xd, Rd, dR=dR)
        Md = torch.tensor(Mo, dtype=torch.float32).unsqueeze(0).cuda()
        vd = torch.tensor([vo], dtype=torch.float32).cuda()
        kt.kt_cayley_adam_step(Rd, dR, Md, vd, k, 0.05)
        torch.cuda.synchronize()
        o = oracle.cayley_adam_step(Ro, lg["dR"], Mo, vo, k, F(0.05), **HP)
        assert rel_fro(Rd[0].cpu().numpy().astype(np.float64) - Ro, o["R"] - Ro) <= 2e-4, k
        assert rel_fro(Md[0].cpu().numpy().astype(np.float64), o["M"]) <= 2e-4, k
        Ro, Mo, vo = o["R"], o["M"], o["v"]
    assert last < 0.97 * first
