"""GPU parity at the benchmark's full size (C3: d = 4096, n = 131072, bf16), in the launch
configuration bench.py times.  The oracle cannot do the whole problem, so: per-row kurtosis on
sampled rows and loss/gradient on a 1024-row chunk are compared with the oracle directly, and
the full result is tied to them by properties that hold at any size (invariants of the gradient,
the loss as the mean of the row values, additivity over row chunks)."""
import numpy as np
import pytest
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt
from parity_util import rel_fro

pytestmark = pytest.mark.gpu


def test_c3_full_size():
    X, R, cfg = ktgen.make_problem("C3", seed=0, device="cuda")
    b, n, d = X.shape
    assert (n, d) == (131072, 4096)
    ws = kt.Workspace()
    rk = torch.empty((1, n), device="cuda")
    dR = torch.empty((1, d, d), device="cuda")
    loss = kt.kt_kurtosis_loss_grad(X, R, row_kurt=rk, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    rk_h = rk[0].cpu().numpy().astype(np.float64)
    dR_h = dR[0].cpu().numpy().astype(np.float64)
    Rb = ktgen.to_f64(ktgen.bf16_round(R[0]))

    # loss is the mean of the per-row values
    assert abs(loss.item() - rk_h.mean()) <= 1e-5 * rk_h.mean()
    # sampled rows against the oracle, one by one
    rows = np.random.default_rng(0).choice(n, size=96, replace=False)
    o = oracle.loss_grad(ktgen.to_f64(X[0, torch.as_tensor(rows, device="cuda")]), Rb, want_dR=False)
    assert np.max(np.abs(rk_h[rows] - o["row_kurt"]) / o["row_kurt"]) <= 2e-2
    # invariants of the gradient (shift / scale invariance of kurtosis), no oracle needed
    nrm = np.linalg.norm(dR_h)
    assert np.linalg.norm(dR_h.sum(1)) <= 1e-3 * nrm * np.sqrt(d)
    assert abs((dR_h * Rb).sum()) <= 1e-3 * nrm * np.linalg.norm(Rb)

    # a chunk the oracle can do, at the real d
    m = 1024
    l2 = torch.empty(1, device="cuda")
    d2 = torch.empty((1, d, d), device="cuda")
    kt.kt_kurtosis_loss_grad(X[:, :m], R, loss=l2, dR=d2, workspace=ws)
    torch.cuda.synchronize()
    oc = oracle.loss_grad(ktgen.to_f64(X[0, :m]), Rb)
    assert abs(l2.item() - oc["loss"]) <= 2e-2 * oc["loss"]
    assert rel_fro(d2[0].cpu().numpy(), oc["dR"]) <= 2e-2

    # additivity over four row chunks ties the full gradient to chunk results
    acc = np.zeros((d, d))
    q = n // 4
    for c in range(4):
        kt.kt_kurtosis_loss_grad(X[:, c * q:(c + 1) * q], R, loss=l2, dR=d2, workspace=ws)
        torch.cuda.synchronize()
        acc += q * d2[0].cpu().numpy().astype(np.float64)
    assert rel_fro(n * dR_h, acc) <= 5e-3


def test_c3_full_size_step_is_orthogonal_and_descends():
    X, R, cfg = ktgen.make_problem("C3", seed=0, device="cuda", n=32768)
    d = cfg["d"]
    ws = kt.Workspace()
    dR = torch.empty((1, d, d), device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    oe = torch.zeros(1, device="cuda")
    Rw = R.clone()
    l0 = kt.kt_kurtosis_loss_grad(X, Rw, dR=dR, workspace=ws).item()
    kt.kt_cayley_step(Rw, dR, 1e-2, ortho_err=oe, info=info, workspace=ws)
    l1 = kt.kt_kurtosis_loss_grad(X, Rw, workspace=ws).item()
    torch.cuda.synchronize()
    assert 1 <= info.item() <= 32 and oe.item() < 1e-6
    RtR = Rw[0].double().T @ Rw[0].double()
    assert float((RtR - torch.eye(d, dtype=torch.float64, device="cuda")).abs().max()) < 1e-6
    assert l1 < l0


def test_c4_full_size_sampled_problems():
    """C4 (256 head-dimension problems, d = 128, n = 131072 each) in the launch configuration
    bench.py times: one workgroup walks all 1024 token tiles of a problem.  At d = 128 the
    oracle can do whole problems, so sampled problems are compared in full."""
    X, R, cfg = ktgen.make_problem("C4", seed=0, device="cuda")
    b, n, d = X.shape
    assert (b, n, d) == (256, 131072, 128)
    ws = kt.Workspace()
    rk = torch.empty((b, n), device="cuda")
    dR = torch.empty((b, d, d), device="cuda")
    loss = torch.empty(b, device="cuda")
    kt.kt_kurtosis_loss_grad(X, R, loss=loss, row_kurt=rk, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    for p in (0, 101, 255):
        o = oracle.loss_grad(ktgen.to_f64(X[p]), ktgen.to_f64(ktgen.bf16_round(R[p])))
        assert abs(loss[p].item() - o["loss"]) <= 2e-2 * o["loss"], p
        assert np.max(np.abs(rk[p].cpu().numpy() - o["row_kurt"]) / o["row_kurt"]) <= 2e-2, p
        assert rel_fro(dR[p].cpu().numpy(), o["dR"]) <= 2e-2, p
    # every problem: loss is the mean of its row values
    means = rk.double().mean(1)
    assert float(((loss.double() - means).abs() / means).max()) <= 1e-5


@pytest.mark.parametrize("name,rows_checked,chunk", [("C2", 128, 2048), ("C5", 48, 256)])
def test_c2_c5_full_size(name, rows_checked, chunk):
    """C2 (d = 2048, n = 65536) and C5 (d = 8192, n = 1048576: 16 GiB of X, 4096-token blocks of the
    token-minor copies, split-K) in the launch configuration bench.py times: sampled rows and a row
    chunk against the oracle, the gradient invariants, and additivity over two halves."""
    X, R, cfg = ktgen.make_problem(name, seed=0, device="cuda")
    b, n, d = X.shape
    ws = kt.Workspace()
    rk = torch.empty((1, n), device="cuda")
    dR = torch.empty((1, d, d), device="cuda")
    loss = kt.kt_kurtosis_loss_grad(X, R, row_kurt=rk, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    rk_h = rk[0].cpu().numpy().astype(np.float64)
    Rb = ktgen.to_f64(ktgen.bf16_round(R[0]))
    assert abs(loss.item() - rk_h.mean()) <= 1e-5 * rk_h.mean()
    rows = np.random.default_rng(1).choice(n, size=rows_checked, replace=False)
    o = oracle.loss_grad(ktgen.to_f64(X[0, torch.as_tensor(rows, device="cuda")]), Rb, want_dR=False)
    assert np.max(np.abs(rk_h[rows] - o["row_kurt"]) / o["row_kurt"]) <= 2e-2
    dR_d = dR[0].double()
    nrm = float(dR_d.norm())
    assert float(dR_d.sum(1).norm()) <= 1e-3 * nrm * np.sqrt(d)
    assert abs(float((dR_d * torch.as_tensor(Rb, device="cuda")).sum())) <= 1e-3 * nrm * np.linalg.norm(Rb)
    # a chunk the oracle can do at the real d
    l2 = torch.empty(1, device="cuda")
    d2 = torch.empty((1, d, d), device="cuda")
    kt.kt_kurtosis_loss_grad(X[:, :chunk], R, loss=l2, dR=d2, workspace=ws)
    torch.cuda.synchronize()
    oc = oracle.loss_grad(ktgen.to_f64(X[0, :chunk]), Rb)
    assert abs(l2.item() - oc["loss"]) <= 2e-2 * oc["loss"]
    assert rel_fro(d2[0].cpu().numpy(), oc["dR"]) <= 2e-2
    # additivity over two halves ties the full gradient to the halves
    acc = torch.zeros((d, d), dtype=torch.float64, device="cuda")
    h = n // 2
    for c in range(2):
        kt.kt_kurtosis_loss_grad(X[:, c * h:(c + 1) * h], R, loss=l2, dR=d2, workspace=ws)
        acc += h * d2[0].double()
    torch.cuda.synchronize()
    assert float((n * dR_d - acc).norm()) <= 5e-3 * float(acc.norm())


def test_c5_size_cayley_step_against_a_double_precision_solve():
    """SECONDARY check (not against the oracle): d = 8192 (the C5 rotation) is too large for the CPU oracle's
    plain LU in test time, so the step is compared with the same formula evaluated by the framework's fp64
    solver on the device (R+ = (I + lr/2 A)^-1 (I - lr/2 A) R, A = G R^T - R G^T), a library routine that is
    independent of the HIP path.  The comparison with the oracle itself, on the same tile path (256 x 256,
    three-term products), is test_gpu_cayley.py::test_d4096_headline_tiles_against_oracle."""
    d, lr = 8192, 1e-2
    R = ktgen.random_orthogonal(d, seed=2, device="cuda").unsqueeze(0).contiguous()
    g = torch.Generator(device="cuda").manual_seed(3)
    G = torch.randn((1, d, d), generator=g, device="cuda") / np.sqrt(d)
    Rn = R.clone()
    oe = torch.zeros(1, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    kt.kt_cayley_step(Rn, G, lr, ortho_err=oe, info=info)
    torch.cuda.synchronize()
    Rd, Gd = R[0].double(), G[0].double()
    A = Gd @ Rd.T - Rd @ Gd.T
    I = torch.eye(d, dtype=torch.float64, device="cuda")
    ref = torch.linalg.solve(I + 0.5 * lr * A, (I - 0.5 * lr * A) @ Rd)
    step = ref - Rd
    assert float((Rn[0].double() - Rd - step).norm() / step.norm()) <= 1e-4
    assert 1 <= info.item() <= 32 and oe.item() < 1e-6
    assert float((Rn[0].double().T @ Rn[0].double() - I).abs().max()) < 1e-6


def test_c3_full_size_pooled_loss():
    """The paper-literal pooled loss at C3 size.  The comparison with the ORACLE is the 512-row chunk at the end
    (at the real d).  SECONDARY to it, because the CPU oracle cannot rotate 131072 x 4096 in test time: the
    pooled kurtosis of the definition evaluated in fp64 by the framework's matmul on the device (an independent
    library routine on the same bf16 values), and the invariants the RMSNorm forces on the gradient (every row
    of dL/dY is orthogonal to y, so <dR, R> = 0)."""
    X, R, cfg = ktgen.make_problem("C3", seed=0, device="cuda")
    b, n, d = X.shape
    ws = kt.Workspace()
    kap = torch.zeros(1, device="cuda")
    dR = torch.empty((1, d, d), device="cuda")
    loss = kt.kt_pooled_kurtosis_loss_grad(X, R, kappa=kap, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    Rb = R[0].to(torch.bfloat16).double()
    s1 = torch.zeros((), dtype=torch.float64, device="cuda")
    parts = []
    for c in range(0, n, 16384):                      # fp64 definition, chunked to bound memory
        Y = X[0, c:c + 16384].double() @ Rb
        Z = Y / (Y * Y).mean(1, keepdim=True).sqrt()
        parts.append(torch.stack([Z.sum(), (Z ** 2).sum(), (Z ** 3).sum(), (Z ** 4).sum()]))
    T = torch.stack(parts).sum(0) / (n * d)
    mu, r2, r3, r4 = [float(v) for v in T]
    m2 = r2 - mu * mu
    m4 = r4 - 4 * mu * r3 + 6 * mu * mu * r2 - 3 * mu ** 4
    kappa_ref = m4 / (m2 * m2)
    assert abs(kap.item() - kappa_ref) <= 2e-2 * kappa_ref
    assert abs(loss.item() - abs(kappa_ref - 1.8)) <= 2e-2 * kappa_ref
    dR_d = dR[0].double()
    assert abs(float((dR_d * Rb).sum())) <= 1e-3 * float(dR_d.norm()) * float(Rb.norm())
    # a chunk the oracle can do, at the real d
    m = 512
    l2 = torch.empty(1, device="cuda")
    d2 = torch.empty((1, d, d), device="cuda")
    kt.kt_pooled_kurtosis_loss_grad(X[:, :m], R, loss=l2, dR=d2, workspace=ws)
    torch.cuda.synchronize()
    oc = oracle.pooled_loss_grad(ktgen.to_f64(X[0, :m]), ktgen.to_f64(ktgen.bf16_round(R[0])))
    assert abs(l2.item() - oc["loss"]) <= 2e-2 * oc["kappa"]
    assert rel_fro(d2[0].cpu().numpy(), oc["dR"]) <= 2e-2


# ---- the largest sizes the boundary accepts ---------------------------------------------------------
@pytest.mark.parametrize("d,dtype", [(128, "bf16"), (128, "f32"), (256, "bf16")])
def test_maximum_token_count(d, dtype):
    """n = 2^22 tokens of one problem (d = 128 bf16: the single-pass kernel; fp32 and d = 256: the
    three-GEMM path with 1024 token blocks of the token-minor copies).  Sampled rows (the first, the
    last, random ones) against the oracle, the loss as the mean of the row values, the gradient
    invariants, and additivity over four quarters; n + 1 is refused."""
    n = 1 << 22
    X = ktgen.make_x(n, d, seed=d, outlier_cols=3, outlier_scale=30.0, t_frac=0.01, dtype=dtype,
                     device="cuda", chunk_rows=1 << 18).unsqueeze(0)
    R = ktgen.random_orthogonal(d, seed=5, device="cuda").unsqueeze(0)
    ws = kt.Workspace()
    rk = torch.empty((1, n), device="cuda")
    dR = torch.empty((1, d, d), device="cuda")
    loss = kt.kt_kurtosis_loss_grad(X, R, row_kurt=rk, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    tol = 2e-2 if dtype == "bf16" else 1e-4
    rk_d = rk[0].double()
    assert abs(loss.item() - float(rk_d.mean())) <= 1e-5 * float(rk_d.mean())
    rows = np.concatenate([np.arange(40), np.arange(n - 40, n),
                           np.random.default_rng(2).choice(n, size=60, replace=False)])
    Ro = ktgen.to_f64(ktgen.bf16_round(R[0]) if dtype == "bf16" else R[0])
    o = oracle.loss_grad(ktgen.to_f64(X[0, torch.as_tensor(rows, device="cuda")]), Ro, want_dR=False)
    assert np.max(np.abs(rk_d[torch.as_tensor(rows, device="cuda")].cpu().numpy() - o["row_kurt"]) / o["row_kurt"]) <= tol
    dR_d = dR[0].double()
    nrm = float(dR_d.norm())
    assert float(dR_d.sum(1).norm()) <= 1e-3 * nrm * np.sqrt(d)
    assert abs(float((dR_d * torch.as_tensor(Ro, device="cuda")).sum())) <= 1e-3 * nrm * np.linalg.norm(Ro)
    acc = torch.zeros((d, d), dtype=torch.float64, device="cuda")
    l2 = torch.empty(1, device="cuda")
    d2 = torch.empty((1, d, d), device="cuda")
    q = n // 4
    for c in range(4):
        kt.kt_kurtosis_loss_grad(X[:, c * q:(c + 1) * q], R, loss=l2, dR=d2, workspace=ws)
        acc += q * d2[0].double()
    torch.cuda.synchronize()
    assert float((n * dR_d - acc).norm()) <= (5e-3 if dtype == "bf16" else 1e-4) * float(acc.norm())
    with pytest.raises(Exception):
        kt.kt_kurtosis_loss_grad(torch.empty((1, n + 1, d), dtype=X.dtype, device="cuda"), R, workspace=ws)


def test_maximum_hidden_size():
    """d = 16384, the largest hidden size the boundary accepts: loss and gradient of a few token rows
    against the oracle at that d, and a Cayley step against the framework's fp64 solve (a SECONDARY check, as
    for d = 8192 above: the oracle's LU is out of reach at this size); d = 16384 + 128 is refused."""
    d, n, lr = 16384, 16, 1e-2
    g = torch.Generator(device="cuda").manual_seed(11)
    q, r = torch.linalg.qr(torch.randn((d, d), generator=g, device="cuda"))
    R = (q * torch.sign(torch.diagonal(r)).unsqueeze(0)).contiguous().unsqueeze(0)
    del q, r
    X = ktgen.make_x(n, d, seed=3, outlier_cols=16, outlier_scale=50.0, t_frac=0.02, dtype="bf16", device="cuda").unsqueeze(0)
    ws = kt.Workspace()
    rk = torch.empty((1, n), device="cuda")
    dR = torch.empty((1, d, d), device="cuda")
    loss = kt.kt_kurtosis_loss_grad(X, R, row_kurt=rk, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    o = oracle.loss_grad(ktgen.to_f64(X[0]), ktgen.to_f64(ktgen.bf16_round(R[0])))
    assert abs(loss.item() - o["loss"]) <= 2e-2 * o["loss"]
    assert np.max(np.abs(rk[0].cpu().numpy() - o["row_kurt"]) / o["row_kurt"]) <= 2e-2
    assert rel_fro(dR[0].cpu().numpy(), o["dR"]) <= 2e-2
    del o
    Rn = R.clone()
    oe = torch.zeros(1, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    G = torch.randn((1, d, d), generator=g, device="cuda") / np.sqrt(d)   # as in the d = 8192 test above
    kt.kt_cayley_step(Rn, G, lr, ortho_err=oe, info=info, workspace=ws)
    torch.cuda.synchronize()
    Rd, Gd = R[0].double(), G[0].double()
    A = Gd @ Rd.T - Rd @ Gd.T
    I = torch.eye(d, dtype=torch.float64, device="cuda")
    ref = torch.linalg.solve(I + 0.5 * lr * A, (I - 0.5 * lr * A) @ Rd)
    step = ref - Rd
    # the fixed point stops at an ABSOLUTE change per entry (3e-7, the scale of the orthogonality bound);
    # the entries of a step shrink like 1/sqrt(d), so relative to the step that is ~1e-4 at this size
    assert float((Rn[0].double() - Rd - step).norm() / step.norm()) <= 3e-4
    assert 1 <= info.item() <= 32 and oe.item() < 1e-6
    del A, ref, step
    with pytest.raises(Exception):
        kt.kt_kurtosis_loss_grad(torch.zeros((1, 4, d + 128), dtype=torch.bfloat16, device="cuda"),
                                 torch.zeros((1, d + 128, d + 128), device="cuda"))


def test_maximum_problem_count():
    """batch = 65535 independent d = 128 problems of 64 tokens (the largest grid the batched kernels are
    launched with): loss, gradient and Cayley step of the first, a middle and the last problem against
    the oracle; batch + 1 is refused."""
    batch, n, d, lr = 65535, 64, 128, 1e-2
    X = ktgen.make_x(batch * n, d, seed=9, base="t4", outlier_cols=2, outlier_scale=8.0, dtype="bf16",
                     device="cuda", chunk_rows=1 << 18).reshape(batch, n, d)
    R1 = torch.stack([ktgen.random_orthogonal(d, seed=s) for s in range(3)]).cuda()
    R = R1[torch.arange(batch, device="cuda") % 3].contiguous()
    ws = kt.Workspace()
    dR = torch.empty((batch, d, d), device="cuda")
    rk = torch.empty((batch, n), device="cuda")
    loss = kt.kt_kurtosis_loss_grad(X, R, row_kurt=rk, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    picked = (0, 32767, batch - 1)
    G = torch.randn((batch, d, d), generator=torch.Generator(device="cuda").manual_seed(5), device="cuda") * 1e-3
    for p in picked:
        Ro = ktgen.to_f64(ktgen.bf16_round(R[p]))
        o = oracle.loss_grad(ktgen.to_f64(X[p]), Ro)
        assert abs(loss[p].item() - o["loss"]) <= 2e-2 * o["loss"], p
        assert np.max(np.abs(rk[p].cpu().numpy() - o["row_kurt"]) / o["row_kurt"]) <= 2e-2, p
        assert rel_fro(dR[p].cpu().numpy(), o["dR"]) <= 2e-2, p
        G[p] = torch.tensor(o["dR"], dtype=torch.float32).cuda()     # the oracle's gradient where it is checked
    Rn = R.clone()
    oe = torch.zeros(batch, device="cuda")
    info = torch.zeros(batch, dtype=torch.int32, device="cuda")
    kt.kt_cayley_step(Rn, G, lr, ortho_err=oe, info=info, workspace=ws)
    torch.cuda.synchronize()
    assert float(oe.max()) < 1e-6 and int(info.min()) >= 1
    for p in picked:
        ref = oracle.cayley_step(ktgen.to_f64(R[p]), ktgen.to_f64(G[p]), lr)
        stepn = np.linalg.norm(ref - ktgen.to_f64(R[p]))
        assert np.linalg.norm(Rn[p].cpu().double().numpy() - ref) <= 1e-3 * stepn, p
    with pytest.raises(Exception):
        kt.kt_cayley_step(torch.empty((batch + 1, d, d), device="cuda"), torch.empty((batch + 1, d, d), device="cuda"), lr)
