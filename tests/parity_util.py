"""Helpers shared by the GPU parity tests (not a test module)."""
import numpy as np
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def gpu_loss_grad(X, R, kappa_target=0.0, want_dR=True, want_rows=True, ws=None):
    """X [b][n][d] / R [b][d][d] torch tensors (any device) -> dict of numpy results."""
    Xd, Rd = X.cuda(), R.cuda()
    if Xd.dim() == 2:
        Xd, Rd = Xd.unsqueeze(0), Rd.unsqueeze(0)
    b, n, d = Xd.shape
    rk = torch.full((b, n), float("nan"), device="cuda") if want_rows else None
    dR = torch.full((b, d, d), float("nan"), device="cuda") if want_dR else None
    loss = kt.kt_kurtosis_loss_grad(Xd, Rd, kappa_target=kappa_target, row_kurt=rk, dR=dR, workspace=ws)
    torch.cuda.synchronize()
    return {"loss": loss.cpu().numpy().astype(np.float64),
            "row_kurt": None if rk is None else rk.cpu().numpy(),
            "dR": None if dR is None else dR.cpu().numpy()}


def oracle_loss_grad(X, R, kappa_target=0.0, want_dR=True, r_as_bf16=None):
    """Oracle on the exact values the GPU GEMM sees: X widened to fp64, R rounded to bf16
    first when X is bf16 (the loss and gradient are those at the rounded R)."""
    if X.dim() == 2:
        X, R = X.unsqueeze(0), R.unsqueeze(0)
    if r_as_bf16 is None:
        r_as_bf16 = X.dtype == torch.bfloat16
    outs = []
    for b in range(X.shape[0]):
        Rb = ktgen.bf16_round(R[b]) if r_as_bf16 else R[b]
        outs.append(oracle.loss_grad(ktgen.to_f64(X[b]), ktgen.to_f64(Rb), kappa_target=kappa_target,
                                     want_dR=want_dR))
    return {"loss": np.array([o["loss"] for o in outs]),
            "row_kurt": np.stack([o["row_kurt"] for o in outs]),
            "dR": np.stack([o["dR"] for o in outs]) if want_dR else None}


def check_loss_grad(g, o, tol, want_dR=True):
    assert np.all(np.abs(g["loss"] - o["loss"]) <= tol * np.abs(o["loss"])), (g["loss"], o["loss"])
    if g["row_kurt"] is not None:
        ok = o["row_kurt"]
        assert np.all(np.abs(g["row_kurt"] - ok) <= tol * np.maximum(np.abs(ok), 1e-30)), \
            float(np.max(np.abs(g["row_kurt"] - ok) / np.maximum(np.abs(ok), 1e-30)))
    if want_dR:
        for b in range(o["dR"].shape[0]):
            r = rel_fro(g["dR"][b], o["dR"][b])
            assert r <= tol, r
