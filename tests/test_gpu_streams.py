"""Every entry point enqueues on the stream it is given and nowhere else: on a side stream (default
priority) the input is produced by a copy enqueued just before the call, with no synchronisation in
between, and the results must be bit for bit those of the same call on the default stream after a
full synchronisation.  Work that landed on another stream would read the input before the copy."""
import pytest
import torch

import ktgen
import paper_2503_01483_amd as kt

pytestmark = pytest.mark.gpu


def _both_ways(make_inputs, call):
    """call(inputs) -> tuple of output tensors.  Returns (default-stream outputs, side-stream outputs)."""
    src = make_inputs()
    torch.cuda.synchronize()
    ref = call([t.clone() for t in src])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    staged = [torch.zeros_like(t) for t in src]
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for dst, s in zip(staged, src):
            dst.copy_(s, non_blocking=True)
        got = call(staged)
    side.synchronize()
    torch.cuda.synchronize()
    return ref, got


def _same(ref, got):
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


@pytest.mark.parametrize("n,d,batch,dtype", [(3000, 512, 1, "bf16"), (2000, 128, 3, "bf16"), (1500, 256, 1, "f32")])
def test_step_entry_points(n, d, batch, dtype):
    def inputs():
        X = ktgen.make_x(n * batch, d, seed=1, outlier_cols=3, outlier_scale=30.0, dtype=dtype, device="cuda").reshape(batch, n, d)
        R = torch.stack([ktgen.random_orthogonal(d, seed=b, device="cuda") for b in range(batch)])
        return [X, R]

    def call(t):
        X, R = t
        ws = kt.Workspace()
        dR = torch.empty((batch, d, d), device="cuda")
        rk = torch.empty((batch, n), device="cuda")
        loss = kt.kt_kurtosis_loss_grad(X, R, row_kurt=rk, dR=dR, workspace=ws)
        dRp = torch.empty_like(dR)
        lp = torch.zeros(batch, device="cuda")
        kt.kt_pooled_kurtosis_loss_grad(X, R, loss=lp, dR=dRp, workspace=ws)
        R1, R2 = R.clone(), R.clone()
        low = torch.empty((batch, d, d), dtype=torch.bfloat16, device="cuda")
        kt.kt_cayley_step(R1, dR, 0.01, R_lowp=low, workspace=ws)
        M, v = torch.zeros_like(R), torch.zeros(batch, device="cuda")
        kt.kt_cayley_adam_step(R2, dR, M, v, 1, 0.05, workspace=ws)
        return loss, rk, dR, lp, dRp, R1, low, R2, M, v

    _same(*_both_ways(inputs, call))


@pytest.mark.parametrize("n,d,batch,dtype", [(5000, 512, 1, "bf16"), (2000, 128, 2, "bf16"), (900, 256, 1, "f32")])
def test_evaluation_entry_points(n, d, batch, dtype):
    def inputs():
        X = ktgen.make_x(n * batch, d, seed=2, outlier_cols=3, outlier_scale=30.0, dtype=dtype, device="cuda").reshape(batch, n, d)
        R = torch.stack([ktgen.random_orthogonal(d, seed=5 + b, device="cuda") for b in range(batch)])
        return [X, R]

    def call(t):
        X, R = t
        ws = kt.Workspace()
        so = torch.empty((batch, n), device="cuda")
        codes = torch.empty((batch, n, d), dtype=torch.int8, device="cuda")
        err = torch.empty((batch, n, 2), device="cuda")
        kt.kt_rotate_fakequant_int4(X, R, scales_out=so, codes=codes, err=err, workspace=ws)
        codes2 = torch.empty_like(codes)
        kt.kt_rotate_fakequant_int4(X, R, scales_in=so, codes=codes2, workspace=ws)
        Y = torch.empty((batch, n, d), device="cuda")
        thr = torch.empty((batch, n), device="cuda")
        es = torch.empty((batch, n, 2), device="cuda")
        succ = torch.zeros(batch, dtype=torch.int64, device="cuda")
        kt.kt_rotate_quant_metrics(X, R, quantile=0.98, Y=Y, threshold=thr, err_sym=es, success=succ, workspace=ws)
        alphas = torch.tensor([-0.5, 0.0, 0.5], device="cuda")
        out, gamma = kt.kt_quant_sensitivity(Y[0].contiguous(), alphas, workspace=ws)
        H = kt.kt_hadamard_rows(X[0], signs=None)
        W = kt.kt_fuse_rotation(Y[0, :64].contiguous(), R[0], 0, workspace=ws)
        return so, codes, err, codes2, Y, thr, es, succ, out, gamma, H, W

    _same(*_both_ways(inputs, call))
