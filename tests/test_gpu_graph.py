"""The library launches only kernels (no memset nodes, no allocation, no host sync), so a caller may
capture a whole step into a HIP graph.  Every replay must reproduce the eager result bit for bit,
also with eager work and synchronisations between the replays."""
import pytest
import torch

import ktgen
import paper_2503_01483_amd as kt

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,n,batch,adam", [("C1", 1024, 1, False), ("C2", 2048, 1, True), ("C4", 3000, 5, False),
                                                ("C4", 1500, 3, True)])
def test_captured_step_replays_like_the_eager_step(name, n, batch, adam):
    X, R, cfg = ktgen.make_problem(name, seed=1, device="cuda", n=n, batch=batch)
    b, n, d = X.shape
    bf16 = cfg["dtype"] == "bf16"
    need = max(kt.kt_workspace_bytes(kt.KT_OP_LOSS_GRAD, b, n, d, kt.KT_BF16 if bf16 else kt.KT_F32),
               kt.kt_workspace_bytes(kt.KT_OP_CAYLEY, b, 0, d, kt.KT_F32))

    def state():
        ws = kt.Workspace("cuda")
        ws.get(need)
        return dict(R=R.clone(), dR=torch.empty((b, d, d), device="cuda"), loss=torch.zeros(b, device="cuda"),
                    M=torch.zeros((b, d, d), device="cuda"), v=torch.ones(b, device="cuda"), ws=ws)

    def step(s, k):
        kt.kt_kurtosis_loss_grad(X, s["R"], loss=s["loss"], dR=s["dR"], workspace=s["ws"])
        if adam:   # the step counter is a host scalar baked into the captured launch: replay the same k
            kt.kt_cayley_adam_step(s["R"], s["dR"], s["M"], s["v"], k, 0.01, workspace=s["ws"])
        else:
            kt.kt_cayley_step(s["R"], s["dR"], 0.01, workspace=s["ws"])

    eager, cap = state(), state()
    step(eager, 1)
    step(cap, 1)                       # warm-up outside the capture (function attributes are set here)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step(cap, 2)
    torch.cuda.synchronize()
    # the capture itself executed nothing: cap is still at the state after one step
    assert torch.equal(cap["R"], eager["R"])
    for _ in range(3):
        g.replay()
        step(eager, 2)
        torch.cuda.synchronize()
        assert torch.equal(cap["R"], eager["R"]) and torch.equal(cap["loss"], eager["loss"])
        if adam:
            assert torch.equal(cap["M"], eager["M"]) and torch.equal(cap["v"], eager["v"])
        _ = (X[:, :64].float() ** 2).sum().item()    # unrelated eager work and a sync between replays


@pytest.mark.parametrize("n,d,batch", [(3000, 512, 1), (2500, 128, 3)])
def test_captured_evaluation_calls_replay_like_eager_ones(n, d, batch):
    """Fake-quant (scales computed in the call, and handed in), quantisation figures and the Hadamard rows in
    one captured graph; the inputs change between replays, every replay must match the eager calls."""
    X = ktgen.make_x(n * batch, d, seed=4, outlier_cols=3, outlier_scale=30.0, dtype="bf16", device="cuda").reshape(batch, n, d)
    R = torch.stack([ktgen.random_orthogonal(d, seed=30 + b, device="cuda") for b in range(batch)])

    def state():
        return dict(ws=kt.Workspace("cuda"), so=torch.zeros((batch, n), device="cuda"),
                    codes=torch.zeros((batch, n, d), dtype=torch.int8, device="cuda"), err=torch.zeros((batch, n, 2), device="cuda"),
                    codes2=torch.zeros((batch, n, d), dtype=torch.int8, device="cuda"), thr=torch.zeros((batch, n), device="cuda"),
                    es=torch.zeros((batch, n, 2), device="cuda"), succ=torch.zeros(batch, dtype=torch.int64, device="cuda"),
                    H=torch.zeros((n, d), dtype=torch.bfloat16, device="cuda"))

    def calls(s, Xin):
        kt.kt_rotate_fakequant_int4(Xin, R, scales_out=s["so"], codes=s["codes"], err=s["err"], workspace=s["ws"])
        kt.kt_rotate_fakequant_int4(Xin, R, scales_in=s["so"], codes=s["codes2"], workspace=s["ws"])
        kt.kt_rotate_quant_metrics(Xin, R, quantile=0.98, threshold=s["thr"], err_sym=s["es"], success=s["succ"], workspace=s["ws"])
        kt.kt_hadamard_rows(Xin[0], out=s["H"])

    eager, cap = state(), state()
    Xc = X.clone()
    calls(eager, Xc)
    calls(cap, Xc)                     # warm-up outside the capture (function attributes, workspace size)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            calls(cap, Xc)
    torch.cuda.synchronize()
    for rep in range(3):
        Xc.copy_(torch.roll(X, rep + 1, dims=1))     # new input in the captured buffer
        torch.cuda.synchronize()
        g.replay()
        calls(eager, Xc)
        torch.cuda.synchronize()
        for k in ("so", "codes", "err", "codes2", "thr", "es", "succ", "H"):
            assert torch.equal(cap[k], eager[k]), (rep, k)
        _ = (X[:, :64].float() ** 2).sum().item()    # unrelated eager work and a sync between replays
