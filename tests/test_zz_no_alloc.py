"""kt_cayley_step_static (the entry point for callers that cannot allocate: the scratch is a static device
array inside the library) against kt_cayley_step on a caller's workspace: same kernels, so the same bits.
Two calls in a row on the shared array, the second with a smaller problem, then a batch; whatever the
earlier call left in the array must not reach the later results."""
import pytest
import torch

import ktgen
import paper_2503_01483_amd as kt

pytestmark = pytest.mark.gpu


def _both(d, batch, lr, seed):
    g = torch.Generator().manual_seed(seed)
    R = torch.stack([ktgen.random_orthogonal(d, seed=seed + b) for b in range(batch)]).cuda()
    G = (torch.randn((batch, d, d), generator=g) / d ** 0.5).cuda()
    out = []
    for fn in (kt.kt_cayley_step, kt.kt_cayley_step_static):
        Rw = R.clone()
        lowp = torch.zeros((batch, d, d), dtype=torch.bfloat16, device="cuda")
        oe = torch.full((batch,), float("nan"), device="cuda")
        info = torch.zeros(batch, dtype=torch.int32, device="cuda")
        print(f"{fn.__name__} d={d} batch={batch} lr={lr}", flush=True)
        fn(Rw, G, lr, R_lowp=lowp, ortho_err=oe, info=info)
        torch.cuda.synchronize()
        out.append((Rw.cpu(), lowp.cpu(), oe.cpu(), info.cpu()))
    return R.cpu(), out


def test_static_scratch_matches_the_workspace_form_on_consecutive_calls():
    before = torch.cuda.memory_allocated()
    for d, batch, lr, seed in ((512, 1, 0.05, 1), (256, 1, 0.02, 2), (256, 5, 0.1, 3), (128, 3, 0.05, 4), (384, 2, 0.01, 5)):
        R, (ws_form, static_form) = _both(d, batch, lr, seed)
        for a, b in zip(ws_form, static_form):
            assert torch.equal(a, b)
        Rn, _, oe, info = static_form
        assert float(oe.max()) < 1e-6 and int(info.min()) >= 1
        assert not torch.equal(Rn, R)
    assert torch.cuda.memory_allocated() == before      # nothing of the test's own leaked either


def test_too_large_for_the_static_scratch():
    R = torch.eye(1024, device="cuda").unsqueeze(0)
    with pytest.raises(kt.KtError) as e:
        kt.kt_cayley_step_static(R, torch.zeros_like(R), 0.01)
    assert e.value.status == 6
