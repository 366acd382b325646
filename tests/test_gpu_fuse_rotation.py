"""GPU parity of kt_fuse_rotation (fp32 MFMA GEMM) against the oracle: 1e-4 relative (Frobenius),
plus the computational-invariance identity on the device results."""
import numpy as np
import pytest
import torch

import ktgen
import oracle
import paper_2503_01483_amd as kt
from parity_util import rel_fro

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k,d,side", [(300, 128, 0), (300, 128, 1), (1000, 256, 0), (344, 512, 1), (2048, 1024, 0),
                                      (1100, 1024, 1)])
def test_against_oracle(k, d, side):
    g = torch.Generator().manual_seed(k + d + side)
    R = ktgen.random_orthogonal(d, seed=k)
    W = torch.randn((k, d) if side == 0 else (d, k), generator=g)
    out = kt.kt_fuse_rotation(W.cuda(), R.cuda(), side)
    torch.cuda.synchronize()
    ref = oracle.fuse_rotation(ktgen.to_f64(W), ktgen.to_f64(R), side)
    assert rel_fro(out.cpu().numpy(), ref) <= 1e-4


def test_fused_weights_keep_the_layer_output():
    d, k, n = 256, 640, 200
    g = torch.Generator().manual_seed(0)
    R = ktgen.random_orthogonal(d, seed=1).cuda()
    X = torch.randn((n, d), generator=g).cuda()
    Wup = torch.randn((d, k), generator=g).cuda()
    Wdown = torch.randn((k, d), generator=g).cuda()
    Wup_f = kt.kt_fuse_rotation(Wup, R, 1)
    Wdown_f = kt.kt_fuse_rotation(Wdown, R, 0)
    # a block x -> relu(x W_up) W_down fed the rotated stream returns the rotated output
    y = torch.relu(X.double() @ Wup.double()) @ Wdown.double()
    y_rot = torch.relu((X.double() @ R.double()) @ Wup_f.double()) @ Wdown_f.double()
    assert float((y_rot - y @ R.double()).abs().max()) < 1e-3 * float(y.abs().max())
