"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol the
header declares, sizes its workspace sensibly and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2503_01483_amd as kt
from paper_2503_01483_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "kt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kt_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    L = kt.lib()
    for name in names:
        assert getattr(L, name) is not None


def test_version_and_error_text():
    assert kt.kt_version() >= 100
    assert isinstance(kt.kt_last_error(), str)


def test_workspace_bytes():
    f = kt.kt_workspace_bytes
    assert f(kt.KT_OP_LOSS_GRAD, 1, 2048, 256, kt.KT_F32) > 2 * 2048 * 256 * 4
    small = f(kt.KT_OP_LOSS_GRAD_RECOMPUTE, 1, 131072, 4096, kt.KT_BF16)
    assert 2**30 < small < 1.25 * 2**30         # the token-minor dL/dY dominates (X is read in place)
    big = f(kt.KT_OP_LOSS_GRAD, 1, 131072, 4096, kt.KT_BF16)
    assert big - small == 131072 * 4096 * 4     # plus Y kept in fp32
    assert f(kt.KT_OP_POOLED_LOSS_GRAD, 1, 4096, 512, kt.KT_BF16) - \
        f(kt.KT_OP_POOLED_LOSS_GRAD_RECOMPUTE, 1, 4096, 512, kt.KT_BF16) == 4096 * 512 * 4
    assert f(kt.KT_OP_LOSS_GRAD, 1, 100, 100, kt.KT_BF16) == 0   # d not a multiple of 128
    assert f(kt.KT_OP_LOSS_GRAD, 0, 100, 128, kt.KT_BF16) == 0
    assert f(kt.KT_OP_CAYLEY, 1, 0, 4096, kt.KT_F32) >= 5 * 4096 * 4096 * 4
    assert f(kt.KT_OP_FAKEQUANT, 2, 1000, 128, kt.KT_BF16) > 0
    assert f(99, 1, 10, 128, kt.KT_BF16) == 0
    # monotone in n
    assert f(kt.KT_OP_LOSS_GRAD, 1, 4096, 256, kt.KT_BF16) > f(kt.KT_OP_LOSS_GRAD, 1, 1024, 256, kt.KT_BF16)


def test_argument_errors_are_synchronous():
    L = kt.lib()
    fake = ctypes.c_void_p(4096)  # never dereferenced: every call below fails its checks first
    ws = ctypes.c_void_p(1 << 20)
    st = L.kt_kurtosis_loss_grad(None, 128, fake, 128, 1, 16, 128, 1, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 1 and "null" in kt.kt_last_error()
    st = L.kt_kurtosis_loss_grad(fake, 100, fake, 100, 1, 16, 100, 1, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 2 and "multiple of 128" in kt.kt_last_error()
    st = L.kt_kurtosis_loss_grad(fake, 132, fake, 128, 1, 16, 128, 1, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 2 and "ldx" in kt.kt_last_error()
    st = L.kt_kurtosis_loss_grad(fake, 128, fake, 128, 1, 16, 128, 0, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 3
    st = L.kt_kurtosis_loss_grad(fake, 128, fake, 128, 1, 16, 128, 7, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 3
    st = L.kt_kurtosis_loss_grad(fake, 128, fake, 128, 1, 16, 128, 1, 1, 0.0, fake, None, None, ws, 16, None)
    assert st == 4 and "workspace" in kt.kt_last_error()
    st = L.kt_kurtosis_loss_grad(fake, 128, fake, 128, 1, 16, 128, 1, 1, -1.0, fake, None, None, ws, 1 << 30, None)
    assert st == 1
    st = L.kt_cayley_step(None, fake, None, 1, 128, 0.01, None, None, ws, 1 << 30, None)
    assert st == 1
    st = L.kt_cayley_step(fake, fake, None, 1, 64, 0.01, None, None, ws, 1 << 30, None)
    assert st == 2
    st = L.kt_cayley_adam_step(fake, fake, None, fake, 1, None, 1, 128, 0.01, 0.9, 0.99, 1e-8, 0.5, None, None, None,
                               ws, 1 << 30, None)
    assert st == 1 and "null" in kt.kt_last_error()
    st = L.kt_cayley_adam_step(fake, fake, fake, fake, 0, None, 1, 128, 0.01, 0.9, 0.99, 1e-8, 0.5, None, None, None,
                               ws, 1 << 30, None)
    assert st == 1 and "step" in kt.kt_last_error()
    st = L.kt_cayley_adam_step(fake, fake, fake, fake, 1, None, 1, 128, 0.01, 1.0, 0.99, 1e-8, 0.5, None, None, None,
                               ws, 1 << 30, None)
    assert st == 1 and "beta" in kt.kt_last_error()
    st = L.kt_cayley_step(fake, fake, None, 1, 128, float("nan"), None, None, ws, 1 << 30, None)
    assert st == 1
    st = L.kt_rotate_fakequant_int4(fake, 128, fake, 128, 1, 16, 128, 1, 1, 1.5, None, fake, None, None, ws, 1 << 30, None)
    assert st == 1 and "clip" in kt.kt_last_error()
    st = L.kt_rotate_fakequant_int4(fake, 128, fake, 128, 1, 16, 128, 1, 1, 1.0, None, None, None, None, ws, 1 << 30, None)
    assert st == 1
    st = L.kt_rotate_fakequant_int4(fake, 128, fake, 128, 1, 16, 128, 1, 1, 1.0, None, None, ctypes.c_void_p(0x1004), None,
                                    ws, 1 << 30, None)
    assert st == 2 and "16-byte" in kt.kt_last_error()
    # sizes beyond the documented limits
    st = L.kt_kurtosis_loss_grad(fake, 16512, fake, 16512, 1, 16, 16512, 1, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 2 and "16384" in kt.kt_last_error()
    st = L.kt_kurtosis_loss_grad(fake, (1 << 22) + 8, fake, 128, 1, 16, 128, 1, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 2 and "2^22" in kt.kt_last_error()
    st = L.kt_kurtosis_loss_grad(fake, 128, fake, 128, 1, (1 << 22) + 1, 128, 1, 1, 0.0, fake, None, None, ws, 1 << 30, None)
    assert st == 2
    # a good call clears the text only when it runs; bad ones leave their own message
    assert kt.kt_last_error() != ""


def test_binding_has_no_fallback():
    src = open(os.path.join(ROOT, "paper_2503_01483_amd", "binding.py")).read()
    assert "oracle" not in src


def test_argument_errors_of_the_widened_entry_points():
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every call below must fail before any launch
    ws = ctypes.c_void_p(0x100000)
    big = 1 << 40
    st = L.kt_rotate_quant_metrics(fake, 128, fake, 128, 1, 16, 128, 1, 1, 1.5, None, None, None, None, None, None,
                                   ws, big, None)
    assert st == 1 and "quantile" in kt.kt_last_error()
    st = L.kt_rotate_quant_metrics(fake, 16384, fake, 16384, 1, 16, 16384, 1, 1, 0.98, None, None, None, None, None,
                                   None, ws, big, None)
    assert st == 6 and "8192" in kt.kt_last_error()
    st = L.kt_hadamard_rows(fake, 96, fake, 96, None, 4, 96, 0, None)
    assert st == 2 and "power of two" in kt.kt_last_error()
    st = L.kt_hadamard_rows(fake, 130, fake, 128, None, 4, 128, 0, None)
    assert st == 2 and "aligned" in kt.kt_last_error()
    st = L.kt_fuse_rotation(fake, 128, fake, 128, fake, 128, 64, 128, 2, ws, big, None)
    assert st == 1 and "side" in kt.kt_last_error()
    st = L.kt_fuse_rotation(fake, 128, fake, 128, fake, 128, 64, 100, 0, ws, big, None)
    assert st == 2
    st = L.kt_quant_sensitivity(fake, 100, 1, None, 0, fake, None, ws, big, None)
    assert st == 1 and "bits" in kt.kt_last_error()
    st = L.kt_quant_sensitivity(fake, 100, 4, None, 3, fake, None, ws, big, None)
    assert st == 1 and "alphas" in kt.kt_last_error()
    st = L.kt_pooled_kurtosis_loss_grad(fake, 128, fake, 128, 1, 16, 128, 1, 1, 1.8, -1.0, fake, None, None, ws, big,
                                        None)
    assert st == 1 and "rms_eps" in kt.kt_last_error()
    st = L.kt_kurtosis_loss_grad(fake, 128, fake, 128, 1, 16, 128, 1, 1, 0.0, fake, None, None, ws, 16, None)
    assert st == 4                   # workspace too small


def test_workspace_queries_of_the_widened_ops():
    f = kt.kt_workspace_bytes
    assert f(kt.KT_OP_POOLED_LOSS_GRAD, 256, 4096, 128, kt.KT_BF16) > f(kt.KT_OP_LOSS_GRAD, 256, 4096, 128, kt.KT_BF16)
    assert f(kt.KT_OP_QUANT_METRICS, 1, 1024, 256, kt.KT_BF16) >= 1024 * 256 * 4
    assert f(kt.KT_OP_FUSE_ROTATION, 1, 1000, 256, kt.KT_F32) >= 1000 * 256 * 4
    assert f(kt.KT_OP_SENSITIVITY, 1, 1, 128, kt.KT_F32) > 0
    # fake-quant: the fp32 staging slice of rotated rows is bounded (1 GiB), whatever n is
    small, large = f(kt.KT_OP_FAKEQUANT, 1, 1 << 14, 4096, kt.KT_BF16), f(kt.KT_OP_FAKEQUANT, 1, 1 << 20, 4096, kt.KT_BF16)
    assert small >= (1 << 14) * 4096 * 4 and large - small < (1 << 20) * 1200 + (1 << 30)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_static_scratch_entry_rejects_what_does_not_fit_before_touching_a_device():
    L = kt.lib()
    fake = ctypes.c_void_p(4096)
    assert L.kt_cayley_step_static(fake, fake, None, 2, 512, 0.01, None, None, None) == 6
    assert "static scratch" in kt.kt_last_error()
    assert L.kt_cayley_step_static(fake, fake, None, 1, 1024, 0.01, None, None, None) == 6
    assert L.kt_cayley_step_static(None, fake, None, 1, 256, 0.01, None, None, None) == 1
    assert L.kt_cayley_step_static(fake, fake, None, 1, 200, 0.01, None, None, None) == 2
    assert L.kt_cayley_step_static(fake, fake, None, 1, 256, float("nan"), None, None, None) == 1


def test_header_compiles_as_plain_c(tmp_path):
    """The boundary is a C ABI: include/kt.h must be valid C99 on its own (no C++-isms, no torch types)."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_kt.c"
    src.write_text('#include "kt.h"\n'
                   "int main(void) { kt_dtype t = KT_BF16; kt_op o = KT_OP_CAYLEY; kt_status s = KT_OK;\n"
                   "  return (int)t + (int)o + (int)s == 2 ? 0 : 1; }\n")
    res = subprocess.run([cc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                          "-c", str(src), "-o", str(tmp_path / "use_kt.o")], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
