"""ctypes binding of libkurtail.so; same names as the C entry points."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkurtail.so")
_lib = None

KT_F32, KT_BF16 = 0, 1
KT_OP_LOSS_GRAD, KT_OP_CAYLEY, KT_OP_FAKEQUANT, KT_OP_POOLED_LOSS_GRAD, KT_OP_QUANT_METRICS = 0, 1, 2, 3, 4
KT_OP_FUSE_ROTATION, KT_OP_SENSITIVITY, KT_OP_LOSS_GRAD_RECOMPUTE, KT_OP_POOLED_LOSS_GRAD_RECOMPUTE = 5, 6, 7, 8

EXPORTS = ("kt_version", "kt_last_error", "kt_workspace_bytes", "kt_kurtosis_loss_grad",
           "kt_pooled_kurtosis_loss_grad", "kt_cayley_step", "kt_cayley_adam_step", "kt_rotate_fakequant_int4", "kt_rotate_quant_metrics", "kt_hadamard_rows", "kt_fuse_rotation", "kt_quant_sensitivity", "kt_profile_enable", "kt_profile_read",
           "kt_profile_reset", "kt_cayley_step_static", "kt_build_id")


class KtError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"kt status {status}: {text}")
        self.status = status


def lib_path():
    return _LIB_PATH


def lib():
    """Load the library.  It is built first when no built library is present, and rebuilt when the one present
    was compiled from other sources than those in csrc/ now (it carries an id of its sources): a stale library
    is never loaded silently."""
    global _lib
    if _lib is not None:
        return _lib
    from .build import build_library, source_id
    if not os.path.exists(_LIB_PATH):
        build_library()
    L = ctypes.CDLL(_LIB_PATH)
    want = source_id()
    try:
        L.kt_build_id.restype = ctypes.c_char_p
        have = L.kt_build_id().decode()
    except AttributeError:
        have = "(none)"
    if have != want:
        import warnings
        warnings.warn(f"libkurtail.so was built from other sources (id {have}, csrc/ now {want}): rebuilding")
        tmp = _LIB_PATH + ".stale"
        os.replace(_LIB_PATH, tmp)     # the mapped file stays valid; the new one gets a fresh inode
        build_library()
        os.remove(tmp)
        L = ctypes.CDLL(_LIB_PATH)
        L.kt_build_id.restype = ctypes.c_char_p
        if L.kt_build_id().decode() != want:
            raise RuntimeError("libkurtail.so does not match its sources after a rebuild")
    vp, i64, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    i32 = ctypes.c_int32
    L.kt_version.restype = i32
    L.kt_version.argtypes = []
    L.kt_last_error.restype = ctypes.c_char_p
    L.kt_last_error.argtypes = []
    L.kt_workspace_bytes.restype = sz
    L.kt_workspace_bytes.argtypes = [i32, i64, i64, i64, i32]
    L.kt_kurtosis_loss_grad.restype = i32
    L.kt_kurtosis_loss_grad.argtypes = [vp, i64, vp, i64, i64, i64, i64, i32, i32, f32,
                                        vp, vp, vp, vp, sz, vp]
    L.kt_pooled_kurtosis_loss_grad.restype = i32
    L.kt_pooled_kurtosis_loss_grad.argtypes = [vp, i64, vp, i64, i64, i64, i64, i32, i32, f32, f32, vp, vp, vp,
                                               vp, sz, vp]
    L.kt_rotate_quant_metrics.restype = i32
    L.kt_rotate_quant_metrics.argtypes = [vp, i64, vp, i64, i64, i64, i64, i32, i32, f32, vp, vp, vp, vp, vp, vp,
                                          vp, sz, vp]
    L.kt_hadamard_rows.restype = i32
    L.kt_hadamard_rows.argtypes = [vp, i64, vp, i64, vp, i64, i64, i32, vp]
    L.kt_fuse_rotation.restype = i32
    L.kt_fuse_rotation.argtypes = [vp, i64, vp, i64, vp, i64, i64, i64, i32, vp, sz, vp]
    L.kt_quant_sensitivity.restype = i32
    L.kt_quant_sensitivity.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, sz, vp]
    L.kt_cayley_step.restype = i32
    L.kt_cayley_step.argtypes = [vp, vp, vp, i64, i64, f32, vp, vp, vp, sz, vp]
    L.kt_cayley_step_static.restype = i32
    L.kt_cayley_step_static.argtypes = [vp, vp, vp, i64, i64, f32, vp, vp, vp]
    L.kt_cayley_adam_step.restype = i32
    L.kt_cayley_adam_step.argtypes = [vp, vp, vp, vp, i64, vp, i64, i64, f32, f32, f32, f32, f32, vp, vp, vp,
                                      vp, sz, vp]
    L.kt_rotate_fakequant_int4.restype = i32
    L.kt_rotate_fakequant_int4.argtypes = [vp, i64, vp, i64, i64, i64, i64, i32, i32, f32,
                                           vp, vp, vp, vp, vp, sz, vp]
    L.kt_profile_enable.restype = i32
    L.kt_profile_enable.argtypes = [i32]
    L.kt_profile_read.restype = i32
    L.kt_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    L.kt_profile_reset.restype = i32
    L.kt_profile_reset.argtypes = []
    _lib = L
    return L


def kt_version():
    return int(lib().kt_version())


def kt_last_error():
    return lib().kt_last_error().decode()


def kt_workspace_bytes(op, batch, n, d, x_dtype):
    return int(lib().kt_workspace_bytes(op, batch, n, d, x_dtype))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return KT_BF16
    if t.dtype == torch.float32:
        return KT_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream) if hasattr(stream, "cuda_stream") else ctypes.c_void_p(stream)


def _check(status):
    if status != 0:
        raise KtError(status, kt_last_error())


class Workspace:
    """A caller-owned scratch buffer (torch uint8 tensor) that grows on demand."""

    def __init__(self, device="cuda"):
        self.device = device
        self.buf = None

    def get(self, nbytes):
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = None
            self.buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=self.device)
        return self.buf


def _xr_dims(X, R):
    if X.dim() == 2:
        X = X.unsqueeze(0)
    if R.dim() == 2:
        R = R.unsqueeze(0)
    batch, n, d = X.shape
    assert R.shape == (batch, d, d), (X.shape, R.shape)
    assert X.stride(2) == 1 and R.stride(2) == 1
    assert batch == 1 or (X.stride(0) == n * X.stride(1) and R.stride(0) == d * R.stride(1))
    return X, R, batch, n, d


def kt_kurtosis_loss_grad(X, R, *, kappa_target=0.0, loss=None, row_kurt=None, dR=None,
                          workspace=None, stream=None, recompute=False):
    """loss [batch] fp32 (returned), optional row_kurt [batch][n] and dR [batch][d][d] outputs.
    recompute=True hands the library only the smaller workspace, with which it recomputes Y for the
    backward pass instead of keeping it (same result)."""
    X, R, batch, n, d = _xr_dims(X, R)
    if loss is None:
        loss = torch.empty(batch, dtype=torch.float32, device=X.device)
    xdt = _dtype_code(X)
    need = kt_workspace_bytes(KT_OP_LOSS_GRAD_RECOMPUTE if recompute else KT_OP_LOSS_GRAD, batch, n, d, xdt)
    ws = (workspace or Workspace(X.device)).get(need)
    _check(lib().kt_kurtosis_loss_grad(_ptr(X), X.stride(1), _ptr(R), R.stride(1), batch, n, d, xdt,
                                       _dtype_code(R), float(kappa_target), _ptr(loss),
                                       _ptr(row_kurt), _ptr(dR), _ptr(ws), need if recompute else ws.numel(),
                                       _stream(stream)))
    return loss


def kt_pooled_kurtosis_loss_grad(X, R, *, kappa_target=1.8, rms_eps=0.0, loss=None, kappa=None, dR=None,
                                 workspace=None, stream=None, recompute=False):
    """Paper-literal pooled loss [batch] fp32 (returned), optional kappa [batch] and dR outputs.
    recompute: as for kt_kurtosis_loss_grad."""
    X, R, batch, n, d = _xr_dims(X, R)
    if loss is None:
        loss = torch.empty(batch, dtype=torch.float32, device=X.device)
    xdt = _dtype_code(X)
    need = kt_workspace_bytes(KT_OP_POOLED_LOSS_GRAD_RECOMPUTE if recompute else KT_OP_POOLED_LOSS_GRAD,
                              batch, n, d, xdt)
    ws = (workspace or Workspace(X.device)).get(need)
    _check(lib().kt_pooled_kurtosis_loss_grad(_ptr(X), X.stride(1), _ptr(R), R.stride(1), batch, n, d, xdt,
                                              _dtype_code(R), float(kappa_target), float(rms_eps), _ptr(loss),
                                              _ptr(kappa), _ptr(dR), _ptr(ws), need if recompute else ws.numel(),
                                              _stream(stream)))
    return loss


def kt_cayley_step(R, dR, lr, *, R_lowp=None, ortho_err=None, info=None, workspace=None, stream=None):
    """In-place Cayley step on R [batch][d][d] fp32."""
    Rv = R if R.dim() == 3 else R.unsqueeze(0)
    batch, d, _ = Rv.shape
    assert Rv.is_contiguous() and dR.is_contiguous() and dR.numel() == Rv.numel()
    assert R.dtype == torch.float32 and dR.dtype == torch.float32
    need = kt_workspace_bytes(KT_OP_CAYLEY, batch, 0, d, KT_F32)
    ws = (workspace or Workspace(R.device)).get(need)
    _check(lib().kt_cayley_step(_ptr(Rv), _ptr(dR), _ptr(R_lowp), batch, d, float(lr), _ptr(ortho_err),
                                _ptr(info), _ptr(ws), ws.numel(), _stream(stream)))
    return R


def kt_cayley_step_static(R, dR, lr, *, R_lowp=None, ortho_err=None, info=None, stream=None):
    """kt_cayley_step on the library's own static device scratch: no workspace, no allocation (small sizes)."""
    Rv = R if R.dim() == 3 else R.unsqueeze(0)
    batch, d, _ = Rv.shape
    assert Rv.is_contiguous() and dR.is_contiguous() and dR.numel() == Rv.numel()
    assert R.dtype == torch.float32 and dR.dtype == torch.float32
    _check(lib().kt_cayley_step_static(_ptr(Rv), _ptr(dR), _ptr(R_lowp), batch, d, float(lr), _ptr(ortho_err),
                                       _ptr(info), _stream(stream)))
    return R


def kt_cayley_adam_step(R, dR, M, v, step, lr, *, beta1=0.9, beta2=0.99, eps=1e-8, q=0.5, R_lowp=None,
                        ortho_err=None, info=None, scalars=None, workspace=None, stream=None):
    """In-place Cayley Adam step on R [batch][d][d] fp32 with state M [batch][d][d], v [batch]."""
    Rv = R if R.dim() == 3 else R.unsqueeze(0)
    batch, d, _ = Rv.shape
    assert Rv.is_contiguous() and dR.is_contiguous() and M.is_contiguous() and v.is_contiguous()
    assert dR.numel() == Rv.numel() and M.numel() == Rv.numel() and v.numel() == batch
    assert R.dtype == dR.dtype == M.dtype == v.dtype == torch.float32
    need = kt_workspace_bytes(KT_OP_CAYLEY, batch, 0, d, KT_F32)
    ws = (workspace or Workspace(R.device)).get(need)
    _check(lib().kt_cayley_adam_step(_ptr(Rv), _ptr(dR), _ptr(M), _ptr(v), int(step), _ptr(R_lowp), batch, d,
                                     float(lr), float(beta1), float(beta2), float(eps), float(q),
                                     _ptr(ortho_err), _ptr(info), _ptr(scalars), _ptr(ws), ws.numel(),
                                     _stream(stream)))
    return R


def kt_rotate_fakequant_int4(X, R, *, clip_ratio=1.0, scales_in=None, scales_out=None, codes=None,
                             err=None, workspace=None, stream=None):
    X, R, batch, n, d = _xr_dims(X, R)
    xdt = _dtype_code(X)
    need = kt_workspace_bytes(KT_OP_FAKEQUANT, batch, n, d, xdt)
    ws = (workspace or Workspace(X.device)).get(need)
    _check(lib().kt_rotate_fakequant_int4(_ptr(X), X.stride(1), _ptr(R), R.stride(1), batch, n, d, xdt,
                                          _dtype_code(R), float(clip_ratio), _ptr(scales_in),
                                          _ptr(scales_out), _ptr(codes), _ptr(err), _ptr(ws),
                                          ws.numel(), _stream(stream)))


def kt_rotate_quant_metrics(X, R, *, quantile=0.98, Y=None, amax=None, threshold=None, err_sym=None,
                            err_asym=None, success=None, workspace=None, stream=None):
    X, R, batch, n, d = _xr_dims(X, R)
    xdt = _dtype_code(X)
    need = kt_workspace_bytes(KT_OP_QUANT_METRICS, batch, n, d, xdt)
    ws = (workspace or Workspace(X.device)).get(need)
    _check(lib().kt_rotate_quant_metrics(_ptr(X), X.stride(1), _ptr(R), R.stride(1), batch, n, d, xdt,
                                         _dtype_code(R), float(quantile), _ptr(Y), _ptr(amax), _ptr(threshold),
                                         _ptr(err_sym), _ptr(err_asym), _ptr(success), _ptr(ws), ws.numel(),
                                         _stream(stream)))


def kt_hadamard_rows(X, *, signs=None, out=None, stream=None):
    """Y = (X * signs) H_d / sqrt(d) on the rows of X [n][d] (fp32 or bf16); returns Y (out or new)."""
    assert X.dim() == 2 and X.stride(1) == 1
    n, d = X.shape
    Y = torch.empty_like(X) if out is None else out
    assert Y.shape == X.shape and Y.dtype == X.dtype and Y.stride(1) == 1
    if signs is not None:
        assert signs.dtype == torch.int8 and signs.numel() == d and signs.is_contiguous()
    _check(lib().kt_hadamard_rows(_ptr(X), X.stride(0), _ptr(Y), Y.stride(0), _ptr(signs), n, d, _dtype_code(X),
                                  _stream(stream)))
    return Y


def kt_fuse_rotation(W, R, side, *, out=None, workspace=None, stream=None):
    """side 0: W [k][d] -> W R;  side 1: W [d][k] -> R^T W  (fp32)."""
    d = R.shape[-1]
    k = W.shape[0] if side == 0 else W.shape[1]
    assert W.dtype == R.dtype == torch.float32 and W.stride(1) == 1 and R.stride(-1) == 1 and R.dim() == 2
    out = torch.empty_like(W) if out is None else out
    need = kt_workspace_bytes(KT_OP_FUSE_ROTATION, 1, k, d, KT_F32)
    ws = (workspace or Workspace(W.device)).get(need)
    _check(lib().kt_fuse_rotation(_ptr(W), W.stride(0), _ptr(R), R.stride(0), _ptr(out), out.stride(0), k, d,
                                  int(side), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def kt_quant_sensitivity(Y, alphas, *, bits=4, workspace=None, stream=None):
    """Returns (out [2] = {s_opt, MSE(s_opt)}, gamma [len(alphas)]) as device tensors."""
    assert Y.dtype == torch.float32 and Y.is_contiguous() and alphas.dtype == torch.float32
    out = torch.empty(2, dtype=torch.float32, device=Y.device)
    gamma = torch.empty(alphas.numel(), dtype=torch.float32, device=Y.device)
    need = kt_workspace_bytes(KT_OP_SENSITIVITY, 1, 1, 128, KT_F32)
    ws = (workspace or Workspace(Y.device)).get(need)
    _check(lib().kt_quant_sensitivity(_ptr(Y), Y.numel(), int(bits), _ptr(alphas), alphas.numel(), _ptr(out),
                                      _ptr(gamma), _ptr(ws), ws.numel(), _stream(stream)))
    return out, gamma


def kt_profile_enable(max_records):
    _check(lib().kt_profile_enable(int(max_records)))


def kt_profile_reset():
    _check(lib().kt_profile_reset())


def kt_profile_read(kernel_id):
    """(total_ms, launches) of the bracketed launches with this id since the last reset."""
    tot, cnt = ctypes.c_double(0.0), ctypes.c_int32(0)
    _check(lib().kt_profile_read(int(kernel_id), ctypes.byref(tot), ctypes.byref(cnt)))
    return tot.value, cnt.value
