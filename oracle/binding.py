"""ctypes access to ``libkt_oracle.so`` (test infrastructure, see package doc)."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kt_oracle.c")
_LIB = os.path.join(_HERE, "libkt_oracle.so")
_lib = None


def build_oracle(force=False):
    """Compile kt_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_oracle()
    lib = ctypes.CDLL(_LIB)
    dp = ctypes.POINTER(ctypes.c_double)
    fp = ctypes.POINTER(ctypes.c_float)
    i8p = ctypes.POINTER(ctypes.c_int8)
    i64 = ctypes.c_int64
    lib.kto_num_threads.restype = ctypes.c_int
    lib.kto_rotate.argtypes = [dp, dp, i64, i64, dp]
    lib.kto_rotate.restype = None
    lib.kto_row_moments.argtypes = [dp, i64, dp]
    lib.kto_row_moments.restype = ctypes.c_int
    lib.kto_loss_grad.argtypes = [dp, dp, i64, i64, ctypes.c_double, dp, dp, dp, dp]
    lib.kto_loss_grad.restype = None
    lib.kto_pooled_loss_grad.argtypes = [dp, dp, i64, i64, ctypes.c_double, ctypes.c_double, dp, dp, dp, dp]
    lib.kto_pooled_loss_grad.restype = None
    lib.kto_cayley_step.argtypes = [dp, dp, i64, ctypes.c_double, dp, dp]
    lib.kto_cayley_step.restype = ctypes.c_int
    lib.kto_cayley_step_right.argtypes = [dp, dp, i64, ctypes.c_double, dp]
    lib.kto_cayley_step_right.restype = ctypes.c_int
    cd = ctypes.c_double
    lib.kto_cayley_adam_step.argtypes = [dp, dp, dp, cd, i64, i64, cd, cd, cd, cd, cd, dp, dp, dp, dp]
    lib.kto_cayley_adam_step.restype = ctypes.c_int
    lib.kto_quant_metrics.argtypes = [dp, dp, i64, i64, ctypes.c_double, fp, fp, dp, dp]
    lib.kto_quant_metrics.restype = ctypes.c_int64
    lib.kto_hadamard_rows.argtypes = [dp, dp, i64, i64, dp]
    lib.kto_hadamard_rows.restype = ctypes.c_int
    lib.kto_hadamard_factor.argtypes = [i64, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_int)]
    lib.kto_hadamard_factor.restype = ctypes.c_int
    lib.kto_hadamard_matrix.argtypes = [i64, ctypes.c_int, ctypes.POINTER(ctypes.c_int8)]
    lib.kto_hadamard_matrix.restype = None
    lib.kto_fuse_rotation.argtypes = [dp, dp, i64, i64, ctypes.c_int, dp]
    lib.kto_fuse_rotation.restype = None
    lib.kto_quant_sensitivity.argtypes = [fp, i64, ctypes.c_int, fp, ctypes.c_int, ctypes.c_double, dp, dp]
    lib.kto_quant_mse.argtypes = [fp, i64, ctypes.c_int, ctypes.c_float]
    lib.kto_quant_mse.restype = ctypes.c_double
    lib.kto_quant_sensitivity.restype = None
    lib.kto_fakequant_int4.argtypes = [dp, dp, i64, i64, ctypes.c_float, fp, fp, i8p, dp]
    lib.kto_fakequant_int4.restype = None
    _lib = lib
    return lib


def _d(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a, ct=ctypes.c_double):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def num_threads():
    return int(_load().kto_num_threads())


def rotate(X, R):
    X, R = _d(X), _d(R)
    n, d = X.shape
    assert R.shape == (d, d)
    Y = np.empty((n, d), dtype=np.float64)
    _load().kto_rotate(_p(X), _p(R), n, d, _p(Y))
    return Y


def row_moments(y):
    """Returns (mu, m2, m3, m4, kappa, degenerate) of one row."""
    y = _d(y).ravel()
    out = np.empty(5, dtype=np.float64)
    deg = _load().kto_row_moments(_p(y), y.size, _p(out))
    return (*out.tolist(), bool(deg))


def loss_grad(X, R, kappa_target=0.0, want_G=False, want_dR=True):
    """Returns dict(loss, row_kurt, dR[, G]) for Y = X R."""
    X, R = _d(X), _d(R)
    n, d = X.shape
    assert R.shape == (d, d)
    loss = np.zeros(1, dtype=np.float64)
    rk = np.empty(n, dtype=np.float64)
    G = np.empty((n, d), dtype=np.float64) if want_G else None
    dR = np.empty((d, d), dtype=np.float64) if want_dR else None
    _load().kto_loss_grad(_p(X), _p(R), n, d, float(kappa_target), _p(loss), _p(rk),
                          _p(G), _p(dR))
    out = {"loss": float(loss[0]), "row_kurt": rk, "dR": dR}
    if want_G:
        out["G"] = G
    return out


def pooled_loss_grad(X, R, kappa_target=1.8, rms_eps=0.0, want_G=False, want_dR=True):
    """Paper-literal pooled loss of one problem.  Returns dict(loss, kappa, G, dR)."""
    X, R = _d(X), _d(R)
    n, d = X.shape
    assert R.shape == (d, d)
    loss = np.zeros(1); kap = np.zeros(1)
    G = np.empty((n, d)) if want_G else None
    dR = np.empty((d, d)) if want_dR else None
    _load().kto_pooled_loss_grad(_p(X), _p(R), n, d, float(kappa_target), float(rms_eps), _p(loss), _p(kap),
                                 _p(G), _p(dR))
    return {"loss": float(loss[0]), "kappa": float(kap[0]), "G": G, "dR": dR}


def cayley_step(R, G, lr, want_A=False):
    R, G = _d(R), _d(G)
    d = R.shape[0]
    assert R.shape == (d, d) and G.shape == (d, d)
    out = np.empty((d, d), dtype=np.float64)
    A = np.empty((d, d), dtype=np.float64) if want_A else None
    rc = _load().kto_cayley_step(_p(R), _p(G), d, float(lr), _p(out), _p(A))
    if rc != 0:
        raise ArithmeticError("singular system in Cayley step")
    return (out, A) if want_A else out


def cayley_step_right(R, G, lr):
    R, G = _d(R), _d(G)
    d = R.shape[0]
    out = np.empty((d, d), dtype=np.float64)
    rc = _load().kto_cayley_step_right(_p(R), _p(G), d, float(lr), _p(out))
    if rc != 0:
        raise ArithmeticError("singular system in Cayley step")
    return out


def cayley_adam_step(R, G, M, v, k, lr, beta1=0.9, beta2=0.99, eps=1e-8, q=0.5):
    """One Cayley Adam step.  Returns dict(R, M, v, r, alpha, w_norm)."""
    R, G, M = _d(R), _d(G), _d(M)
    d = R.shape[0]
    Rout = np.empty((d, d), dtype=np.float64)
    Mout = np.empty((d, d), dtype=np.float64)
    vout = np.empty(1, dtype=np.float64)
    scal = np.empty(3, dtype=np.float64)
    rc = _load().kto_cayley_adam_step(_p(R), _p(G), _p(M), float(v), d, int(k), float(lr), float(beta1),
                                      float(beta2), float(eps), float(q), _p(Rout), _p(Mout), _p(vout), _p(scal))
    if rc != 0:
        raise ArithmeticError("singular system in Cayley Adam step")
    return {"R": Rout, "M": Mout, "v": float(vout[0]), "r": float(scal[0]), "alpha": float(scal[1]),
            "w_norm": float(scal[2])}


def fakequant_int4(X, R, clip=1.0, scales_in=None):
    """Returns dict(scales float32[n], codes int8[n][d], err float64[n][2])."""
    X, R = _d(X), _d(R)
    n, d = X.shape
    assert R.shape == (d, d)
    sin = None
    if scales_in is not None:
        sin = np.ascontiguousarray(np.asarray(scales_in, dtype=np.float32))
        assert sin.shape == (n,)
    sout = np.empty(n, dtype=np.float32)
    codes = np.empty((n, d), dtype=np.int8)
    err = np.empty((n, 2), dtype=np.float64)
    _load().kto_fakequant_int4(_p(X), _p(R), n, d, float(clip), _p(sin, ctypes.c_float),
                               _p(sout, ctypes.c_float), _p(codes, ctypes.c_int8), _p(err))
    return {"scales": sout, "codes": codes, "err": err}


def quant_metrics(X, R, quantile=0.98):
    """Per-token quantisation-quality figures of Y = X R.
    Returns dict(success int, amax float32[n][2], thr float32[n], err_sym, err_asym float64[n][2])."""
    X, R = _d(X), _d(R)
    n, d = X.shape
    amax = np.empty((n, 2), dtype=np.float32)
    thr = np.empty(n, dtype=np.float32)
    es = np.empty((n, 2), dtype=np.float64)
    ea = np.empty((n, 2), dtype=np.float64)
    succ = _load().kto_quant_metrics(_p(X), _p(R), n, d, float(quantile),
                                     _p(amax, ctypes.c_float), _p(thr, ctypes.c_float), _p(es), _p(ea))
    return {"success": int(succ), "amax": amax, "thr": thr, "err_sym": es, "err_asym": ea}


def hadamard_factor(d):
    """d = m * 2^k as the library splits it: (m, 2^k, kind), kind 0 Sylvester / 1 Paley I / 2 Paley II;
    None when d has no construction."""
    m, p2, kind = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int()
    if _load().kto_hadamard_factor(int(d), ctypes.byref(m), ctypes.byref(p2), ctypes.byref(kind)) != 0:
        return None
    return int(m.value), int(p2.value), int(kind.value)


def hadamard_matrix(m, kind):
    """The order-m factor H_m (entries +-1) of the given kind."""
    H = np.empty((m, m), dtype=np.int8)
    _load().kto_hadamard_matrix(int(m), int(kind), H.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)))
    return H


def hadamard_rows(X, signs=None):
    """Y = (X * signs) H_d / sqrt(d), rows of X; H_d = H_m (x) Sylvester_{2^k}."""
    X = _d(X)
    n, d = X.shape
    sg = None if signs is None else _d(signs)
    Y = np.empty((n, d), dtype=np.float64)
    if _load().kto_hadamard_rows(_p(X), _p(sg), n, d, _p(Y)) != 0:
        raise ValueError(f"no Hadamard construction for d = {d}")
    return Y


def fuse_rotation(W, R, side):
    """side 0: W [k][d] -> W R;  side 1: W [d][k] -> R^T W."""
    W, R = _d(W), _d(R)
    d = R.shape[0]
    k = W.shape[0] if side == 0 else W.shape[1]
    assert W.shape == ((k, d) if side == 0 else (d, k))
    out = np.empty_like(W)
    _load().kto_fuse_rotation(_p(W), _p(R), k, d, int(side), _p(out))
    return out


def quant_mse(y, s, bits=4):
    """Eq. 1: mean squared error of the symmetric `bits`-bit quantiser with step s over all of y."""
    yf = np.ascontiguousarray(np.asarray(y, dtype=np.float32)).ravel()
    return float(_load().kto_quant_mse(_p(yf, ctypes.c_float), yf.size, int(bits), float(np.float32(s))))


def quant_sensitivity(y, alphas, bits=4, flat_tol=1e-3):
    """Optimal step of a symmetric `bits`-bit quantiser over all of y (float32), by a dense scan and a
    bracketed refinement, and the sensitivity Gamma at the step fractions `alphas`.
    Returns dict(s_opt, mse_opt, flat (s_lo, s_hi): the smallest and largest scanned step whose MSE is within
    (1 + flat_tol) of the minimum, gamma float64[len(alphas)])."""
    yf = np.ascontiguousarray(np.asarray(y, dtype=np.float32)).ravel()
    al = np.ascontiguousarray(np.asarray(alphas, dtype=np.float32))
    out = np.empty(4, dtype=np.float64)
    gam = np.empty(al.size, dtype=np.float64)
    _load().kto_quant_sensitivity(_p(yf, ctypes.c_float), yf.size, int(bits), _p(al, ctypes.c_float), al.size,
                                  float(flat_tol), _p(out), _p(gam))
    return {"s_opt": float(out[0]), "mse_opt": float(out[1]), "flat": (float(out[2]), float(out[3])), "gamma": gam}
