"""ctypes front end of the CPU oracle (``eqat_oracle.c``)  --  test infrastructure.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It takes and returns numpy arrays; bf16 data must be widened to
float32 by the caller (exact).  Nothing here imports the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "eqat_oracle.c")
# EQAT_ORACLE_SANITIZE=1: a build with AddressSanitizer and UndefinedBehaviorSanitizer (the process must then run with
# gcc's libasan preloaded); tests/test_sanitizers.py runs the oracle's pins that way
_SANITIZE = os.environ.get("EQAT_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libeqat_oracle_san.so" if _SANITIZE else "libeqat_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] \
            if _SANITIZE else ["-O2"]
        cmd = ["gcc", *opt, "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _ll(v):
    return ctypes.c_longlong(int(v))


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"oracle {name} rejected its arguments (rc={rc})")


def num_threads() -> int:
    return int(_load().eqo_num_threads())


def _group(I, g):
    return int(I) if g == -1 else int(g)


def packed_w_row_bytes(I, bits):
    return int(I) * int(bits) // 8


def packed_z_row_bytes(G, bits):
    return 4 * ((int(G) * int(bits) + 31) // 32)


def init_minmax(W, bits, g):
    W, pW = _f32(W)
    O, I = W.shape
    g = _group(I, g)
    s = np.empty((O, I // g), np.float32)
    z = np.empty((O, I // g), np.float32)
    _check(_load().eqo_init_minmax(pW, _ll(O), _ll(I), int(bits), _ll(g), _ptr(s), _ptr(z)), "init_minmax")
    return s, z


def quantize(W, s, z, bits, g):
    """Eq.(1): integer codes [O,I] and clamp side (-1 below, 0 in range, +1 above)."""
    W, pW = _f32(W); s, ps = _f32(s); z, pz = _f32(z)
    O, I = W.shape
    g = _group(I, g)
    codes = np.empty((O, I), np.int32)
    side = np.empty((O, I), np.int8)
    _check(_load().eqo_quantize(pW, ps, pz, _ll(O), _ll(I), int(bits), _ll(g), _ptr(codes), _ptr(side)), "quantize")
    return codes, side


def fake_quant(W, s, z, bits, g):
    """Eq.(2) after Eq.(1): the dequantised weights, fp64."""
    W, pW = _f32(W); s, ps = _f32(s); z, pz = _f32(z)
    O, I = W.shape
    g = _group(I, g)
    out = np.empty((O, I), np.float64)
    _check(_load().eqo_fake_quant(pW, ps, pz, _ll(O), _ll(I), int(bits), _ll(g), _ptr(out)), "fake_quant")
    return out


def fq_linear_fwd(X, W, s, z, bits, g):
    X, pX = _f32(X); W, pW = _f32(W); s, ps = _f32(s); z, pz = _f32(z)
    T, I = X.shape
    O = W.shape[0]
    g = _group(I, g)
    Y = np.empty((T, O), np.float64)
    _check(_load().eqo_fq_linear_fwd(pX, pW, ps, pz, _ll(T), _ll(I), _ll(O), int(bits), _ll(g), _ptr(Y)), "fq_linear_fwd")
    return Y


def fq_linear_bwd(X, W, s, z, dY, bits, g, want=("dX", "dW", "ds", "dz")):
    """Returns a dict with the requested gradients (fp64)."""
    W, pW = _f32(W); s, ps = _f32(s); z, pz = _f32(z); dY, pdY = _f32(dY)
    O, I = W.shape
    T = dY.shape[0]
    g = _group(I, g)
    G = I // g
    pX = None
    if X is not None:
        X, pX = _f32(X)
    out = {}
    if "dX" in want: out["dX"] = np.empty((T, I), np.float64)
    if "dW" in want: out["dW"] = np.empty((O, I), np.float64)
    if "ds" in want: out["ds"] = np.empty((O, G), np.float64)
    if "dz" in want: out["dz"] = np.empty((O, G), np.float64)
    _check(_load().eqo_fq_linear_bwd(pX, pW, ps, pz, pdY, _ll(T), _ll(I), _ll(O), int(bits), _ll(g),
                                     _ptr(out.get("dX")), _ptr(out.get("dW")), _ptr(out.get("ds")),
                                     _ptr(out.get("dz"))), "fq_linear_bwd")
    return out


def pack(W, s, z, bits, g):
    W, pW = _f32(W); s, ps = _f32(s); z, pz = _f32(z)
    O, I = W.shape
    g = _group(I, g)
    Wp = np.empty((O, packed_w_row_bytes(I, bits)), np.uint8)
    zp = np.empty((O, packed_z_row_bytes(I // g, bits)), np.uint8)
    _check(_load().eqo_pack(pW, ps, pz, _ll(O), _ll(I), int(bits), _ll(g), _ptr(Wp), _ptr(zp)), "pack")
    return Wp, zp


def unpack(Wp, zp, I, bits, g):
    Wp = np.ascontiguousarray(Wp, np.uint8); zp = np.ascontiguousarray(zp, np.uint8)
    O = Wp.shape[0]
    g = _group(I, g)
    codes = np.empty((O, I), np.int32)
    zc = np.empty((O, I // g), np.int32)
    _check(_load().eqo_unpack(_ptr(Wp), _ptr(zp), _ll(O), _ll(I), int(bits), _ll(g), _ptr(codes), _ptr(zc)), "unpack")
    return codes, zc


def qlinear_fwd(X, Wp, s, zp, bits, g):
    X, pX = _f32(X); s, ps = _f32(s)
    Wp = np.ascontiguousarray(Wp, np.uint8); zp = np.ascontiguousarray(zp, np.uint8)
    T, I = X.shape
    O = Wp.shape[0]
    g = _group(I, g)
    Y = np.empty((T, O), np.float64)
    _check(_load().eqo_qlinear_fwd(pX, _ptr(Wp), ps, _ptr(zp), _ll(T), _ll(I), _ll(O), int(bits), _ll(g), _ptr(Y)), "qlinear_fwd")
    return Y


def qlinear_bwd(X, Wp, s, zp, dY, I, bits, g, want=("dX", "ds")):
    s, ps = _f32(s); dY, pdY = _f32(dY)
    Wp = np.ascontiguousarray(Wp, np.uint8); zp = np.ascontiguousarray(zp, np.uint8)
    O = Wp.shape[0]
    T = dY.shape[0]
    g = _group(I, g)
    pX = None
    if X is not None:
        X, pX = _f32(X)
    out = {}
    if "dX" in want: out["dX"] = np.empty((T, I), np.float64)
    if "ds" in want: out["ds"] = np.empty((O, I // g), np.float64)
    _check(_load().eqo_qlinear_bwd(pX, _ptr(Wp), ps, _ptr(zp), pdY, _ll(T), _ll(I), _ll(O), int(bits), _ll(g),
                                   _ptr(out.get("dX")), _ptr(out.get("ds"))), "qlinear_bwd")
    return out


def qlinear_fwd_z(X, Wp, s, z, bits, g):
    """E2E-QP forward with floating-point (trainable) zero points: What = (w_q - z) * s, z not rounded (Sec. 3.3)."""
    X, pX = _f32(X); s, ps = _f32(s); z, pz = _f32(z)
    Wp = np.ascontiguousarray(Wp, np.uint8)
    T, I = X.shape
    O = Wp.shape[0]
    g = _group(I, g)
    Y = np.empty((T, O), np.float64)
    _check(_load().eqo_qlinear_fwd_z(pX, _ptr(Wp), ps, pz, _ll(T), _ll(I), _ll(O), int(bits), _ll(g), _ptr(Y)), "qlinear_fwd_z")
    return Y


def qlinear_bwd_z(X, Wp, s, z, dY, I, bits, g, want=("dX", "ds", "dz")):
    """E2E-QP backward with trainable s and z: dX, ds = group-sum dWhat * (w_q - z), dz = -s * group-sum dWhat."""
    s, ps = _f32(s); z, pz = _f32(z); dY, pdY = _f32(dY)
    Wp = np.ascontiguousarray(Wp, np.uint8)
    O = Wp.shape[0]
    T = dY.shape[0]
    g = _group(I, g)
    pX = None
    if X is not None:
        X, pX = _f32(X)
    out = {}
    if "dX" in want: out["dX"] = np.empty((T, I), np.float64)
    if "ds" in want: out["ds"] = np.empty((O, I // g), np.float64)
    if "dz" in want: out["dz"] = np.empty((O, I // g), np.float64)
    _check(_load().eqo_qlinear_bwd_z(pX, _ptr(Wp), ps, pz, pdY, _ll(T), _ll(I), _ll(O), int(bits), _ll(g),
                                     _ptr(out.get("dX")), _ptr(out.get("ds")), _ptr(out.get("dz"))), "qlinear_bwd_z")
    return out


def recon_loss(Y, Yref, want_dY=True):
    """Block reconstruction loss (Sec. 3.2; the form is our reading): mean squared error and its gradient 2 (Y - Yref) / n."""
    Y, pY = _f32(Y); Yref, pR = _f32(Yref)
    if Y.shape != Yref.shape:
        raise ValueError("shapes differ")
    loss = ctypes.c_double(0.0)
    dY = np.empty(Y.shape, np.float64) if want_dY else None
    _check(_load().eqo_recon_loss(pY, pR, _ll(Y.size), ctypes.byref(loss), _ptr(dY)), "recon_loss")
    return float(loss.value), dY


S_MIN = float(np.float32(1e-10))      # lower bound of a step size: the floor of its min/max initialisation


def adamw(p, grad, m, v, lr, beta1, beta2, eps, weight_decay, step, p_min=-np.inf):
    """One AdamW step (decoupled weight decay, bias correction; step counted from 1), then p = max(p, p_min) (step sizes:
    p_min = S_MIN).  Returns new (p, m, v) as fp64 arrays."""
    p = np.array(p, dtype=np.float64, order="C"); m = np.array(m, dtype=np.float64, order="C")
    v = np.array(v, dtype=np.float64, order="C")
    grad, pg = _f32(grad)
    if not (p.shape == grad.shape == m.shape == v.shape):
        raise ValueError("shapes differ")
    d = ctypes.c_double
    _check(_load().eqo_adamw(_ptr(p), pg, _ptr(m), _ptr(v), _ll(p.size), d(lr), d(beta1), d(beta2), d(eps), d(weight_decay),
                             int(step), d(p_min)), "adamw")
    return p, m, v
