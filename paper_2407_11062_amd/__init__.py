"""Thin Python binding of the eqat C ABI (``include/eqat.h``).

Argument marshalling only: every function here turns torch tensors into raw
device pointers and sizes, allocates outputs / workspace with torch when the
caller did not pass them, and calls the entry point of the same name in
``libeqat.so`` on torch's current stream.  No arithmetic of the method runs in
Python, and there is no fallback: without the built library every call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("EQAT_LIB", os.path.join(_HERE, "libeqat.so"))   # EQAT_LIB: a build under test

F32, BF16 = 0, 1
OP_FQ_FWD, OP_FQ_BWD, OP_Q_FWD, OP_Q_BWD, OP_QP_FWD, OP_QP_BWD = 0, 1, 2, 3, 4, 5
STATE_FQ_KEPT, STATE_Q_KEPT, STATE_PREPARED = 0, 1, 2

STATUS_NAMES = ["EQAT_OK", "EQAT_ERR_NULL", "EQAT_ERR_SHAPE", "EQAT_ERR_BITS", "EQAT_ERR_GROUP", "EQAT_ERR_DTYPE",
                "EQAT_ERR_ALIGN", "EQAT_ERR_WORKSPACE", "EQAT_ERR_DEVICE", "EQAT_ERR_HYPER"]

EXPORTS = ["eqat_status_string", "eqat_validate_desc", "eqat_packed_w_bytes", "eqat_packed_z_bytes",
           "eqat_workspace_bytes", "eqat_init_minmax", "eqat_fq_linear_fwd", "eqat_fq_linear_bwd",
           "eqat_fq_linear_fwd_keep", "eqat_fq_linear_bwd_kept", "eqat_fq_linear_fwd_kept", "eqat_pack",
           "eqat_init_minmax_batched", "eqat_pack_batched", "eqat_fq_quantize_batched",
           "eqat_unpack", "eqat_qlinear_fwd", "eqat_qlinear_bwd", "eqat_qlinear_fwd_keep", "eqat_qlinear_bwd_kept",
           "eqat_qlinear_fwd_z", "eqat_qlinear_bwd_z", "eqat_prepared_bytes", "eqat_qlinear_prepare",
           "eqat_qlinear_fwd_prepared", "eqat_qlinear_bwd_prepared", "eqat_qlinear_fwd_prepared_keep",
           "eqat_qlinear_bwd_prepared_kept", "eqat_unpack_state", "eqat_plan_item",
           "eqat_recon_loss_workspace_bytes", "eqat_recon_loss", "eqat_recon_loss_static", "eqat_block_ap_update",
           "eqat_profile_kernels", "eqat_profile_kernel_name",
           "eqat_profile_start", "eqat_profile_stop"]


class Desc(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int64), ("in_features", ctypes.c_int64), ("out_features", ctypes.c_int64),
                ("bits", ctypes.c_int32), ("group", ctypes.c_int32), ("act_dtype", ctypes.c_int32),
                ("w_dtype", ctypes.c_int32)]


class AdamW(ctypes.Structure):
    _fields_ = [("lr_w", ctypes.c_float), ("lr_q", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay_w", ctypes.c_float), ("weight_decay_q", ctypes.c_float),
                ("step", ctypes.c_int32)]


class EqatError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{fn}: {name}: {lib().eqat_status_string(status).decode()}")


_lib = None


def lib():
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_11062_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, dp, sz = ctypes.c_void_p, ctypes.POINTER(Desc), ctypes.c_size_t
        L.eqat_status_string.restype = ctypes.c_char_p
        L.eqat_status_string.argtypes = [ctypes.c_int]
        L.eqat_validate_desc.argtypes = [dp]
        for f in (L.eqat_packed_w_bytes, L.eqat_packed_z_bytes):
            f.restype, f.argtypes = sz, [dp]
        L.eqat_workspace_bytes.restype, L.eqat_workspace_bytes.argtypes = sz, [dp, ctypes.c_int]
        L.eqat_init_minmax.argtypes = [dp, vp, vp, vp, vp]
        L.eqat_fq_linear_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_fq_linear_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_fq_linear_fwd_keep.argtypes = L.eqat_fq_linear_fwd.argtypes
        L.eqat_fq_linear_bwd_kept.argtypes = L.eqat_fq_linear_bwd.argtypes
        L.eqat_fq_linear_fwd_kept.argtypes = L.eqat_fq_linear_fwd.argtypes
        L.eqat_init_minmax_batched.argtypes = [ctypes.c_int, dp, vp, vp, vp, vp]
        L.eqat_pack_batched.argtypes = [ctypes.c_int, dp, vp, vp, vp, vp, vp, vp]
        L.eqat_fq_quantize_batched.argtypes = [ctypes.c_int, dp, vp, vp, vp, vp, vp, vp]
        L.eqat_pack.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.eqat_unpack.argtypes = [dp, vp, vp, vp, vp, vp]
        L.eqat_qlinear_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_qlinear_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_qlinear_fwd_keep.argtypes = L.eqat_qlinear_fwd.argtypes
        L.eqat_qlinear_bwd_kept.argtypes = L.eqat_qlinear_bwd.argtypes
        L.eqat_qlinear_fwd_z.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_qlinear_bwd_z.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_prepared_bytes.restype, L.eqat_prepared_bytes.argtypes = sz, [dp]
        L.eqat_qlinear_prepare.argtypes = [dp, vp, vp, vp, sz, vp]
        L.eqat_qlinear_fwd_prepared.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_qlinear_bwd_prepared.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_qlinear_fwd_prepared_keep.argtypes = L.eqat_qlinear_fwd_prepared.argtypes
        L.eqat_plan_item.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        L.eqat_qlinear_bwd_prepared_kept.argtypes = L.eqat_qlinear_bwd_prepared.argtypes
        L.eqat_unpack_state.argtypes = [dp, ctypes.c_int, vp, vp, vp, vp, vp]
        L.eqat_recon_loss_workspace_bytes.restype, L.eqat_recon_loss_workspace_bytes.argtypes = sz, []
        L.eqat_recon_loss.argtypes = [ctypes.c_int64, ctypes.c_int32, vp, vp, vp, vp, vp, sz, vp]
        L.eqat_recon_loss_static.argtypes = [ctypes.c_int64, ctypes.c_int32, vp, vp, vp, vp, vp]
        L.eqat_block_ap_update.argtypes = [dp, ctypes.POINTER(AdamW)] + [vp] * 13
        L.eqat_profile_kernel_name.restype = ctypes.c_char_p
        L.eqat_profile_kernel_name.argtypes = [ctypes.c_int]
        L.eqat_profile_stop.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64), ctypes.c_int]
        _lib = L
    return _lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _tdt(code: int):
    return torch.bfloat16 if code == BF16 else torch.float32


def _p(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("eqat tensors must be contiguous device tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(fn, status):
    if status != 0:
        raise EqatError(fn, status)


def make_desc(T, I, O, bits, group, act_dtype, w_dtype) -> Desc:
    return Desc(int(T), int(I), int(O), int(bits), int(group), int(act_dtype), int(w_dtype))


def workspace(desc: Desc, op: int, device) -> torch.Tensor | None:
    n = lib().eqat_workspace_bytes(ctypes.byref(desc), op)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def _groups(I, group):
    return 1 if group == -1 else I // group


def eqat_init_minmax(W, bits, group, s=None, z=None):
    O, I = W.shape
    d = make_desc(0, I, O, bits, group, BF16, _dt(W))
    G = _groups(I, group)
    s = torch.empty((O, G), dtype=torch.float32, device=W.device) if s is None else s
    z = torch.empty((O, G), dtype=torch.float32, device=W.device) if z is None else z
    _check("eqat_init_minmax", lib().eqat_init_minmax(ctypes.byref(d), _p(W), _p(s), _p(z), _stream()))
    return s, z


class Batch:
    """Host arrays of device pointers (and the descriptors) for the *_batched entry points; build once, call often."""

    def __init__(self, descs, **tensor_lists):
        self.n = len(descs)
        self.descs = (Desc * self.n)(*descs)
        self.keep = tensor_lists                     # the tensors must outlive the pointer arrays
        self.ptr = {k: (ctypes.c_void_p * self.n)(*[t.data_ptr() for t in v]) for k, v in tensor_lists.items()}
        if "ws" in tensor_lists:
            self.ws_bytes = (ctypes.c_size_t * self.n)(*[t.numel() for t in tensor_lists["ws"]])


def eqat_init_minmax_batched(b: Batch):
    """b: Batch(descs, W=[...], s=[...], z=[...])"""
    _check("eqat_init_minmax_batched", lib().eqat_init_minmax_batched(b.n, b.descs, b.ptr["W"], b.ptr["s"], b.ptr["z"], _stream()))


def eqat_pack_batched(b: Batch):
    """b: Batch(descs, W=, s=, z=, Wpacked=, zpacked=)"""
    _check("eqat_pack_batched", lib().eqat_pack_batched(b.n, b.descs, b.ptr["W"], b.ptr["s"], b.ptr["z"], b.ptr["Wpacked"],
                                                        b.ptr["zpacked"], _stream()))


def eqat_fq_quantize_batched(b: Batch):
    """b: Batch(descs, W=, s=, z=, ws=): Eq.(1) of every linear in one launch, kept in its workspace (EQAT_OP_FQ_BWD size)."""
    _check("eqat_fq_quantize_batched", lib().eqat_fq_quantize_batched(b.n, b.descs, b.ptr["W"], b.ptr["s"], b.ptr["z"],
                                                                      b.ptr["ws"], b.ws_bytes, _stream()))


def eqat_fq_linear_fwd(X, W, s, z, bits, group, Y=None, ws=None, keep=False, kept=False):
    """keep=True: `ws` (EQAT_OP_FQ_BWD size, must then be given) is left holding what eqat_fq_linear_bwd(kept=True) needs.
    kept=True: `ws` already holds that (from keep=True or eqat_fq_quantize_batched) and Eq.(1) is not run again."""
    T, I = X.shape
    O = W.shape[0]
    d = make_desc(T, I, O, bits, group, _dt(X), _dt(W))
    Y = torch.empty((T, O), dtype=X.dtype, device=X.device) if Y is None else Y
    if (keep or kept) and ws is None:
        raise ValueError("keep / kept need the caller's workspace (it is the thing that is kept)")
    ws = workspace(d, OP_FQ_FWD, X.device) if ws is None else ws
    name = "eqat_fq_linear_fwd_kept" if kept else "eqat_fq_linear_fwd_keep" if keep else "eqat_fq_linear_fwd"
    _check(name, getattr(lib(), name)(ctypes.byref(d), _p(X), _p(W), _p(s), _p(z), _p(Y), _p(ws), ws.numel(), _stream()))
    return Y


def eqat_fq_linear_bwd(X, W, s, z, dY, bits, group, want=("dX", "dW", "ds", "dz"), out=None, ws=None, kept=False):
    T, O = dY.shape
    I = W.shape[1]
    d = make_desc(T, I, O, bits, group, _dt(dY), _dt(W))
    G = _groups(I, group)
    out = {} if out is None else out
    if "dX" in want and "dX" not in out: out["dX"] = torch.empty((T, I), dtype=dY.dtype, device=dY.device)
    if "dW" in want and "dW" not in out: out["dW"] = torch.empty((O, I), dtype=W.dtype, device=dY.device)
    if "ds" in want and "ds" not in out: out["ds"] = torch.empty((O, G), dtype=torch.float32, device=dY.device)
    if "dz" in want and "dz" not in out: out["dz"] = torch.empty((O, G), dtype=torch.float32, device=dY.device)
    if kept and ws is None:
        raise ValueError("kept=True needs the workspace the forward call left")
    ws = workspace(d, OP_FQ_BWD, dY.device) if ws is None else ws
    name = "eqat_fq_linear_bwd_kept" if kept else "eqat_fq_linear_bwd"
    _check(name, getattr(lib(), name)(
        ctypes.byref(d), _p(X), _p(W), _p(s), _p(z), _p(dY), _p(out.get("dX")), _p(out.get("dW")), _p(out.get("ds")),
        _p(out.get("dz")), _p(ws), ws.numel(), _stream()))
    return out


def eqat_pack(W, s, z, bits, group, Wpacked=None, zpacked=None):
    O, I = W.shape
    d = make_desc(0, I, O, bits, group, BF16, _dt(W))
    nw, nz = lib().eqat_packed_w_bytes(ctypes.byref(d)), lib().eqat_packed_z_bytes(ctypes.byref(d))
    if nw == 0:
        _check("eqat_pack", lib().eqat_validate_desc(ctypes.byref(d)) or 2)
    Wpacked = torch.empty((O, nw // O), dtype=torch.uint8, device=W.device) if Wpacked is None else Wpacked
    zpacked = torch.empty((O, nz // O), dtype=torch.uint8, device=W.device) if zpacked is None else zpacked
    _check("eqat_pack", lib().eqat_pack(ctypes.byref(d), _p(W), _p(s), _p(z), _p(Wpacked), _p(zpacked), _stream()))
    return Wpacked, zpacked


def eqat_unpack(Wpacked, zpacked, in_features, bits, group):
    O, I = Wpacked.shape[0], int(in_features)
    d = make_desc(0, I, O, bits, group, BF16, BF16)
    codes = torch.empty((O, I), dtype=torch.int32, device=Wpacked.device)
    zc = torch.empty((O, _groups(I, group)), dtype=torch.int32, device=Wpacked.device)
    _check("eqat_unpack", lib().eqat_unpack(ctypes.byref(d), _p(Wpacked), _p(zpacked), _p(codes), _p(zc), _stream()))
    return codes, zc


def eqat_qlinear_fwd(X, Wpacked, s, zpacked, bits, group, Y=None, ws=None, keep=False):
    """keep=True: `ws` (EQAT_OP_Q_BWD size, must then be given) is left holding what eqat_qlinear_bwd(kept=True) needs."""
    T, I = X.shape
    O = Wpacked.shape[0]
    d = make_desc(T, I, O, bits, group, _dt(X), BF16)
    Y = torch.empty((T, O), dtype=X.dtype, device=X.device) if Y is None else Y
    if keep and ws is None:
        raise ValueError("keep=True needs the caller's workspace (it is the thing that is kept)")
    ws = workspace(d, OP_Q_FWD, X.device) if ws is None else ws
    name = "eqat_qlinear_fwd_keep" if keep else "eqat_qlinear_fwd"
    _check(name, getattr(lib(), name)(ctypes.byref(d), _p(X), _p(Wpacked), _p(s), _p(zpacked), _p(Y), _p(ws), ws.numel(),
                                      _stream()))
    return Y


def eqat_qlinear_bwd(X, Wpacked, s, zpacked, dY, in_features, bits, group, want=("dX", "ds"), out=None, ws=None,
                     kept=False):
    T, O = dY.shape
    I = int(in_features)
    d = make_desc(T, I, O, bits, group, _dt(dY), BF16)
    out = {} if out is None else out
    if "dX" in want and "dX" not in out: out["dX"] = torch.empty((T, I), dtype=dY.dtype, device=dY.device)
    if "ds" in want and "ds" not in out: out["ds"] = torch.empty((O, _groups(I, group)), dtype=torch.float32, device=dY.device)
    if kept and ws is None:
        raise ValueError("kept=True needs the workspace the forward call left")
    ws = workspace(d, OP_Q_BWD, dY.device) if ws is None else ws
    name = "eqat_qlinear_bwd_kept" if kept else "eqat_qlinear_bwd"
    _check(name, getattr(lib(), name)(ctypes.byref(d), _p(X), _p(Wpacked), _p(s), _p(zpacked), _p(dY),
                                      _p(out.get("dX")), _p(out.get("ds")), _p(ws), ws.numel(), _stream()))
    return out


def eqat_qlinear_fwd_z(X, Wpacked, s, z, bits, group, Y=None, ws=None):
    """E2E-QP forward with floating-point (trained) zero points z [O,G]."""
    T, I = X.shape
    O = Wpacked.shape[0]
    d = make_desc(T, I, O, bits, group, _dt(X), BF16)
    Y = torch.empty((T, O), dtype=X.dtype, device=X.device) if Y is None else Y
    ws = workspace(d, OP_Q_FWD, X.device) if ws is None else ws
    _check("eqat_qlinear_fwd_z", lib().eqat_qlinear_fwd_z(ctypes.byref(d), _p(X), _p(Wpacked), _p(s), _p(z), _p(Y),
                                                          _p(ws), ws.numel(), _stream()))
    return Y


def eqat_qlinear_bwd_z(X, Wpacked, s, z, dY, in_features, bits, group, want=("dX", "ds", "dz"), out=None, ws=None):
    """E2E-QP backward with trained step sizes and zero points: dX, ds, dz."""
    T, O = dY.shape
    I = int(in_features)
    d = make_desc(T, I, O, bits, group, _dt(dY), BF16)
    out = {} if out is None else out
    G = _groups(I, group)
    if "dX" in want and "dX" not in out: out["dX"] = torch.empty((T, I), dtype=dY.dtype, device=dY.device)
    if "ds" in want and "ds" not in out: out["ds"] = torch.empty((O, G), dtype=torch.float32, device=dY.device)
    if "dz" in want and "dz" not in out: out["dz"] = torch.empty((O, G), dtype=torch.float32, device=dY.device)
    ws = workspace(d, OP_Q_BWD, dY.device) if ws is None else ws
    _check("eqat_qlinear_bwd_z", lib().eqat_qlinear_bwd_z(ctypes.byref(d), _p(X), _p(Wpacked), _p(s), _p(z), _p(dY),
                                                          _p(out.get("dX")), _p(out.get("ds")), _p(out.get("dz")),
                                                          _p(ws), ws.numel(), _stream()))
    return out


def eqat_qlinear_prepare(Wpacked, zpacked, in_features, bits, group, act_dtype=BF16, prepared=None):
    """One-time preparation of a packed layer for E2E-QP steps (codes frozen): returns the prepared buffer."""
    O, I = Wpacked.shape[0], int(in_features)
    d = make_desc(0, I, O, bits, group, act_dtype, BF16)
    n = lib().eqat_prepared_bytes(ctypes.byref(d))
    if n == 0:
        _check("eqat_qlinear_prepare", lib().eqat_validate_desc(ctypes.byref(d)) or 2)
    prepared = torch.empty(n, dtype=torch.uint8, device=Wpacked.device) if prepared is None else prepared
    _check("eqat_qlinear_prepare", lib().eqat_qlinear_prepare(ctypes.byref(d), _p(Wpacked), _p(zpacked), _p(prepared),
                                                               prepared.numel(), _stream()))
    return prepared


def eqat_qlinear_fwd_prepared(X, prepared, s, out_features, bits, group, z=None, Y=None, ws=None, keep=False):
    """keep=True: eqat_qlinear_fwd_prepared_keep (ws of OP_QP_BWD size, left holding the (s, z) pairs)."""
    T, I = X.shape
    O = int(out_features)
    d = make_desc(T, I, O, bits, group, _dt(X), BF16)
    Y = torch.empty((T, O), dtype=X.dtype, device=X.device) if Y is None else Y
    ws = workspace(d, OP_QP_BWD if keep else OP_QP_FWD, X.device) if ws is None else ws
    name = "eqat_qlinear_fwd_prepared_keep" if keep else "eqat_qlinear_fwd_prepared"
    _check(name, getattr(lib(), name)(
        ctypes.byref(d), _p(X), _p(prepared), _p(s), _p(z), _p(Y), _p(ws), ws.numel(), _stream()))
    return Y


def eqat_qlinear_bwd_prepared(X, prepared, s, dY, in_features, bits, group, z=None, want=("dX", "ds"), out=None, ws=None,
                              kept=False):
    """kept=True: eqat_qlinear_bwd_prepared_kept (ws as eqat_qlinear_fwd_prepared_keep left it, same s and z)."""
    T, O = dY.shape
    I = int(in_features)
    d = make_desc(T, I, O, bits, group, _dt(dY), BF16)
    out = {} if out is None else out
    G = _groups(I, group)
    if "dX" in want and "dX" not in out: out["dX"] = torch.empty((T, I), dtype=dY.dtype, device=dY.device)
    if "ds" in want and "ds" not in out: out["ds"] = torch.empty((O, G), dtype=torch.float32, device=dY.device)
    if "dz" in want and "dz" not in out: out["dz"] = torch.empty((O, G), dtype=torch.float32, device=dY.device)
    ws = workspace(d, OP_QP_BWD, dY.device) if ws is None else ws
    name = "eqat_qlinear_bwd_prepared_kept" if kept else "eqat_qlinear_bwd_prepared"
    _check(name, getattr(lib(), name)(
        ctypes.byref(d), _p(X), _p(prepared), _p(s), _p(z), _p(dY), _p(out.get("dX")), _p(out.get("ds")), _p(out.get("dz")),
        _p(ws), ws.numel(), _stream()))
    return out


def eqat_unpack_state(kind, state, out_features, in_features, bits, group, want_clamped=False):
    """Test aid: (codes int32 [O,I], clamped uint8 [O,I] or None, zbar float32 [O,G]) of a kept workspace / prepared layer."""
    O, I = int(out_features), int(in_features)
    d = make_desc(0, I, O, bits, group, BF16, BF16)
    codes = torch.empty((O, I), dtype=torch.int32, device=state.device)
    clamped = torch.empty((O, I), dtype=torch.uint8, device=state.device) if want_clamped else None
    zbar = torch.empty((O, _groups(I, group)), dtype=torch.float32, device=state.device)
    _check("eqat_unpack_state", lib().eqat_unpack_state(ctypes.byref(d), int(kind), _p(state), _p(codes), _p(clamped),
                                                        _p(zbar), _stream()))
    return codes, clamped, zbar


def eqat_recon_loss(Y, Yref, want_dY=True, loss=None, dY=None, ws=None):
    """(loss, dY): loss is a 1-element fp32 device tensor, dY has Y's dtype (None if not wanted)."""
    n = Y.numel()
    loss = torch.empty(1, dtype=torch.float32, device=Y.device) if loss is None else loss
    if want_dY and dY is None:
        dY = torch.empty_like(Y)
    if ws is None:
        ws = torch.empty(lib().eqat_recon_loss_workspace_bytes(), dtype=torch.uint8, device=Y.device)
    _check("eqat_recon_loss", lib().eqat_recon_loss(n, _dt(Y), _p(Y), _p(Yref), _p(loss), _p(dY if want_dY else None),
                                                    _p(ws), ws.numel(), _stream()))
    return loss, (dY if want_dY else None)


def eqat_recon_loss_static(Y, Yref, loss, dY=None):
    """eqat_recon_loss without a workspace and without any allocation: the caller passes every output."""
    _check("eqat_recon_loss_static", lib().eqat_recon_loss_static(Y.numel(), _dt(Y), _p(Y), _p(Yref), _p(loss), _p(dY),
                                                                  _stream()))
    return loss, dY


def eqat_block_ap_update(hyper: AdamW, bits, group, W=None, dW=None, mW=None, vW=None, s=None, ds=None, ms=None, vs=None,
                         z=None, dz=None, mz=None, vz=None, shape=None):
    """One AdamW step in place on whichever of W, s, z is given (with its gradient and two fp32 moment tensors).
    `shape` = (O, I) is needed only when W is not given."""
    O, I = W.shape if W is not None else shape
    d = make_desc(0, I, O, bits, group, BF16, _dt(W) if W is not None else F32)
    _check("eqat_block_ap_update", lib().eqat_block_ap_update(
        ctypes.byref(d), ctypes.byref(hyper), _p(W), _p(s), _p(z), _p(dW), _p(ds), _p(dz), _p(mW), _p(vW), _p(ms), _p(vs),
        _p(mz), _p(vz), _stream()))


def eqat_profile_start():
    _check("eqat_profile_start", lib().eqat_profile_start())


def eqat_profile_stop():
    """{kernel class: (total ms, launches)} for every class that ran since eqat_profile_start()."""
    n = lib().eqat_profile_kernels()
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check("eqat_profile_stop", lib().eqat_profile_stop(ms, cnt, n))
    return {lib().eqat_profile_kernel_name(k).decode(): (ms[k], cnt[k]) for k in range(n) if cnt[k]}
