"""ctypes binding of libpard2cat.so: argument marshalling only.

The functions carry the C ABI's names (include/pard2_cat.h).  Tensors are torch CUDA
tensors used purely as device-memory handles; every step of the computation runs in
the library's HIP kernels.  There is no fallback: if the library has not been built,
or a call returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int32, c_int64, c_size_t, c_void_p
from typing import Optional

PARD2_BF16, PARD2_FP32 = 0, 1
PARD2_W_CAT, PARD2_W_DECAY, PARD2_W_UNIFORM = 0, 1, 2
PARD2_RED_MEAN_VALID, PARD2_RED_SUM = 0, 1
PARD2_FLAG_DW_FP32 = 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpard2cat.so")
EXPORTS = ("pard2_cat_validate", "pard2_cat_workspace_bytes", "pard2_status_string", "pard2_cat_abi_version",
           "pard2_cat_weights", "pard2_cat_weights_seq", "pard2_cat_fwd", "pard2_cat_bwd",
           "pard2_cat_kd_workspace_bytes", "pard2_cat_kd_fwd", "pard2_cat_kd_bwd",
           "pard2_inject_fwd", "pard2_inject_bwd",
           "pard2_cat_kernel_timing",
           "pard2_cat_kernel_timing_read")
KERNEL_NAMES = ("fwd_stats_kernel", "dz_kernel", "dh_kernel", "dw_kernel", "kd_stats_kernel", "kd_dz_kernel",
                "inject_fwd_kernel", "inject_dp_kernel")


class Pard2Error(RuntimeError):
    pass


class pard2_cat_desc(ctypes.Structure):
    _fields_ = [("T", c_int32), ("d", c_int32), ("V", c_int32), ("B", c_int32), ("K", c_int32),
                ("dtype", c_int32), ("weight_mode", c_int32), ("reduction", c_int32),
                ("beta", c_float), ("gamma", c_float), ("ignore_index", c_int32), ("flags", c_int32),
                ("ldH", c_int64), ("ldW", c_int64)]


class pard2_kd_teacher(ctypes.Structure):
    _fields_ = [("H", c_void_p), ("W", c_void_p), ("ldH", c_int64), ("ldW", c_int64), ("d", c_int32),
                ("reserved", c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library (once).  Raises if it is missing: there is no CPU path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise Pard2Error(f"{LIB_PATH} not found: build it with `python -m paper_2605_08632_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    D = POINTER(pard2_cat_desc)
    L.pard2_cat_validate.argtypes = [D]
    L.pard2_cat_validate.restype = ctypes.c_int
    L.pard2_cat_workspace_bytes.argtypes = [D]
    L.pard2_cat_workspace_bytes.restype = c_size_t
    L.pard2_status_string.argtypes = [ctypes.c_int]
    L.pard2_status_string.restype = c_char_p
    L.pard2_cat_abi_version.argtypes = []
    L.pard2_cat_abi_version.restype = ctypes.c_int
    L.pard2_cat_weights.argtypes = [D, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.pard2_cat_weights.restype = ctypes.c_int
    L.pard2_cat_weights_seq.argtypes = [D, c_void_p, c_int64] + [c_void_p] * 8
    L.pard2_cat_weights_seq.restype = ctypes.c_int
    L.pard2_cat_fwd.argtypes = [D] + [c_void_p] * 13 + [c_void_p, c_size_t, c_void_p]
    L.pard2_cat_fwd.restype = ctypes.c_int
    L.pard2_cat_bwd.argtypes = [D] + [c_void_p] * 9 + [c_int32, c_void_p, c_size_t, c_void_p]
    L.pard2_cat_bwd.restype = ctypes.c_int
    TE = POINTER(pard2_kd_teacher)
    L.pard2_cat_kd_workspace_bytes.argtypes = [D, c_int32]
    L.pard2_cat_kd_workspace_bytes.restype = c_size_t
    L.pard2_cat_kd_fwd.argtypes = [D, c_void_p, c_void_p, TE] + [c_void_p] * 13 + [c_void_p, c_size_t, c_void_p]
    L.pard2_cat_kd_fwd.restype = ctypes.c_int
    L.pard2_cat_kd_bwd.argtypes = ([D, c_void_p, c_void_p, TE] + [c_void_p] * 8 + [c_int32] + [c_void_p] * 3 +
                                   [c_void_p, c_size_t, c_void_p])
    L.pard2_cat_kd_bwd.restype = ctypes.c_int
    L.pard2_inject_fwd.argtypes = [c_int32] * 4 + [c_void_p, POINTER(c_void_p), c_int64, c_void_p, c_void_p, c_void_p,
                                                 c_void_p]
    L.pard2_inject_fwd.restype = ctypes.c_int
    L.pard2_inject_bwd.argtypes = [c_int32] * 4 + [c_void_p, POINTER(c_void_p), c_int64, c_void_p, c_void_p, c_void_p,
                                                 c_int32, c_void_p]
    L.pard2_inject_bwd.restype = ctypes.c_int
    L.pard2_cat_kernel_timing.argtypes = [ctypes.c_int]
    L.pard2_cat_kernel_timing.restype = ctypes.c_int
    L.pard2_cat_kernel_timing_read.argtypes = [ctypes.c_int, POINTER(ctypes.c_double), POINTER(c_int64)]
    L.pard2_cat_kernel_timing_read.restype = ctypes.c_int
    _lib = L
    return L


def pard2_cat_kernel_timing(enable: bool) -> None:
    _check(lib().pard2_cat_kernel_timing(1 if enable else 0), "pard2_cat_kernel_timing")


def pard2_cat_kernel_timing_read(kernel: int):
    """(total milliseconds, launch count) of the recorded launches of one contraction kernel."""
    ms, n = ctypes.c_double(0), c_int64(0)
    _check(lib().pard2_cat_kernel_timing_read(kernel, ctypes.byref(ms), ctypes.byref(n)),
           "pard2_cat_kernel_timing_read")
    return ms.value, n.value


def _check(status: int, what: str) -> None:
    if status != 0:
        raise Pard2Error(f"{what} failed: {lib().pard2_status_string(status).decode()} ({status})")


def make_desc(T, d, V, B, K, dtype, weight_mode=PARD2_W_CAT, reduction=PARD2_RED_MEAN_VALID, beta=0.1,
              gamma=1.0, ignore_index=-100, ldH=None, ldW=None, flags=0) -> pard2_cat_desc:
    return pard2_cat_desc(T, d, V, B, K, dtype, weight_mode, reduction, beta, gamma, ignore_index, flags,
                          d if ldH is None else ldH, d if ldW is None else ldW)


def pard2_cat_validate(desc: pard2_cat_desc) -> int:
    return lib().pard2_cat_validate(ctypes.byref(desc))


def pard2_cat_workspace_bytes(desc: pard2_cat_desc) -> int:
    return lib().pard2_cat_workspace_bytes(ctypes.byref(desc))


def pard2_status_string(status: int) -> str:
    return lib().pard2_status_string(status).decode()


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _torch_dtype(desc):
    import torch
    return torch.bfloat16 if desc.dtype == PARD2_BF16 else torch.float32


def _check_tensor(t, name, dtype, numel_min, device):
    if t is None:
        return
    if not t.is_cuda or t.device != device:
        raise Pard2Error(f"{name} must live on {device}")
    if t.dtype != dtype:
        raise Pard2Error(f"{name} must be {dtype}, got {t.dtype}")
    if t.numel() < numel_min:
        raise Pard2Error(f"{name} has {t.numel()} elements, needs {numel_min}")
    if not t.is_contiguous() and name not in ("H", "W"):
        raise Pard2Error(f"{name} must be contiguous")


def alloc_workspace(desc: pard2_cat_desc, device):
    import torch
    n = pard2_cat_workspace_bytes(desc)
    if n == 0:
        _check(pard2_cat_validate(desc), "pard2_cat_validate")
    return torch.empty(n + 256, dtype=torch.uint8, device=device)


def _ws_args(ws):
    base = ws.data_ptr()
    aligned = (base + 255) // 256 * 256
    return aligned, ws.numel() - (aligned - base)


def pard2_cat_weights(desc, conf, y=None, valid_len=None, w=None, exp_len=None):
    """CAT weights (Eq.10) from given confidences.  Returns (w, exp_len)."""
    import torch
    dev = conf.device
    _check_tensor(conf, "conf", torch.float32, desc.T, dev)
    _check_tensor(y, "y", torch.int32, desc.T, dev)
    _check_tensor(valid_len, "valid_len", torch.int32, desc.B, dev)
    w = torch.empty(desc.T, dtype=torch.float32, device=dev) if w is None else w
    exp_len = torch.empty(desc.B, dtype=torch.float32, device=dev) if exp_len is None else exp_len
    _check_tensor(w, "w", torch.float32, desc.T, dev)
    _check_tensor(exp_len, "exp_len", torch.float32, desc.B, dev)
    rc = lib().pard2_cat_weights(ctypes.byref(desc), _ptr(conf), _ptr(y), _ptr(valid_len), _ptr(w), _ptr(exp_len),
                                 _stream())
    _check(rc, "pard2_cat_weights")
    return w, exp_len


def pard2_cat_weights_seq(desc, c_seq, anchor_pos, seq_end, y=None):
    """CAT weights gathered from per-position teacher confidences (Sec.3.3).
    Returns (w, conf, valid_len, exp_len)."""
    import torch
    dev = c_seq.device
    _check_tensor(c_seq, "c_seq", torch.float32, 1, dev)
    _check_tensor(anchor_pos, "anchor_pos", torch.int32, desc.B, dev)
    _check_tensor(seq_end, "seq_end", torch.int32, desc.B, dev)
    _check_tensor(y, "y", torch.int32, desc.T, dev)
    w = torch.empty(desc.T, dtype=torch.float32, device=dev)
    conf = torch.empty(desc.T, dtype=torch.float32, device=dev)
    valid_len = torch.empty(desc.B, dtype=torch.int32, device=dev)
    exp_len = torch.empty(desc.B, dtype=torch.float32, device=dev)
    rc = lib().pard2_cat_weights_seq(ctypes.byref(desc), _ptr(c_seq), c_seq.numel(), _ptr(anchor_pos), _ptr(seq_end),
                                     _ptr(y), _ptr(w), _ptr(conf), _ptr(valid_len), _ptr(exp_len), _stream())
    _check(rc, "pard2_cat_weights_seq")
    return w, conf, valid_len, exp_len


def pard2_cat_fwd(desc, H, W, y, conf_in=None, valid_len=None, workspace=None, stats_only=False, out=None):
    """Forward.  Returns a dict of device tensors: loss, lse, logp_y, w, argmax, accept_len,
    exp_len, dev_status (loss and w are absent when stats_only)."""
    import torch
    dev = H.device
    td = _torch_dtype(desc)
    _check_tensor(H, "H", td, 0, dev)
    _check_tensor(W, "W", td, 0, dev)
    if H.stride(-1) != 1 or W.stride(-1) != 1 or H.stride(0) != desc.ldH or W.stride(0) != desc.ldW:
        raise Pard2Error("H/W strides do not match the descriptor")
    if tuple(H.shape) != (desc.T, desc.d) or tuple(W.shape) != (desc.V, desc.d):
        raise Pard2Error("H/W shapes do not match the descriptor")
    _check_tensor(y, "y", torch.int32, desc.T, dev)
    _check_tensor(conf_in, "conf_in", torch.float32, desc.T, dev)
    _check_tensor(valid_len, "valid_len", torch.int32, desc.B, dev)
    ws = alloc_workspace(desc, dev) if workspace is None else workspace
    o = {} if out is None else out
    f32 = dict(dtype=torch.float32, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    o.setdefault("lse", torch.empty(desc.T, **f32))
    o.setdefault("logp_y", torch.empty(desc.T, **f32))
    o.setdefault("argmax", torch.empty(desc.T, **i32))
    o.setdefault("accept_len", torch.empty(desc.B, **i32))
    o.setdefault("exp_len", torch.empty(desc.B, **f32))
    o.setdefault("dev_status", torch.empty(1, **i32))
    if not stats_only:
        o.setdefault("loss", torch.empty(1, **f32))
        o.setdefault("w", torch.empty(desc.T, **f32))
    wp, wn = _ws_args(ws)
    rc = lib().pard2_cat_fwd(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(y), _ptr(conf_in), _ptr(valid_len),
                             _ptr(o.get("loss")), _ptr(o["lse"]), _ptr(o["logp_y"]), _ptr(o.get("w")),
                             _ptr(o["argmax"]), _ptr(o["accept_len"]), _ptr(o["exp_len"]), _ptr(o["dev_status"]),
                             wp, wn, _stream())
    _check(rc, "pard2_cat_fwd")
    return o


def pard2_cat_bwd(desc, H, W, y, lse, w, valid_len=None, grad_loss=None, dH=None, dW=None, accumulate_dW=False,
                  workspace=None):
    """Backward.  Returns (dH, dW)."""
    import torch
    dev = H.device
    td = _torch_dtype(desc)
    _check_tensor(H, "H", td, 0, dev)
    _check_tensor(W, "W", td, 0, dev)
    if H.stride(-1) != 1 or W.stride(-1) != 1 or H.stride(0) != desc.ldH or W.stride(0) != desc.ldW:
        raise Pard2Error("H/W strides do not match the descriptor")
    _check_tensor(y, "y", torch.int32, desc.T, dev)
    _check_tensor(lse, "lse", torch.float32, desc.T, dev)
    _check_tensor(w, "w", torch.float32, desc.T, dev)
    _check_tensor(valid_len, "valid_len", torch.int32, desc.B, dev)
    _check_tensor(grad_loss, "grad_loss", torch.float32, 1, dev)
    tdw = torch.float32 if desc.flags & PARD2_FLAG_DW_FP32 else td
    dH = torch.empty(desc.T, desc.d, dtype=td, device=dev) if dH is None else dH
    if dW is None:
        if accumulate_dW:
            raise Pard2Error("accumulate_dW needs an existing dW")
        dW = torch.empty(desc.V, desc.d, dtype=tdw, device=dev)
    _check_tensor(dH, "dH", td, desc.T * desc.d, dev)
    _check_tensor(dW, "dW", tdw, desc.V * desc.d, dev)
    ws = alloc_workspace(desc, dev) if workspace is None else workspace
    wp, wn = _ws_args(ws)
    rc = lib().pard2_cat_bwd(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(y), _ptr(valid_len), _ptr(lse), _ptr(w),
                             _ptr(grad_loss), _ptr(dH), _ptr(dW), 1 if accumulate_dW else 0, wp, wn, _stream())
    _check(rc, "pard2_cat_bwd")
    return dH, dW


# ---------------------------------------------------------------- Eq.12 token loss with the KD term
def pard2_cat_kd_workspace_bytes(desc: pard2_cat_desc, teacher_d: int) -> int:
    return lib().pard2_cat_kd_workspace_bytes(ctypes.byref(desc), teacher_d)


def alloc_kd_workspace(desc: pard2_cat_desc, teacher_d: int, device):
    import torch
    n = pard2_cat_kd_workspace_bytes(desc, teacher_d)
    if n == 0:
        raise Pard2Error("pard2_cat_kd_workspace_bytes: invalid descriptor or teacher width")
    return torch.empty(n + 256, dtype=torch.uint8, device=device)


def _teacher(desc, Ht, Wt, dev):
    td = _torch_dtype(desc)
    _check_tensor(Ht, "H", td, 0, dev)
    _check_tensor(Wt, "W", td, 0, dev)
    if Ht.stride(-1) != 1 or Wt.stride(-1) != 1 or Ht.shape[0] != desc.T or Wt.shape[0] != desc.V or \
            Ht.shape[1] != Wt.shape[1]:
        raise Pard2Error("teacher H/W shapes do not match the descriptor")
    return pard2_kd_teacher(Ht.data_ptr(), Wt.data_ptr(), Ht.stride(0), Wt.stride(0), Ht.shape[1], 0)


def pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y, conf_in=None, valid_len=None, workspace=None, out=None,
                     defer_loss=False):
    """Forward of the weighted (beta CE + KD) loss.  Returns a dict of device tensors: loss, lse,
    lse_t, logp_y, kd, w, argmax, accept_len, exp_len, dev_status.  With defer_loss the cheaper
    forward without loss and kd runs (ask pard2_cat_kd_bwd for them)."""
    import torch
    dev = H.device
    td = _torch_dtype(desc)
    _check_tensor(H, "H", td, 0, dev)
    _check_tensor(W, "W", td, 0, dev)
    if H.stride(-1) != 1 or W.stride(-1) != 1 or H.stride(0) != desc.ldH or W.stride(0) != desc.ldW:
        raise Pard2Error("H/W strides do not match the descriptor")
    if tuple(H.shape) != (desc.T, desc.d) or tuple(W.shape) != (desc.V, desc.d):
        raise Pard2Error("H/W shapes do not match the descriptor")
    te = _teacher(desc, Ht, Wt, dev)
    _check_tensor(y, "y", torch.int32, desc.T, dev)
    _check_tensor(conf_in, "conf_in", torch.float32, desc.T, dev)
    _check_tensor(valid_len, "valid_len", torch.int32, desc.B, dev)
    ws = alloc_kd_workspace(desc, te.d, dev) if workspace is None else workspace
    o = {} if out is None else out
    f32 = dict(dtype=torch.float32, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    for k in ("lse", "lse_t", "logp_y", "w") + (() if defer_loss else ("kd",)):
        o.setdefault(k, torch.empty(desc.T, **f32))
    if not defer_loss:
        o.setdefault("loss", torch.empty(1, **f32))
    o.setdefault("argmax", torch.empty(desc.T, **i32))
    o.setdefault("accept_len", torch.empty(desc.B, **i32))
    o.setdefault("exp_len", torch.empty(desc.B, **f32))
    o.setdefault("dev_status", torch.empty(1, **i32))
    wp, wn = _ws_args(ws)
    rc = lib().pard2_cat_kd_fwd(ctypes.byref(desc), _ptr(H), _ptr(W), ctypes.byref(te), _ptr(y), _ptr(conf_in),
                                _ptr(valid_len), None if defer_loss else _ptr(o["loss"]), _ptr(o["lse"]),
                                _ptr(o["lse_t"]), _ptr(o["logp_y"]), None if defer_loss else _ptr(o["kd"]), _ptr(o["w"]), _ptr(o["argmax"]), _ptr(o["accept_len"]),
                                _ptr(o["exp_len"]), _ptr(o["dev_status"]), wp, wn, _stream())
    _check(rc, "pard2_cat_kd_fwd")
    return o


def pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, lse, lse_t, w, valid_len=None, grad_loss=None, dH=None, dW=None,
                     accumulate_dW=False, workspace=None, logp_y=None, kd=None, loss=None):
    """Backward of pard2_cat_kd_fwd's loss into the draft's H and W.  Returns (dH, dW).  Optional
    outputs kd [T] and loss [1] (loss needs logp_y) receive the step's KL and loss."""
    import torch
    dev = H.device
    td = _torch_dtype(desc)
    _check_tensor(H, "H", td, 0, dev)
    _check_tensor(W, "W", td, 0, dev)
    if H.stride(-1) != 1 or W.stride(-1) != 1 or H.stride(0) != desc.ldH or W.stride(0) != desc.ldW:
        raise Pard2Error("H/W strides do not match the descriptor")
    te = _teacher(desc, Ht, Wt, dev)
    _check_tensor(y, "y", torch.int32, desc.T, dev)
    for name, t in (("lse", lse), ("lse_t", lse_t), ("w", w), ("logp_y", logp_y), ("kd", kd)):
        _check_tensor(t, name, torch.float32, desc.T, dev)
    _check_tensor(loss, "loss", torch.float32, 1, dev)
    _check_tensor(valid_len, "valid_len", torch.int32, desc.B, dev)
    _check_tensor(grad_loss, "grad_loss", torch.float32, 1, dev)
    tdw = torch.float32 if desc.flags & PARD2_FLAG_DW_FP32 else td
    dH = torch.empty(desc.T, desc.d, dtype=td, device=dev) if dH is None else dH
    if dW is None:
        if accumulate_dW:
            raise Pard2Error("accumulate_dW needs an existing dW")
        dW = torch.empty(desc.V, desc.d, dtype=tdw, device=dev)
    _check_tensor(dH, "dH", td, desc.T * desc.d, dev)
    _check_tensor(dW, "dW", tdw, desc.V * desc.d, dev)
    ws = alloc_kd_workspace(desc, te.d, dev) if workspace is None else workspace
    wp, wn = _ws_args(ws)
    rc = lib().pard2_cat_kd_bwd(ctypes.byref(desc), _ptr(H), _ptr(W), ctypes.byref(te), _ptr(y), _ptr(valid_len),
                                _ptr(lse), _ptr(lse_t), _ptr(w), _ptr(grad_loss), _ptr(dH), _ptr(dW),
                                1 if accumulate_dW else 0, _ptr(logp_y), _ptr(kd), _ptr(loss), wp, wn, _stream())
    _check(rc, "pard2_cat_kd_bwd")
    return dH, dW


# ---------------------------------------------------------------- gated target-feature injection (Sec.3.3)
def _inject_args(feats, d, dev):
    import torch
    F = len(feats)
    if not 1 <= F <= 8:
        raise Pard2Error("1..8 target features")
    T, dt = feats[0].shape
    for f in feats:
        _check_tensor(f, "H", torch.bfloat16, 0, dev)      # name "H": a strided 2-D operand
        if tuple(f.shape) != (T, dt) or f.stride(1) != 1 or f.stride(0) != feats[0].stride(0):
            raise Pard2Error("target features must share shape [T, dt] and row stride")
    arr = (c_void_p * F)(*[f.data_ptr() for f in feats])
    return T, dt, F, arr, feats[0].stride(0)


def pard2_inject_fwd(E, feats, P, xi, Eout=None):
    """e' = e + xi * Proj([x_1; ...; x_F]).  Returns Eout [T, d] bf16."""
    import torch
    dev = E.device
    d = E.shape[1]
    T, dt, F, arr, ldX = _inject_args(feats, d, dev)
    _check_tensor(E, "E", torch.bfloat16, T * d, dev)
    _check_tensor(P, "P", torch.bfloat16, d * F * dt, dev)
    _check_tensor(xi, "xi", torch.float32, T, dev)
    if tuple(E.shape) != (T, d) or tuple(P.shape) != (d, F * dt):
        raise Pard2Error("E must be [T, d] and P [d, F*dt]")
    Eout = torch.empty_like(E) if Eout is None else Eout
    _check_tensor(Eout, "Eout", torch.bfloat16, T * d, dev)
    rc = lib().pard2_inject_fwd(T, d, dt, F, _ptr(E), arr, ldX, _ptr(P), _ptr(xi), _ptr(Eout), _stream())
    _check(rc, "pard2_inject_fwd")
    return Eout


def pard2_inject_bwd(dEout, feats, xi, dP=None, accumulate_dP=False):
    """Returns (dT [T, d] = xi * dEout, dP [d, F*dt]); the gradient of e is dEout itself."""
    import torch
    dev = dEout.device
    d = dEout.shape[1]
    T, dt, F, arr, ldX = _inject_args(feats, d, dev)
    _check_tensor(dEout, "dEout", torch.bfloat16, T * d, dev)
    _check_tensor(xi, "xi", torch.float32, T, dev)
    dT = torch.empty(T, d, dtype=torch.bfloat16, device=dev)
    if dP is None:
        if accumulate_dP:
            raise Pard2Error("accumulate_dP needs an existing dP")
        dP = torch.empty(d, F * dt, dtype=torch.bfloat16, device=dev)
    _check_tensor(dP, "dP", torch.bfloat16, d * F * dt, dev)
    rc = lib().pard2_inject_bwd(T, d, dt, F, _ptr(dEout), arr, ldX, _ptr(xi), _ptr(dT), _ptr(dP),
                                1 if accumulate_dP else 0, _stream())
    _check(rc, "pard2_inject_bwd")
    return dT, dP
