"""ctypes binding of libsasq.so: one Python function per C entry point of include/sasq.h.

Only argument marshalling happens here (device pointers, sizes, the current HIP stream taken
from PyTorch); every step of the path runs in the library's kernels.  Tensors must be device
tensors, contiguous, of the dtypes the header states.  A non-zero status raises SasqError.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsasq.so")

SASQ_F16, SASQ_BF16 = 0, 1
SASQ_W_INT8, SASQ_W_INT4_PACKED, SASQ_W_INT8_BLOCKED, SASQ_W_INT4_BLOCKED = 0, 1, 2, 3

SASQ_MAX_BATCH = 8

_DT = {torch.float16: SASQ_F16, torch.bfloat16: SASQ_BF16}


class _LinItem(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("s", ctypes.c_void_p), ("wq", ctypes.c_void_p), ("s_w", ctypes.c_void_p),
                ("bias", ctypes.c_void_p), ("y", ctypes.c_void_p), ("M", ctypes.c_int64), ("N", ctypes.c_int64),
                ("K", ctypes.c_int64)]


class _FqItem(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("dy", ctypes.c_void_p), ("s", ctypes.c_void_p), ("out", ctypes.c_void_p),
                ("ds", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64)]


class SasqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().sasq_status_string(status).decode() if _LIB is not None else str(status)
        super().__init__(f"{where}: {msg}")


_LIB = None


def _lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2512_14481_amd.build` "
                "(there is no CPU fallback for the SASQ kernels)")
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, sz, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
        L.sasq_status_string.restype = ctypes.c_char_p
        L.sasq_status_string.argtypes = [i32]
        L.sasq_version.restype = i32
        L.sasq_set_tuning.argtypes = [i32, i32]
        L.sasq_workspace_init.argtypes = [vp, sz, vp]
        L.sasq_fakequant_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp]
        L.sasq_fakequant_bwd_workspace.restype = sz
        L.sasq_fakequant_bwd_workspace.argtypes = [i64, i64]
        L.sasq_fakequant_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, sz, vp]
        L.sasq_fakequant_bwd_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, vp]
        L.sasq_scale_sgd.argtypes = [vp, vp, f32, vp]
        L.sasq_scale_sgd_vec.argtypes = [vp, vp, i64, f32, vp]
        L.sasq_fakequant_fwd_batch.argtypes = [ctypes.POINTER(_FqItem), i32, i32, i32, vp]
        L.sasq_fakequant_bwd_batch_workspace.restype = sz
        L.sasq_fakequant_bwd_batch_workspace.argtypes = [i32]
        L.sasq_fakequant_bwd_batch.argtypes = [ctypes.POINTER(_FqItem), i32, i32, i32, vp, sz, vp]
        L.sasq_fakequant_fwd_pc_batch.argtypes = [ctypes.POINTER(_FqItem), i32, i32, i32, vp]
        L.sasq_fakequant_bwd_pc_batch_workspace.restype = sz
        L.sasq_fakequant_bwd_pc_batch_workspace.argtypes = [ctypes.POINTER(_FqItem), i32]
        L.sasq_fakequant_bwd_pc_batch.argtypes = [ctypes.POINTER(_FqItem), i32, i32, i32, vp, sz, vp]
        L.sasq_scale_adamw.argtypes = [vp, vp, vp, vp, i64, i64] + [ctypes.c_double] * 5 + [vp]
        L.sasq_fakequant_fwd_pc.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp]
        L.sasq_fakequant_bwd_pc_workspace.restype = sz
        L.sasq_fakequant_bwd_pc_workspace.argtypes = [i64, i64]
        L.sasq_fakequant_bwd_pc.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, sz, vp]
        L.sasq_static_linear_workspace.restype = sz
        L.sasq_static_linear_workspace.argtypes = [i64, i64, i64, i32]
        L.sasq_static_linear.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, vp, sz, vp]
        L.sasq_static_linear_grouped.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, i32, i32, vp, sz, vp]
        L.sasq_dynamic_linear_workspace.restype = sz
        L.sasq_dynamic_linear_workspace.argtypes = [i64, i64, i64, i32]
        L.sasq_dynamic_linear.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, vp, sz, vp]
        L.sasq_static_linear_batch_workspace.restype = sz
        L.sasq_static_linear_batch_workspace.argtypes = [ctypes.POINTER(_LinItem), i32, i32]
        L.sasq_static_linear_batch.argtypes = [ctypes.POINTER(_LinItem), i32, i32, i32, i32, vp, sz, vp]
        L.sasq_quantize_weight.argtypes = [vp, vp, vp, i64, i64, i32, vp]
        L.sasq_packed_weight_bytes.restype = sz
        L.sasq_packed_weight_bytes.argtypes = [i64, i64, i32]
        L.sasq_pack_weight.argtypes = [vp, vp, i64, i64, i32, vp]
        L.sasq_bwd_weight_bytes.restype = sz
        L.sasq_bwd_weight_bytes.argtypes = [i64, i64]
        L.sasq_prepare_bwd_weight.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp]
        L.sasq_linear_bwd_input.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp]
        L.sasq_absmax_scale_workspace.restype = sz
        L.sasq_absmax_scale_workspace.argtypes = [i64, i64]
        L.sasq_absmax_scale.argtypes = [vp, vp, i64, i64, i32, i32, vp, sz, vp]
        _LIB = L
    return _LIB


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("SASQ entry points take device tensors")
    if not t.is_contiguous():
        raise ValueError("SASQ entry points take contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise SasqError(rc, where)


def _want(t: Optional[torch.Tensor], dtype, name: str):
    if t is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")


def _dt(t: torch.Tensor) -> int:
    if t.dtype not in _DT:
        raise TypeError(f"activation dtype must be float16 or bfloat16, got {t.dtype}")
    return _DT[t.dtype]


def sasq_version() -> int:
    return int(_lib().sasq_version())


SASQ_TUNE_LINEAR_PATH, SASQ_TUNE_LINEAR_TILE, SASQ_TUNE_LINEAR_MFMA, SASQ_TUNE_FQ_SHARE, SASQ_TUNE_BWD_TILE = range(5)


def sasq_set_tuning(knob: int, value: int) -> None:
    _check(_lib().sasq_set_tuning(knob, value), "sasq_set_tuning")


def sasq_workspace_init(workspace: torch.Tensor) -> None:
    _check(_lib().sasq_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "sasq_workspace_init")


def new_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Allocate (with PyTorch) and initialise a workspace of at least nbytes."""
    ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    sasq_workspace_init(ws)
    return ws


def sasq_fakequant_fwd(x: torch.Tensor, s: torch.Tensor, y: torch.Tensor,
                       codes: Optional[torch.Tensor] = None, bits: int = 8) -> None:
    _want(s, torch.float32, "s"); _want(codes, torch.int8, "codes")
    if y.dtype != x.dtype or y.shape != x.shape:
        raise ValueError("y must match x")
    rows, cols = (x.shape[0], x.numel() // max(x.shape[0], 1)) if x.dim() >= 1 else (1, 1)
    _check(_lib().sasq_fakequant_fwd(_ptr(x), _ptr(s), _ptr(y), _ptr(codes), rows, cols, bits, _dt(x), _stream()),
           "sasq_fakequant_fwd")


def sasq_fakequant_bwd_workspace(rows: int, cols: int) -> int:
    return int(_lib().sasq_fakequant_bwd_workspace(rows, cols))


def sasq_fakequant_bwd(x: torch.Tensor, dy: torch.Tensor, s: torch.Tensor, dx: Optional[torch.Tensor],
                       ds: torch.Tensor, workspace: torch.Tensor, bits: int = 8) -> None:
    _want(s, torch.float32, "s"); _want(ds, torch.float32, "ds")
    if dy.dtype != x.dtype or dy.shape != x.shape or (dx is not None and (dx.dtype != x.dtype or dx.shape != x.shape)):
        raise ValueError("dy and dx must match x")
    rows, cols = x.shape[0], x.numel() // max(x.shape[0], 1)
    _check(_lib().sasq_fakequant_bwd(_ptr(x), _ptr(dy), _ptr(s), _ptr(dx), _ptr(ds), rows, cols, bits, _dt(x),
                                     _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "sasq_fakequant_bwd")


def sasq_fakequant_bwd_static(x: torch.Tensor, dy: torch.Tensor, s: torch.Tensor, dx: Optional[torch.Tensor],
                              ds: torch.Tensor, bits: int = 8) -> None:
    _want(s, torch.float32, "s"); _want(ds, torch.float32, "ds")
    if dy.dtype != x.dtype or dy.shape != x.shape or (dx is not None and (dx.dtype != x.dtype or dx.shape != x.shape)):
        raise ValueError("dy and dx must match x")
    rows, cols = x.shape[0], x.numel() // max(x.shape[0], 1)
    _check(_lib().sasq_fakequant_bwd_static(_ptr(x), _ptr(dy), _ptr(s), _ptr(dx), _ptr(ds), rows, cols, bits, _dt(x),
                                            _stream()), "sasq_fakequant_bwd_static")


def sasq_fakequant_fwd_pc(x: torch.Tensor, s: torch.Tensor, y: torch.Tensor,
                          codes: Optional[torch.Tensor] = None, bits: int = 8) -> None:
    _want(s, torch.float32, "s"); _want(codes, torch.int8, "codes")
    rows, cols = x.shape
    if y.dtype != x.dtype or y.shape != x.shape or s.numel() != cols:
        raise ValueError("y must match x and s must have one element per column")
    _check(_lib().sasq_fakequant_fwd_pc(_ptr(x), _ptr(s), _ptr(y), _ptr(codes), rows, cols, bits, _dt(x), _stream()),
           "sasq_fakequant_fwd_pc")


def sasq_fakequant_bwd_pc_workspace(rows: int, cols: int) -> int:
    return int(_lib().sasq_fakequant_bwd_pc_workspace(rows, cols))


def sasq_fakequant_bwd_pc(x: torch.Tensor, dy: torch.Tensor, s: torch.Tensor, dx: Optional[torch.Tensor],
                          ds: torch.Tensor, workspace: Optional[torch.Tensor], bits: int = 8) -> None:
    _want(s, torch.float32, "s"); _want(ds, torch.float32, "ds")
    rows, cols = x.shape
    if dy.dtype != x.dtype or dy.shape != x.shape or (dx is not None and (dx.dtype != x.dtype or dx.shape != x.shape)):
        raise ValueError("dy and dx must match x")
    if s.numel() != cols or ds.numel() != cols:
        raise ValueError("s and ds must have one element per column")
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib().sasq_fakequant_bwd_pc(_ptr(x), _ptr(dy), _ptr(s), _ptr(dx), _ptr(ds), rows, cols, bits, _dt(x),
                                        _ptr(workspace), wsb, _stream()), "sasq_fakequant_bwd_pc")


def _fq_items(items, backward: bool):
    """items: sequence of (x, s, y) for the forward or (x, dy, s, dx_or_None, ds) for the backward."""
    if not 1 <= len(items) <= SASQ_MAX_BATCH:
        raise ValueError(f"a batch holds 1..{SASQ_MAX_BATCH} tensors")
    arr = (_FqItem * len(items))()
    dt = None
    for i, it in enumerate(items):
        if backward:
            x, dy, s, dx, ds = it
            if dy.dtype != x.dtype or dy.shape != x.shape or (dx is not None and (dx.dtype != x.dtype or dx.shape != x.shape)):
                raise ValueError("dy and dx must match x")
            _want(ds, torch.float32, "ds")
            arr[i].dy, arr[i].out, arr[i].ds = _ptr(dy).value, (None if dx is None else _ptr(dx).value), _ptr(ds).value
        else:
            x, s, y = it
            if y.dtype != x.dtype or y.shape != x.shape:
                raise ValueError("y must match x")
            arr[i].out = _ptr(y).value
        _want(s, torch.float32, "s")
        if dt is None:
            dt = _dt(x)
        elif _dt(x) != dt:
            raise TypeError("all tensors of a batch must have the same dtype")
        arr[i].x, arr[i].s = _ptr(x).value, _ptr(s).value
        arr[i].rows, arr[i].cols = x.shape[0], x.numel() // max(x.shape[0], 1)
    return arr, dt


def sasq_fakequant_fwd_batch(items, bits: int = 8) -> None:
    arr, dt = _fq_items(items, False)
    _check(_lib().sasq_fakequant_fwd_batch(arr, len(items), bits, dt, _stream()), "sasq_fakequant_fwd_batch")


def sasq_fakequant_bwd_batch_workspace(count: int) -> int:
    return int(_lib().sasq_fakequant_bwd_batch_workspace(count))


def sasq_fakequant_bwd_batch(items, workspace: torch.Tensor, bits: int = 8) -> None:
    arr, dt = _fq_items(items, True)
    _check(_lib().sasq_fakequant_bwd_batch(arr, len(items), bits, dt, _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()),
           "sasq_fakequant_bwd_batch")


def _pc_check(items, backward: bool) -> None:
    for it in items:
        x, s = it[0], (it[2] if backward else it[1])
        if s.numel() != x.shape[1] or (backward and it[4].numel() != x.shape[1]):
            raise ValueError("per-channel s and ds hold one element per column of x")


def sasq_fakequant_fwd_pc_batch(items, bits: int = 8) -> None:
    """items: sequence of (x, s[cols], y)."""
    _pc_check(items, False)
    arr, dt = _fq_items(items, False)
    _check(_lib().sasq_fakequant_fwd_pc_batch(arr, len(items), bits, dt, _stream()), "sasq_fakequant_fwd_pc_batch")


def sasq_fakequant_bwd_pc_batch_workspace(items) -> int:
    """items as for sasq_fakequant_bwd_pc_batch (only the shapes are read)."""
    arr, _ = _fq_items(items, True)
    return int(_lib().sasq_fakequant_bwd_pc_batch_workspace(arr, len(items)))


def sasq_fakequant_bwd_pc_batch(items, workspace: torch.Tensor, bits: int = 8) -> None:
    """items: sequence of (x, dy, s[cols], dx_or_None, ds[cols])."""
    _pc_check(items, True)
    arr, dt = _fq_items(items, True)
    _check(_lib().sasq_fakequant_bwd_pc_batch(arr, len(items), bits, dt, _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream()),
           "sasq_fakequant_bwd_pc_batch")


def sasq_scale_sgd_vec(s: torch.Tensor, ds: torch.Tensor, lr: float) -> None:
    _want(s, torch.float32, "s"); _want(ds, torch.float32, "ds")
    if s.numel() != ds.numel():
        raise ValueError("s and ds must have the same length")
    _check(_lib().sasq_scale_sgd_vec(_ptr(s), _ptr(ds), s.numel(), ctypes.c_float(lr), _stream()), "sasq_scale_sgd_vec")


def sasq_scale_sgd(s: torch.Tensor, ds: torch.Tensor, lr: float) -> None:
    _want(s, torch.float32, "s"); _want(ds, torch.float32, "ds")
    _check(_lib().sasq_scale_sgd(_ptr(s), _ptr(ds), ctypes.c_float(lr), _stream()), "sasq_scale_sgd")


def sasq_scale_adamw(s: torch.Tensor, ds: torch.Tensor, m: torch.Tensor, v: torch.Tensor, step: int, lr: float,
                     beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01) -> None:
    for t_, n_ in ((s, "s"), (ds, "ds"), (m, "m"), (v, "v")):
        _want(t_, torch.float32, n_)
    if not (s.numel() == ds.numel() == m.numel() == v.numel()):
        raise ValueError("s, ds, m, v must have the same length")
    f = ctypes.c_double
    _check(_lib().sasq_scale_adamw(_ptr(s), _ptr(ds), _ptr(m), _ptr(v), s.numel(), int(step), f(lr), f(beta1),
                                   f(beta2), f(eps), f(weight_decay), _stream()), "sasq_scale_adamw")


def sasq_static_linear_workspace(M: int, N: int, K: int, wf: int) -> int:
    return int(_lib().sasq_static_linear_workspace(M, N, K, wf))


def sasq_static_linear(x: torch.Tensor, s: torch.Tensor, wq: torch.Tensor, s_w: torch.Tensor,
                       bias: Optional[torch.Tensor], y: torch.Tensor, wf: int = SASQ_W_INT8,
                       workspace: Optional[torch.Tensor] = None, acc_out: Optional[torch.Tensor] = None,
                       xq_out: Optional[torch.Tensor] = None, a_bits: int = 8) -> None:
    _want(s, torch.float32, "s"); _want(s_w, torch.float32, "s_w"); _want(bias, torch.float32, "bias")
    _want(acc_out, torch.int32, "acc_out"); _want(xq_out, torch.int8, "xq_out")
    if wq.dtype not in (torch.int8, torch.uint8):
        raise TypeError("wq must be int8 (or uint8 bytes for packed int4)")
    M, K = x.shape
    if wf in (SASQ_W_INT8_BLOCKED, SASQ_W_INT4_BLOCKED):
        N = y.shape[1]
        if wq.numel() != sasq_packed_weight_bytes(N, K, wf) or y.shape[0] != M or y.dtype != x.dtype:
            raise ValueError("shape mismatch between x, the packed weights and y")
    else:
        N = wq.shape[0]
        if wq.shape[1] != (K if wf == SASQ_W_INT8 else K // 2) or tuple(y.shape) != (M, N) or y.dtype != x.dtype:
            raise ValueError("shape mismatch between x, wq and y")
    if s_w.numel() != N or (bias is not None and bias.numel() != N):
        raise ValueError("s_w / bias must have N elements")
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib().sasq_static_linear(_ptr(x), _ptr(s), _ptr(wq), _ptr(s_w), _ptr(bias), _ptr(y), _ptr(acc_out),
                                     _ptr(xq_out), M, N, K, a_bits, wf, _dt(x), _ptr(workspace), wsb, _stream()),
           "sasq_static_linear")


def sasq_static_linear_grouped(x: torch.Tensor, s_g: torch.Tensor, wq: torch.Tensor, s_w: torch.Tensor,
                               bias: Optional[torch.Tensor], y: torch.Tensor, group: int, wf: int = SASQ_W_INT8,
                               workspace: Optional[torch.Tensor] = None, f_out: Optional[torch.Tensor] = None,
                               xq_out: Optional[torch.Tensor] = None, a_bits: int = 8) -> None:
    _want(s_g, torch.float32, "s_g"); _want(s_w, torch.float32, "s_w"); _want(bias, torch.float32, "bias")
    _want(f_out, torch.float32, "f_out"); _want(xq_out, torch.int8, "xq_out")
    if wq.dtype not in (torch.int8, torch.uint8):
        raise TypeError("wq must be int8 (or uint8 bytes for packed int4 / pre-arranged weights)")
    M, K = x.shape
    N = y.shape[1]
    if group <= 0 or K % group or s_g.numel() != K // group:
        raise ValueError("group must divide K and s_g must have K / group elements")
    if wf in (SASQ_W_INT8_BLOCKED, SASQ_W_INT4_BLOCKED):
        ok = wq.numel() == sasq_packed_weight_bytes(N, K, wf)
    else:
        ok = tuple(wq.shape) == (N, K if wf == SASQ_W_INT8 else K // 2)
    if not ok or y.shape[0] != M or y.dtype != x.dtype:
        raise ValueError("shape mismatch between x, wq and y")
    if s_w.numel() != N or (bias is not None and bias.numel() != N):
        raise ValueError("s_w / bias must have N elements")
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib().sasq_static_linear_grouped(_ptr(x), _ptr(s_g), _ptr(wq), _ptr(s_w), _ptr(bias), _ptr(y), _ptr(f_out),
                                             _ptr(xq_out), M, N, K, group, a_bits, wf, _dt(x), _ptr(workspace), wsb,
                                             _stream()), "sasq_static_linear_grouped")


def sasq_dynamic_linear_workspace(M: int, N: int, K: int, wf: int) -> int:
    return int(_lib().sasq_dynamic_linear_workspace(M, N, K, wf))


def sasq_dynamic_linear(x: torch.Tensor, wq: torch.Tensor, s_w: torch.Tensor, bias: Optional[torch.Tensor],
                        y: torch.Tensor, wf: int = SASQ_W_INT8, workspace: Optional[torch.Tensor] = None,
                        acc_out: Optional[torch.Tensor] = None, xq_out: Optional[torch.Tensor] = None,
                        s_row_out: Optional[torch.Tensor] = None, a_bits: int = 8) -> None:
    _want(s_w, torch.float32, "s_w"); _want(bias, torch.float32, "bias"); _want(s_row_out, torch.float32, "s_row_out")
    _want(acc_out, torch.int32, "acc_out"); _want(xq_out, torch.int8, "xq_out")
    if wq.dtype not in (torch.int8, torch.uint8):
        raise TypeError("wq must be int8 (or uint8 bytes for packed int4 / pre-arranged weights)")
    M, K = x.shape
    N = y.shape[1]
    if wf in (SASQ_W_INT8_BLOCKED, SASQ_W_INT4_BLOCKED):
        ok = wq.numel() == sasq_packed_weight_bytes(N, K, wf)
    else:
        ok = tuple(wq.shape) == (N, K if wf == SASQ_W_INT8 else K // 2)
    if not ok or y.shape[0] != M or y.dtype != x.dtype:
        raise ValueError("shape mismatch between x, wq and y")
    if s_w.numel() != N or (bias is not None and bias.numel() != N) or (s_row_out is not None and s_row_out.numel() != M):
        raise ValueError("s_w / bias must have N elements, s_row_out M")
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib().sasq_dynamic_linear(_ptr(x), _ptr(wq), _ptr(s_w), _ptr(bias), _ptr(y), _ptr(acc_out), _ptr(xq_out),
                                      _ptr(s_row_out), M, N, K, a_bits, wf, _dt(x), _ptr(workspace), wsb, _stream()),
           "sasq_dynamic_linear")


def _lin_items(items, wf: int):
    """items: sequence of (x, s, wq, s_w, bias_or_None, y)."""
    if not 1 <= len(items) <= SASQ_MAX_BATCH:
        raise ValueError(f"a batch holds 1..{SASQ_MAX_BATCH} projections")
    arr = (_LinItem * len(items))()
    dt = None
    for i, (x, s, wq, s_w, bias, y) in enumerate(items):
        _want(s, torch.float32, "s"); _want(s_w, torch.float32, "s_w"); _want(bias, torch.float32, "bias")
        M, K = x.shape
        N = y.shape[1]
        if wf in (SASQ_W_INT8_BLOCKED, SASQ_W_INT4_BLOCKED):
            ok = wq.numel() == sasq_packed_weight_bytes(N, K, wf)
        else:
            ok = tuple(wq.shape) == (N, K if wf == SASQ_W_INT8 else K // 2)
        if not ok or y.shape[0] != M or y.dtype != x.dtype or s_w.numel() != N or (bias is not None and bias.numel() != N):
            raise ValueError(f"shape mismatch in batch item {i}")
        if dt is None:
            dt = _dt(x)
        elif _dt(x) != dt:
            raise TypeError("all projections of a batch must have the same activation dtype")
        arr[i].x, arr[i].s, arr[i].wq, arr[i].s_w = _ptr(x).value, _ptr(s).value, _ptr(wq).value, _ptr(s_w).value
        arr[i].bias, arr[i].y = (None if bias is None else _ptr(bias).value), _ptr(y).value
        arr[i].M, arr[i].N, arr[i].K = M, N, K
    return arr, dt


def sasq_static_linear_batch_workspace(items, wf: int = SASQ_W_INT8) -> int:
    arr, _ = _lin_items(items, wf)
    return int(_lib().sasq_static_linear_batch_workspace(arr, len(items), wf))


def sasq_static_linear_batch(items, wf: int, workspace: torch.Tensor, a_bits: int = 8) -> None:
    arr, dt = _lin_items(items, wf)
    _check(_lib().sasq_static_linear_batch(arr, len(items), a_bits, wf, dt, _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()),
           "sasq_static_linear_batch")


def sasq_quantize_weight(w: torch.Tensor, wq: torch.Tensor, s_w: torch.Tensor, wf: int = SASQ_W_INT8) -> None:
    _want(w, torch.float32, "w"); _want(s_w, torch.float32, "s_w")
    N, K = w.shape
    _check(_lib().sasq_quantize_weight(_ptr(w), _ptr(wq), _ptr(s_w), N, K, wf, _stream()), "sasq_quantize_weight")


def sasq_packed_weight_bytes(N: int, K: int, wf: int) -> int:
    return int(_lib().sasq_packed_weight_bytes(N, K, wf))


def sasq_pack_weight(wq: torch.Tensor, packed: torch.Tensor, N: int, K: int, wf_src: int = SASQ_W_INT8) -> None:
    blocked = SASQ_W_INT8_BLOCKED if wf_src == SASQ_W_INT8 else SASQ_W_INT4_BLOCKED
    if wq.numel() != (N * K if wf_src == SASQ_W_INT8 else N * (K // 2)):
        raise ValueError("wq does not hold N x K codes in the source format")
    if packed.numel() * packed.element_size() != sasq_packed_weight_bytes(N, K, blocked):
        raise ValueError("packed must have sasq_packed_weight_bytes(N, K, blocked format) bytes")
    _check(_lib().sasq_pack_weight(_ptr(wq), _ptr(packed), N, K, wf_src, _stream()), "sasq_pack_weight")


def sasq_bwd_weight_bytes(N: int, K: int) -> int:
    return int(_lib().sasq_bwd_weight_bytes(N, K))


def sasq_prepare_bwd_weight(wq: torch.Tensor, s_w: torch.Tensor, wt: torch.Tensor, N: int, K: int,
                            wf: int, dtype: torch.dtype) -> None:
    _want(s_w, torch.float32, "s_w")
    if dtype not in _DT:
        raise TypeError("dtype must be float16 or bfloat16")
    if wq.numel() * wq.element_size() != (N * K if wf == SASQ_W_INT8 else N * (K // 2)):
        raise ValueError("wq does not hold N x K codes in the row-major format wf")
    if s_w.numel() != N:
        raise ValueError("s_w must hold N factors")
    if wt.numel() * wt.element_size() != sasq_bwd_weight_bytes(N, K):
        raise ValueError("wt must have sasq_bwd_weight_bytes(N, K) bytes")
    _check(_lib().sasq_prepare_bwd_weight(_ptr(wq), _ptr(s_w), _ptr(wt), N, K, wf, _DT[dtype], _stream()),
           "sasq_prepare_bwd_weight")


def sasq_linear_bwd_input(dy: torch.Tensor, wt: torch.Tensor, dx: torch.Tensor, K: int,
                          acc_out: Optional[torch.Tensor] = None) -> None:
    M, N = dy.shape
    _want(acc_out, torch.float32, "acc_out")
    if acc_out is not None and tuple(acc_out.shape) != (M, K):
        raise ValueError("acc_out must be [M, K]")
    if dx.dtype != dy.dtype or tuple(dx.shape) != (M, K):
        raise ValueError("dx must be [M, K] of dy's dtype")
    if wt.numel() * wt.element_size() != sasq_bwd_weight_bytes(N, K):
        raise ValueError("wt must have sasq_bwd_weight_bytes(N, K) bytes")
    _check(_lib().sasq_linear_bwd_input(_ptr(dy), _ptr(wt), _ptr(dx), _ptr(acc_out), M, N, K, _dt(dy), _stream()),
           "sasq_linear_bwd_input")


def sasq_absmax_scale_workspace(rows: int, cols: int) -> int:
    return int(_lib().sasq_absmax_scale_workspace(rows, cols))


def sasq_absmax_scale(x: torch.Tensor, s: torch.Tensor, workspace: torch.Tensor, bits: int = 8) -> None:
    _want(s, torch.float32, "s")
    rows, cols = x.shape[0], x.numel() // max(x.shape[0], 1)
    _check(_lib().sasq_absmax_scale(_ptr(x), _ptr(s), rows, cols, bits, _dt(x), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream()), "sasq_absmax_scale")
