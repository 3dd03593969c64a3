"""ctypes loader for the SASQ CPU oracle (oracle/sasq_oracle.c).

TEST INFRASTRUCTURE ONLY: importable from tests/, from __graft_entry__.smoke()
and from bench.py's cpu_baseline leg.  The HIP library and its Python binding
never import this package, and this package never imports them.

All 16-bit float tensors cross this interface as numpy uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sasq_oracle.c")
_LIB = os.path.join(_HERE, "libsasq_oracle.so")
# The mutation tests (tests/test_oracle_mutations.py) point this at a deliberately broken copy of
# the source to show that the pins notice; nothing else sets it.
if os.environ.get("SASQ_ORACLE_MUTANT_SRC"):
    _SRC = os.environ["SASQ_ORACLE_MUTANT_SRC"]
    _LIB = os.path.splitext(_SRC)[0] + ".so"

DT = {"f16": 0, "bf16": 1}
WF = {"int8": 0, "int4": 1}
NO_ROUND, NO_CLAMP, STE_ON_V = 1, 2, 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over rows, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.sasq_oracle_scale_sgd.restype = ctypes.c_float
        L.sasq_oracle_scale_sgd.argtypes = [ctypes.c_float] * 3
        L.sasq_oracle_inv_scale.restype = ctypes.c_float
        L.sasq_oracle_inv_scale.argtypes = [ctypes.c_float]
        L.sasq_oracle_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with status {rc}")


def threads() -> int:
    return int(lib().sasq_oracle_threads())


def decode16(bits: np.ndarray, dtype: str) -> np.ndarray:
    bits = _u16(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    lib().sasq_oracle_decode16(_p(bits), _p(out), ctypes.c_int64(bits.size), DT[dtype])
    return out


def encode16(vals: np.ndarray, dtype: str) -> np.ndarray:
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    out = np.empty(vals.shape, dtype=np.uint16)
    lib().sasq_oracle_encode16(_p(vals), _p(out), ctypes.c_int64(vals.size), DT[dtype])
    return out


def inv_scale(s: float) -> np.float32:
    return np.float32(lib().sasq_oracle_inv_scale(ctypes.c_float(float(s))))


def fakequant_fwd(x: np.ndarray, s: float, bits: int, dtype: str, flags: int = 0
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (y bits uint16 [rows, cols], codes int8 [rows, cols])."""
    x = _u16(x)
    rows, cols = (x.shape if x.ndim == 2 else (1, x.size))
    y = np.empty(x.shape, dtype=np.uint16)
    codes = np.empty(x.shape, dtype=np.int8)
    rc = lib().sasq_oracle_fakequant_fwd(_p(x), ctypes.c_float(float(s)), _p(y), _p(codes),
                                         ctypes.c_int64(rows), ctypes.c_int64(cols),
                                         int(bits), DT[dtype], int(flags))
    _check(rc, "fakequant_fwd")
    return y, codes


def fakequant_bwd(x: np.ndarray, dy: np.ndarray, s: float, bits: int, dtype: str, flags: int = 0,
                  want_dx: bool = True):
    """Returns dict(dx=uint16 bits, ds=np.float32, ds64=float, sum_abs=float)."""
    x, dy = _u16(x), _u16(dy)
    assert x.shape == dy.shape
    rows, cols = (x.shape if x.ndim == 2 else (1, x.size))
    dx = np.empty(x.shape, dtype=np.uint16) if want_dx else None
    ds = ctypes.c_float(0.0)
    ds64 = ctypes.c_double(0.0)
    sabs = ctypes.c_double(0.0)
    rc = lib().sasq_oracle_fakequant_bwd(_p(x), _p(dy), ctypes.c_float(float(s)), _p(dx),
                                         ctypes.byref(ds), ctypes.byref(ds64), ctypes.byref(sabs),
                                         ctypes.c_int64(rows), ctypes.c_int64(cols),
                                         int(bits), DT[dtype], int(flags))
    _check(rc, "fakequant_bwd")
    return {"dx": dx, "ds": np.float32(ds.value), "ds64": float(ds64.value),
            "sum_abs": float(sabs.value)}


def static_linear(x: np.ndarray, s: float, wq: np.ndarray, s_w: np.ndarray,
                  bias: Optional[np.ndarray], a_bits: int, w_fmt: str, dtype: str,
                  want_y: bool = True, want_acc: bool = True, want_xq: bool = True):
    """x: [M,K] uint16 bits; wq: [N,K] int8 or [N,K/2] uint8 (packed int4).
    Returns dict(y=uint16 [M,N], acc=int32 [M,N], xq=int8 [M,K])."""
    x = _u16(x)
    M, K = x.shape
    wq = np.ascontiguousarray(wq)
    assert wq.dtype in (np.int8, np.uint8)
    N = wq.shape[0]
    assert wq.shape[1] == (K if w_fmt == "int8" else K // 2), (wq.shape, K, w_fmt)
    s_w = np.ascontiguousarray(s_w, dtype=np.float32)
    assert s_w.shape == (N,)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (N,)
    y = np.empty((M, N), dtype=np.uint16) if want_y else None
    acc = np.empty((M, N), dtype=np.int32) if want_acc else None
    xq = np.empty((M, K), dtype=np.int8) if want_xq else None
    rc = lib().sasq_oracle_static_linear(_p(x), ctypes.c_float(float(s)), _p(wq), _p(s_w), _p(bias),
                                         _p(y), _p(acc), _p(xq), ctypes.c_int64(M),
                                         ctypes.c_int64(N), ctypes.c_int64(K), int(a_bits),
                                         WF[w_fmt], DT[dtype])
    _check(rc, "static_linear")
    return {"y": y, "acc": acc, "xq": xq}


def static_linear_grouped(x: np.ndarray, s_g: np.ndarray, wq: np.ndarray, s_w: np.ndarray,
                          bias: Optional[np.ndarray], group: int, a_bits: int, w_fmt: str, dtype: str):
    """Eq. 3 form: one activation factor per `group` consecutive input channels.
    Returns dict(y=uint16 [M,N], f=float32 [M,N] (the fp32 group sum before s_w), xq=int8 [M,K])."""
    x = _u16(x)
    M, K = x.shape
    wq = np.ascontiguousarray(wq)
    assert wq.dtype in (np.int8, np.uint8)
    N = wq.shape[0]
    assert wq.shape[1] == (K if w_fmt == "int8" else K // 2), (wq.shape, K, w_fmt)
    s_g = np.ascontiguousarray(s_g, dtype=np.float32)
    assert K % group == 0 and s_g.shape == (K // group,)
    s_w = np.ascontiguousarray(s_w, dtype=np.float32)
    assert s_w.shape == (N,)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    y = np.empty((M, N), dtype=np.uint16)
    f = np.empty((M, N), dtype=np.float32)
    xq = np.empty((M, K), dtype=np.int8)
    rc = lib().sasq_oracle_static_linear_grouped(_p(x), _p(s_g), _p(wq), _p(s_w), _p(bias), _p(y), _p(f), _p(xq),
                                                 ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K),
                                                 ctypes.c_int64(group), int(a_bits), WF[w_fmt], DT[dtype])
    _check(rc, "static_linear_grouped")
    return {"y": y, "f": f, "xq": xq}


def dynamic_linear(x: np.ndarray, wq: np.ndarray, s_w: np.ndarray, bias: Optional[np.ndarray],
                   a_bits: int, w_fmt: str, dtype: str):
    """Dynamic per-token linear (one absmax factor per row, computed from the row itself).
    Returns dict(y=uint16 [M,N], acc=int32 [M,N], xq=int8 [M,K], s_row=float32 [M])."""
    x = _u16(x)
    M, K = x.shape
    wq = np.ascontiguousarray(wq)
    assert wq.dtype in (np.int8, np.uint8)
    N = wq.shape[0]
    assert wq.shape[1] == (K if w_fmt == "int8" else K // 2), (wq.shape, K, w_fmt)
    s_w = np.ascontiguousarray(s_w, dtype=np.float32)
    assert s_w.shape == (N,)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    y = np.empty((M, N), dtype=np.uint16)
    acc = np.empty((M, N), dtype=np.int32)
    xq = np.empty((M, K), dtype=np.int8)
    s_row = np.empty((M,), dtype=np.float32)
    rc = lib().sasq_oracle_dynamic_linear(_p(x), _p(wq), _p(s_w), _p(bias), _p(y), _p(acc), _p(xq), _p(s_row),
                                          ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K),
                                          int(a_bits), WF[w_fmt], DT[dtype])
    _check(rc, "dynamic_linear")
    return {"y": y, "acc": acc, "xq": xq, "s_row": s_row}


def linear_bwd_input(dy: np.ndarray, wq: np.ndarray, s_w: np.ndarray, w_fmt: str, dtype: str):
    """dX = dY . Wq with Wq the dequantized frozen weight in the 16-bit type.
    Returns dict(dx=uint16 [M,K], wq16=uint16 [N,K], sum_abs=float64 [M,K], exact=float64 [M,K])."""
    dy = _u16(dy)
    M, N = dy.shape
    wq = np.ascontiguousarray(wq)
    assert wq.dtype in (np.int8, np.uint8) and wq.shape[0] == N
    K = wq.shape[1] * (1 if w_fmt == "int8" else 2)
    s_w = np.ascontiguousarray(s_w, dtype=np.float32)
    assert s_w.shape == (N,)
    dx = np.empty((M, K), dtype=np.uint16)
    w16 = np.empty((N, K), dtype=np.uint16)
    sabs = np.empty((M, K), dtype=np.float64)
    exact = np.empty((M, K), dtype=np.float64)
    rc = lib().sasq_oracle_linear_bwd_input(_p(dy), _p(wq), _p(s_w), _p(dx), _p(w16), _p(sabs), _p(exact),
                                            ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K),
                                            WF[w_fmt], DT[dtype])
    _check(rc, "linear_bwd_input")
    return {"dx": dx, "wq16": w16, "sum_abs": sabs, "exact": exact}


def quantize_weight(w: np.ndarray, w_fmt: str) -> Tuple[np.ndarray, np.ndarray]:
    """w: fp32 [N,K] -> (wq int8 [N,K] | uint8 [N,K/2], s_w fp32 [N])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, K = w.shape
    if w_fmt == "int8":
        wq = np.empty((N, K), dtype=np.int8)
    else:
        wq = np.zeros((N, K // 2), dtype=np.uint8)
    s_w = np.empty((N,), dtype=np.float32)
    rc = lib().sasq_oracle_quantize_weight(_p(w), _p(wq), _p(s_w), ctypes.c_int64(N),
                                           ctypes.c_int64(K), WF[w_fmt])
    _check(rc, "quantize_weight")
    return wq, s_w


def absmax_scale(x: np.ndarray, bits: int, dtype: str) -> np.float32:
    x = _u16(x)
    s = ctypes.c_float(0.0)
    rc = lib().sasq_oracle_absmax_scale(_p(x), ctypes.byref(s), ctypes.c_int64(x.size),
                                        int(bits), DT[dtype])
    _check(rc, "absmax_scale")
    return np.float32(s.value)


def scale_sgd(s: float, ds: float, lr: float) -> np.float32:
    return np.float32(lib().sasq_oracle_scale_sgd(ctypes.c_float(float(s)), ctypes.c_float(float(ds)),
                                                  ctypes.c_float(float(lr))))


def fakequant_fwd_pc(x: np.ndarray, s: np.ndarray, bits: int, dtype: str) -> Tuple[np.ndarray, np.ndarray]:
    """Per-channel forward: s has one fp32 factor per column of x [rows, cols]."""
    x = _u16(x)
    rows, cols = x.shape
    s = np.ascontiguousarray(s, dtype=np.float32)
    assert s.shape == (cols,)
    y = np.empty(x.shape, dtype=np.uint16)
    codes = np.empty(x.shape, dtype=np.int8)
    rc = lib().sasq_oracle_fakequant_fwd_pc(_p(x), _p(s), _p(y), _p(codes), ctypes.c_int64(rows),
                                            ctypes.c_int64(cols), int(bits), DT[dtype])
    _check(rc, "fakequant_fwd_pc")
    return y, codes


def fakequant_bwd_pc(x: np.ndarray, dy: np.ndarray, s: np.ndarray, bits: int, dtype: str):
    """Per-channel backward: dict(dx=uint16 bits, ds=float32 [cols], ds64=float64 [cols], sum_abs=float64 [cols])."""
    x, dy = _u16(x), _u16(dy)
    rows, cols = x.shape
    s = np.ascontiguousarray(s, dtype=np.float32)
    assert s.shape == (cols,) and dy.shape == x.shape
    dx = np.empty(x.shape, dtype=np.uint16)
    ds = np.empty(cols, dtype=np.float32)
    ds64 = np.empty(cols, dtype=np.float64)
    sabs = np.empty(cols, dtype=np.float64)
    rc = lib().sasq_oracle_fakequant_bwd_pc(_p(x), _p(dy), _p(s), _p(dx), _p(ds), _p(ds64), _p(sabs),
                                            ctypes.c_int64(rows), ctypes.c_int64(cols), int(bits), DT[dtype])
    _check(rc, "fakequant_bwd_pc")
    return {"dx": dx, "ds": ds, "ds64": ds64, "sum_abs": sabs}


def scale_adamw(p: np.ndarray, g: np.ndarray, m: np.ndarray, v: np.ndarray, step: int, lr: float,
                b1: float = 0.9, b2: float = 0.999, eps: float = 1e-8, wd: float = 0.01):
    """One AdamW step on fp32 vectors; returns new (p, m, v)."""
    p, m, v = (np.array(a, dtype=np.float32, copy=True) for a in (p, m, v))
    g = np.ascontiguousarray(g, dtype=np.float32)
    d = ctypes.c_double
    lib().sasq_oracle_scale_adamw(_p(p), _p(g), _p(m), _p(v), ctypes.c_int64(p.size), ctypes.c_int64(step),
                                  d(lr), d(b1), d(b2), d(eps), d(wd))
    return p, m, v
