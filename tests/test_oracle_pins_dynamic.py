"""Pins for the oracle's dynamic per-token linear (no GPU): a hand-worked example, row factors
against numpy float32 arithmetic, codes against exact rational arithmetic, accumulators against an
int64 matmul, outputs against float64 and against numpy fp32 in the pinned operation order."""
from __future__ import annotations

import os

import numpy as np
import pytest

import oracle
from paper_2512_14481_amd import workloads as wl
from tests import exact_ref as ex

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _val(bits, dtype):
    return wl.storage_bits_to_f32(bits, dtype).astype(np.float64)


def _w_int64(wq, w_fmt):
    if w_fmt == "int8":
        return wq.astype(np.int64)
    N, K2 = wq.shape
    lo, hi = (wq & 15).astype(np.int64), (wq >> 4).astype(np.int64)
    w8 = np.empty((N, 2 * K2), dtype=np.int64)
    w8[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    w8[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    return w8


def test_dynamic_hand_example():
    rows = {}
    for line in open(os.path.join(GOLD, "dynamic_linear.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = np.array([float(t) for t in v])
    x = wl.f32_to_storage_bits(np.stack([rows["x0"], rows["x1"]]).astype(np.float32), "f16")
    wq = np.stack([rows["w0"], rows["w1"]]).astype(np.int8)
    out = oracle.dynamic_linear(x, wq, rows["s_w"], None, 8, "int8", "f16")
    assert np.array_equal(out["s_row"], rows["s_row"].astype(np.float32))
    assert np.array_equal(out["xq"], np.stack([rows["codes0"], rows["codes1"]]).astype(np.int8))
    assert np.array_equal(out["acc"], np.stack([rows["acc0"], rows["acc1"]]).astype(np.int32))
    assert np.array_equal(_val(out["y"], "f16"), np.stack([rows["y0"], rows["y1"]]))
    out = oracle.dynamic_linear(x, wq, rows["s_w"], rows["bias"], 8, "int8", "f16")
    assert np.array_equal(_val(out["y"], "f16"), np.stack([rows["yb0"], rows["yb1"]]))


@pytest.mark.parametrize("dtype,w_fmt,bits", [("f16", "int8", 8), ("bf16", "int4", 8), ("bf16", "int8", 4)])
def test_dynamic_linear_vs_independent_arithmetic(dtype, w_fmt, bits):
    M, N, K = 13, 17, 64
    x = wl.random_bits(61, f"dx{dtype}", (M, K), dtype, gain=3.0)
    x[5] = 0                                              # an all-zero row
    w = wl.random_f32(61, f"dw{w_fmt}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, w_fmt)
    bias = wl.random_f32(61, "db", (N,), 0.5)
    out = oracle.dynamic_linear(x, wq, s_w, bias, bits, w_fmt, dtype)
    Qp = (1 << (bits - 1)) - 1
    # row factors: numpy float32 division of the row absmax (exactly representable) by Qp
    xv = wl.storage_bits_to_f32(x, dtype)
    s_ref = (np.abs(xv).max(axis=1).astype(np.float32) / np.float32(Qp)).astype(np.float32)
    s_ref[5] = 1.0
    assert np.array_equal(out["s_row"], s_ref)
    # no row clips at its own absmax factor, and the largest element maps to +-Qp
    assert np.abs(out["xq"].astype(np.int64)).max(axis=1)[np.arange(M) != 5].min() == Qp
    # codes: exact rational evaluation of Eq. 1 with the reciprocal reading
    for m in range(M):
        for k in range(0, K, 3):
            _, _, q, _ = ex.quantize_exact(int(x[m, k]), dtype, s_ref[m], bits)
            assert out["xq"][m, k] == q, (m, k)
    ref_acc = out["xq"].astype(np.int64) @ _w_int64(wq, w_fmt).T
    assert np.array_equal(out["acc"].astype(np.int64), ref_acc)
    exact = ref_acc.astype(np.float64) * s_ref.astype(np.float64)[:, None] * s_w.astype(np.float64)[None, :] + bias.astype(np.float64)
    yv = _val(out["y"], dtype)
    ulp = np.abs(_val((out["y"] + 1).astype(np.uint16), dtype) - yv)
    assert (np.abs(yv - exact) <= 0.5 * ulp * (1 + 2.0 ** -9) + 1e-30).all()
    # pinned operation order, replayed with numpy fp32: c = s_m * s_w[n]; y = fl32(acc) * c; + bias
    c = (s_ref[:, None] * s_w[None, :]).astype(np.float32)
    yf = ((ref_acc.astype(np.float32) * c).astype(np.float32) + bias[None, :]).astype(np.float32)
    assert np.array_equal(_val(out["y"], dtype), _val(wl.f32_to_storage_bits(yf, dtype), dtype))


def test_dynamic_rows_are_independent_and_scale_covariant():
    """A row's outputs depend on that row only, and multiplying a row by a power of two leaves its
    codes unchanged and multiplies its factor (dynamic quantization adapts per token)."""
    M, N, K = 6, 5, 32
    dtype = "f16"
    x = wl.random_bits(62, "dix", (M, K), dtype, gain=1.0)
    wq = wl.random_codes(62, "diw", (N, K), -127, 127)
    s_w = np.full(N, 0.01, np.float32)
    full = oracle.dynamic_linear(x, wq, s_w, None, 8, "int8", dtype)
    for m in range(M):
        one = oracle.dynamic_linear(np.ascontiguousarray(x[m:m + 1]), wq, s_w, None, 8, "int8", dtype)
        assert np.array_equal(one["y"][0], full["y"][m]) and np.array_equal(one["xq"][0], full["xq"][m])
    x4 = wl.f32_to_storage_bits(wl.storage_bits_to_f32(x, dtype) * np.float32(4.0), dtype)
    big = oracle.dynamic_linear(x4, wq, s_w, None, 8, "int8", dtype)
    assert np.array_equal(big["xq"], full["xq"])
    assert np.array_equal(big["s_row"], full["s_row"] * np.float32(4.0))
