"""Pins for the oracle's backward of the frozen quantized linear (no GPU): a hand-worked example,
the dequantized weight against numpy float32 arithmetic, the sums against a float64 matmul of
independently decoded operands, the rounding of the result, and the adjoint identity that ties
it to the forward product."""
from __future__ import annotations

import os

import numpy as np
import pytest

import oracle
from paper_2512_14481_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _val(bits, dtype):
    return wl.storage_bits_to_f32(bits, dtype).astype(np.float64)


def _w_int(wq, w_fmt):
    if w_fmt == "int8":
        return wq.astype(np.int64)
    N, K2 = wq.shape
    lo, hi = (wq & 15).astype(np.int64), (wq >> 4).astype(np.int64)
    w = np.empty((N, 2 * K2), dtype=np.int64)
    w[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    w[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    return w


def test_bwd_linear_hand_example():
    rows = {}
    for line in open(os.path.join(GOLD, "linear_bwd_input.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = np.array([float(t) for t in v])
    dy = wl.f32_to_storage_bits(np.stack([rows["dy0"], rows["dy1"]]).astype(np.float32), "f16")
    wq = np.stack([rows["w0"], rows["w1"]]).astype(np.int8)
    out = oracle.linear_bwd_input(dy, wq, rows["s_w"], "int8", "f16")
    assert np.array_equal(_val(out["wq16"], "f16"), np.stack([rows["wq0"], rows["wq1"]]))
    assert np.array_equal(_val(out["dx"], "f16"), np.stack([rows["dx0"], rows["dx1"]]))
    assert np.array_equal(out["exact"], np.stack([rows["dx0"], rows["dx1"]]))


@pytest.mark.parametrize("dtype,w_fmt", [("f16", "int8"), ("bf16", "int8"), ("bf16", "int4"), ("f16", "int4")])
def test_bwd_linear_vs_independent_arithmetic(dtype, w_fmt):
    M, N, K = 11, 19, 26                                   # all different: a transposed index cannot pass
    dy = wl.random_bits(71, f"bdy{dtype}", (M, N), dtype, gain=0.01)
    w = wl.random_f32(71, f"bw{w_fmt}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, w_fmt)
    out = oracle.linear_bwd_input(dy, wq, s_w, w_fmt, dtype)
    # dequantized weight: numpy float32 product, rounded by the input module's own converter
    w32 = (_w_int(wq, w_fmt).astype(np.float32) * s_w[:, None]).astype(np.float32)
    assert np.array_equal(out["wq16"], wl.f32_to_storage_bits(w32, dtype))
    # sums: float64 matmul of independently decoded operands
    dyv, wv = _val(dy, dtype), _val(out["wq16"], dtype)
    ref = dyv @ wv
    sabs = np.abs(dyv) @ np.abs(wv)
    assert np.allclose(out["sum_abs"], sabs, rtol=1e-12, atol=0)
    assert (np.abs(out["exact"] - ref) <= 1e-13 * sabs + 1e-300).all()
    # result: the 16-bit value nearest the sum (through one fp32 rounding, hence the 2^-9 slack)
    dxv = _val(out["dx"], dtype)
    ulp = np.abs(_val((out["dx"] + 1).astype(np.uint16), dtype) - dxv)
    assert (np.abs(dxv - ref) <= 0.5 * ulp * (1 + 2.0 ** -9) + 1e-13 * sabs).all()


def test_bwd_linear_is_the_adjoint_of_the_forward_product():
    """<dY, X Wq^T> == <dY Wq, X> for any X: pins operand roles and index order without restating
    the sum.  X is drawn as small integers so both sides are exact in float64."""
    M, N, K = 7, 12, 10
    dy = wl.f32_to_storage_bits(wl.random_codes(72, "ady", (M, N), -8, 8).astype(np.float32), "f16")
    wq = wl.random_codes(72, "aw", (N, K), -127, 127).astype(np.int8)
    s_w = np.float32(2.0) ** -wl.random_codes(72, "as", (N,), 3, 6).astype(np.float32)
    out = oracle.linear_bwd_input(dy, wq, s_w, "int8", "f16")
    X = wl.random_codes(72, "ax", (M, K), -5, 5).astype(np.float64)
    Wq = wq.astype(np.float64) * s_w.astype(np.float64)[:, None]          # exact: powers of two
    lhs = float((_val(dy, "f16") * (X @ Wq.T)).sum())
    rhs = float((out["exact"] * X).sum())
    assert lhs == rhs


def test_bwd_linear_single_channel_reduces_to_scaling():
    """With one output channel dX is the outer product dy[m] * Wq[k]; with a one-hot dY row it
    returns that channel's dequantized weight row."""
    K = 16
    wq = wl.random_codes(73, "sw", (3, K), -127, 127).astype(np.int8)
    s_w = np.array([0.5, 0.125, 2.0], dtype=np.float32)
    dy = wl.f32_to_storage_bits(np.array([[0, 1, 0], [0, 0, -2]], dtype=np.float32), "bf16")
    out = oracle.linear_bwd_input(dy, wq, s_w, "int8", "bf16")
    assert np.array_equal(_val(out["dx"], "bf16")[0], wq[1].astype(np.float64) * 0.125)
    assert np.array_equal(_val(out["dx"], "bf16")[1], wq[2].astype(np.float64) * -4.0)


def test_bwd_linear_rejects_bad_arguments():
    dy = np.zeros((2, 2), dtype=np.uint16)
    with pytest.raises(Exception):
        oracle.linear_bwd_input(dy, np.zeros((2, 3), dtype=np.int8), np.ones(2, np.float32), "int3", "f16")
