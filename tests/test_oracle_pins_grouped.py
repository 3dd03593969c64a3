"""Pins for the oracle's grouped static linear (Sec. 3, Eq. 3; no GPU): a hand-worked example,
exact rational emulation of the fp32 accumulation chain, reductions to the per-tensor linear and
to the per-channel fake-quant codes, and real-arithmetic bounds."""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2512_14481_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _val(bits, dtype):
    return wl.storage_bits_to_f32(bits, dtype).astype(np.float64)


def _round_f32(v: Fraction) -> np.float32:
    """Nearest float32 to an exact rational, ties to even (integer arithmetic only; normal range)."""
    if v == 0:
        return np.float32(0.0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert -126 <= e <= 127
    scaled = a / Fraction(2) ** (e - 23)            # in [2^23, 2^24)
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    return np.float32(sign * float(Fraction(n) * Fraction(2) ** (e - 23)))


def _codes_int64(wq, w_fmt):
    if w_fmt == "int8":
        return wq.astype(np.int64)
    N, K2 = wq.shape
    lo, hi = (wq & 15).astype(np.int64), (wq >> 4).astype(np.int64)
    w8 = np.empty((N, 2 * K2), dtype=np.int64)
    w8[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    w8[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    return w8


def test_grouped_hand_example():
    rows = {}
    for line in open(os.path.join(GOLD, "grouped_linear.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = np.array([float(t) for t in v])
    x = wl.f32_to_storage_bits(rows["x"].astype(np.float32)[None, :], "f16")
    wq = np.stack([rows["w0"], rows["w1"]]).astype(np.int8)
    out = oracle.static_linear_grouped(x, rows["s_g"], wq, rows["s_w"], None, 2, 8, "int8", "f16")
    assert np.array_equal(out["xq"][0], rows["codes"].astype(np.int8))
    assert np.array_equal(out["f"][0], rows["f"].astype(np.float32))
    assert np.array_equal(_val(out["y"], "f16")[0], rows["y"])
    out = oracle.static_linear_grouped(x, rows["s_g"], wq, rows["s_w"], rows["bias"], 2, 8, "int8", "f16")
    assert np.array_equal(_val(out["y"], "f16")[0], rows["y_bias"])


@pytest.mark.parametrize("dtype,w_fmt", [("f16", "int8"), ("bf16", "int4")])
def test_grouped_chain_vs_exact_rational(dtype, w_fmt):
    """f is the ascending chain of single-rounded fused multiply-adds, nothing else: emulated with
    exact rationals rounded once per step.  The same data must tell it apart from the unfused chain
    and from the descending order (otherwise this pin would not see those mistakes)."""
    M, N, K, group = 6, 7, 96, 16
    G = K // group
    x = wl.random_bits(41, f"gx{dtype}", (M, K), dtype, gain=2.0)
    w = wl.random_f32(41, f"gw{w_fmt}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, w_fmt)
    s_g = (0.01 + 0.05 * wl.random_f32(41, "gs", (G,), 1.0) ** 2).astype(np.float32)
    out = oracle.static_linear_grouped(x, s_g, wq, s_w, None, group, 8, w_fmt, dtype)
    w8 = _codes_int64(wq, w_fmt)
    q = out["xq"].astype(np.int64)
    acc = np.stack([q[:, i * group:(i + 1) * group] @ w8[:, i * group:(i + 1) * group].T for i in range(G)])   # [G, M, N]
    asc = np.empty((M, N), dtype=np.float32)
    desc = np.empty((M, N), dtype=np.float32)
    unfused = np.zeros((M, N), dtype=np.float32)
    for m in range(M):
        for n in range(N):
            f = Fraction(0)
            for i in range(G):
                f = Fraction(float(_round_f32(Fraction(int(acc[i, m, n])) * Fraction(float(s_g[i])) + f)))
            asc[m, n] = np.float32(float(f))
            f = Fraction(0)
            for i in reversed(range(G)):
                f = Fraction(float(_round_f32(Fraction(int(acc[i, m, n])) * Fraction(float(s_g[i])) + f)))
            desc[m, n] = np.float32(float(f))
    for i in range(G):
        unfused = (unfused + acc[i].astype(np.float32) * s_g[i]).astype(np.float32)
    assert np.array_equal(out["f"], asc)
    assert not np.array_equal(asc, desc), "test data cannot tell the accumulation order"
    assert not np.array_equal(asc, unfused), "test data cannot tell fused from unfused accumulation"
    # last step: one fp32 multiply by the weight factor, one rounding to the storage type
    yf = (out["f"] * s_w[None, :]).astype(np.float32)
    assert np.array_equal(_val(out["y"], dtype), _val(wl.f32_to_storage_bits(yf, dtype), dtype))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_grouped_codes_are_per_channel_fakequant_codes(dtype):
    M, K, group = 9, 64, 8
    x = wl.random_bits(42, f"gcx{dtype}", (M, K), dtype, gain=3.0)
    s_g = (0.02 + 0.1 * wl.random_f32(42, "gcs", (K // group,), 1.0) ** 2).astype(np.float32)
    wq = wl.random_codes(42, "gcw", (5, K), -127, 127)
    out = oracle.static_linear_grouped(x, s_g, wq, np.ones(5, np.float32), None, group, 8, "int8", dtype)
    _, codes = oracle.fakequant_fwd_pc(x, np.repeat(s_g, group), 8, dtype)
    assert np.array_equal(out["xq"], codes)


@pytest.mark.parametrize("w_fmt", ["int8", "int4"])
def test_grouped_reduces_to_per_tensor(w_fmt):
    """(a) One group: f = fl32(acc * s) with the per-tensor oracle's accumulator.  (b) Equal
    power-of-two factors: every fp32 step is exact, so Y equals the per-tensor oracle's Y bit for bit."""
    M, N, K = 11, 13, 128
    dtype = "bf16"
    x = wl.random_bits(43, "grx", (M, K), dtype, gain=2.0)
    w = wl.random_f32(43, f"grw{w_fmt}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, w_fmt)
    bias = wl.random_f32(43, "grb", (N,), 0.4)
    s = np.float32(0.037)
    ref = oracle.static_linear(x, s, wq, s_w, None, 8, w_fmt, dtype)
    one = oracle.static_linear_grouped(x, np.array([s], np.float32), wq, s_w, None, K, 8, w_fmt, dtype)
    assert np.array_equal(one["xq"], ref["xq"])
    assert np.array_equal(one["f"], ref["acc"].astype(np.float32) * s)
    p2 = np.float32(2.0 ** -5)
    for b in (None, bias):
        ref = oracle.static_linear(x, p2, wq, s_w, b, 8, w_fmt, dtype)
        for group in (1, 2, 32, 64):
            out = oracle.static_linear_grouped(x, np.full(K // group, p2, np.float32), wq, s_w, b, group, 8, w_fmt, dtype)
            assert np.array_equal(out["y"], ref["y"]), group


@pytest.mark.parametrize("group", [1, 4, 32])
def test_grouped_vs_real_arithmetic(group):
    """Eq. 3 in float64 from the codes: Y = sum_k (s_g[k/group] q_k) (s_w w_k) + b, to half an
    output ulp plus the fp32 accumulation error of G steps."""
    M, N, K = 17, 19, 128
    dtype = "f16"
    G = K // group
    x = wl.random_bits(44, "gvx", (M, K), dtype, gain=2.0)
    w = wl.random_f32(44, "gvw", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, "int8")
    bias = wl.random_f32(44, "gvb", (N,), 0.5)
    s_g = (0.01 + 0.05 * wl.random_f32(44, f"gvs{group}", (G,), 1.0) ** 2).astype(np.float32)
    out = oracle.static_linear_grouped(x, s_g, wq, s_w, bias, group, 8, "int8", dtype)
    sk = np.repeat(s_g.astype(np.float64), group)
    q = out["xq"].astype(np.float64)
    exact_f = (q * sk[None, :]) @ wq.astype(np.float64).T
    mag = (np.abs(q) * sk[None, :]) @ np.abs(wq.astype(np.float64)).T
    assert (np.abs(out["f"].astype(np.float64) - exact_f) <= (G + 1) * 2.0 ** -24 * mag + 1e-30).all()
    exact = exact_f * s_w.astype(np.float64)[None, :] + bias.astype(np.float64)[None, :]
    yv = _val(out["y"], dtype)
    ulp = np.abs(_val((out["y"] + 1).astype(np.uint16), dtype) - yv)
    slack = (G + 3) * 2.0 ** -24 * (mag * s_w.astype(np.float64)[None, :] + np.abs(bias)[None, :])
    assert (np.abs(yv - exact) <= 0.5 * ulp + slack + 1e-30).all()


def test_grouped_rejects_bad_group():
    x = np.zeros((2, 8), np.uint16)
    wq = np.zeros((2, 8), np.int8)
    with pytest.raises(RuntimeError):
        oracle.static_linear_grouped(x, np.ones(2, np.float32), wq, np.ones(2, np.float32), None, 4, 9, "int8", "f16")
    with pytest.raises(AssertionError):
        oracle.static_linear_grouped(x, np.ones(2, np.float32), wq, np.ones(2, np.float32), None, 3, 8, "int8", "f16")
