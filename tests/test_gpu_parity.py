"""GPU parity: the HIP library (through its C ABI via the ctypes binding) against the CPU oracle,
element by element, on seeded inputs small enough for the oracle to finish in seconds.

Bars: integer codes, int32 accumulators and dx bit-exact (dx by value for zeros); 16-bit outputs
within 1e-3 relative (asserted equal by value, which is stricter); ds within 1e-4 relative.
"""
from __future__ import annotations


import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import binding as B
from paper_2512_14481_amd import workloads as wl
from tests.gpu_util import (TDT, assert_same_values, dev_scalar, rel_err, set_tuning, to_bits, to_dev, val)

pytestmark = pytest.mark.gpu

SCALE_SET = [0.5, 2.0 ** -7, 0.0123456789, 0.0371, 3.1, -0.043, 1e-4, 97.0, 7.3e-6, 1.7e4]


@pytest.fixture(scope="module")
def ws():
    return B.new_workspace(1 << 20)


def run_fwd(x_bits, s, bits, dtype, want_codes=True):
    x = to_dev(x_bits, dtype)
    y = torch.empty_like(x)
    codes = torch.empty(x.shape, dtype=torch.int8, device="cuda") if want_codes else None
    B.sasq_fakequant_fwd(x, dev_scalar(s), y, codes, bits)
    torch.cuda.synchronize()
    return to_bits(y), (codes.cpu().numpy() if want_codes else None)


def run_bwd(x_bits, dy_bits, s, bits, dtype, ws, want_dx=True):
    x, dy = to_dev(x_bits, dtype), to_dev(dy_bits, dtype)
    dx = torch.empty_like(x) if want_dx else None
    ds = torch.full((1,), 12345.0, dtype=torch.float32, device="cuda")
    B.sasq_fakequant_bwd(x, dy, dev_scalar(s), dx, ds, ws, bits)
    torch.cuda.synchronize()
    return (to_bits(dx) if want_dx else None), np.float32(ds.item())


# ---------------------------------------------------------------- fake-quant, exhaustive inputs
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [8, 4, 2])
def test_fakequant_all_patterns(dtype, bits, ws):
    """Every finite 16-bit pattern (and +-inf) x a scale set: codes, y, dx, ds."""
    pats = wl.all_finite_patterns(dtype)
    x = pats.reshape(-1, 64) if pats.size % 64 == 0 else pats.reshape(1, -1)
    dy = wl.random_bits(3, f"dy_all_{dtype}", x.shape, dtype)
    for s in SCALE_SET:
        s32 = np.float32(s)
        y_ref, c_ref = oracle.fakequant_fwd(x, s32, bits, dtype)
        y, c = run_fwd(x, s32, bits, dtype)
        assert np.array_equal(c, c_ref), f"codes differ at s={s}"
        assert_same_values(y, y_ref, dtype, f"fwd y s={s}")
        y2, _ = run_fwd(x, s32, bits, dtype, want_codes=False)
        assert np.array_equal(y2, y)
        # backward: drop the infinities from ds (0 * inf style terms are not part of the contract)
        fin = np.isfinite(val(x, dtype))
        xb = np.where(fin, x, 0).astype(np.uint16)
        ref = oracle.fakequant_bwd(xb, dy, s32, bits, dtype)
        dx, ds = run_bwd(xb, dy, s32, bits, dtype, ws)
        assert_same_values(dx, ref["dx"], dtype, f"dx s={s}")
        assert abs(float(ds) - ref["ds64"]) <= 1e-4 * abs(ref["ds64"]) + 1e-7 * ref["sum_abs"], (s, ds, ref["ds64"])
        dxi, _ = run_bwd(x, dy, s32, bits, dtype, ws)
        assert_same_values(dxi, oracle.fakequant_bwd(x, dy, s32, bits, dtype)["dx"], dtype, f"dx(inf) s={s}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_reciprocal_is_correctly_rounded_on_device(dtype, ws):
    """x = 1, dy = 1: ds = round(inv_s) - inv_s exactly, which exposes every bit of the
    device's 1/s for |inv_s| < 128."""
    one = wl.f32_to_storage_bits(np.ones((1, 1), np.float32), dtype)
    rng = np.random.default_rng(5)
    for s in np.exp(rng.uniform(np.log(1 / 100), np.log(50.0), 64)).astype(np.float32):
        inv = np.float32(1.0) / s
        _, ds = run_bwd(one, one, s, 8, dtype, ws)
        assert np.float32(ds) == np.float32(np.rint(np.float64(inv)) - np.float64(inv)), (s, inv, ds)


# ---------------------------------------------------------------- fake-quant, shapes and tails
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1), (1, 7), (3, 5), (1, 8), (17, 33), (64, 256), (257, 1031),
                                   (1, 8 * 256 * 4), (1, 8 * 256 * 4 + 1), (513, 4099)])
def test_fakequant_shapes(dtype, shape, ws):
    x = wl.random_bits(7, f"x{shape}{dtype}", shape, dtype, gain=3.0)
    dy = wl.random_bits(7, f"dy{shape}{dtype}", shape, dtype)
    s0 = oracle.absmax_scale(x, 8, dtype)
    for s in (s0, np.float32(s0 / 4)):
        y_ref, c_ref = oracle.fakequant_fwd(x, s, 8, dtype)
        y, c = run_fwd(x, s, 8, dtype)
        assert np.array_equal(c, c_ref)
        assert_same_values(y, y_ref, dtype, "y")
        ref = oracle.fakequant_bwd(x, dy, s, 8, dtype)
        dx, ds = run_bwd(x, dy, s, 8, dtype, ws)
        assert_same_values(dx, ref["dx"], dtype, "dx")
        assert rel_err(float(ds), ref["ds64"]) <= 1e-4, (ds, ref["ds64"], ref["sum_abs"])
        _, ds_nodx = run_bwd(x, dy, s, 8, dtype, ws, want_dx=False)
        assert ds_nodx == ds


def _half_tie_cases(count=6):
    """(s, q) pairs for which the fp32 product q*s is exactly halfway between two fp16 values while
    the exact product is not: rounding the exact product once and rounding fl32(q*s) differ there."""
    from fractions import Fraction
    rng = np.random.default_rng(20250607)
    out = []
    while len(out) < count:
        s = np.float32(rng.uniform(0.01, 0.1))
        for q in range(3, 128):
            p32 = np.float32(q) * s                                  # numpy: one fp32 rounding
            lo = np.float16(p32)
            if float(lo) == float(p32):
                continue
            other = np.nextafter(lo, np.float16(np.inf) if float(p32) > float(lo) else np.float16(-np.inf))
            if Fraction(float(lo)) + Fraction(float(other)) != 2 * Fraction(float(p32)):
                continue                                             # not a tie
            exact = float(Fraction(q) * Fraction(float(s)))          # at most 31 significant bits: exact in a double
            if np.float16(exact) == lo:
                continue                                             # one rounding of the exact product agrees
            out.append((s, q))
            break
    return out


@pytest.mark.parametrize("shape", [(1, 7), (3, 5), (1, 8), (9, 1031), (64, 256)])
def test_fakequant_fp16_output_rounds_the_fp32_product(shape):
    """Y = round16(fl32(q * s)): the fp32 rounding comes first.  Inputs are chosen so that a fused
    multiply-and-narrow (one rounding of the exact product) would give the other neighbour; they are
    placed everywhere, so both the vector body and the scalar tail of the kernels meet them."""
    for s, q in _half_tie_cases():
        xv = np.full(shape, np.float32(q) * s, dtype=np.float32)
        xv[::2, ::3] *= -1
        x = wl.f32_to_storage_bits(xv, "f16")
        y_ref, c_ref = oracle.fakequant_fwd(x, s, 8, "f16")
        assert np.abs(c_ref).min() == q and np.abs(c_ref).max() == q
        y, c = run_fwd(x, s, 8, "f16")
        assert np.array_equal(c, c_ref)
        assert_same_values(y, y_ref, "f16", f"y s={s} q={q}")
        # per-channel factors: the same case in every column
        s_pc = np.full((shape[1],), s, dtype=np.float32)
        y_ref_pc, _ = oracle.fakequant_fwd_pc(x, s_pc, 8, "f16")
        assert np.array_equal(y_ref_pc, y_ref)
        xd = to_dev(x, "f16")
        yd = torch.empty_like(xd)
        B.sasq_fakequant_fwd_pc(xd, torch.from_numpy(s_pc).cuda(), yd, None, 8)
        torch.cuda.synchronize()
        assert_same_values(to_bits(yd), y_ref, "f16", f"per-channel y s={s} q={q}")


def test_fakequant_in_place_and_determinism(ws):
    dtype = "f16"
    xb = wl.random_bits(8, "inplace", (300, 1000), dtype, gain=2.0)
    dyb = wl.random_bits(8, "inplace_dy", (300, 1000), dtype)
    s = np.float32(0.01)
    y_ref, _ = oracle.fakequant_fwd(xb, s, 8, dtype)
    x = to_dev(xb, dtype)
    B.sasq_fakequant_fwd(x, dev_scalar(s), x, None, 8)
    assert_same_values(to_bits(x), y_ref, dtype, "in-place y")
    x = to_dev(xb, dtype)
    seen = set()
    for _ in range(5):
        dy = to_dev(dyb, dtype)
        ds = torch.zeros(1, dtype=torch.float32, device="cuda")
        B.sasq_fakequant_bwd(x, dy, dev_scalar(s), dy, ds, ws, 8)   # dx aliases dy
        torch.cuda.synchronize()
        seen.add((ds.view(torch.int32).item(), to_bits(dy).tobytes()))
    assert len(seen) == 1, "backward is not bit-reproducible"
    ref = oracle.fakequant_bwd(xb, dyb, s, 8, dtype)
    assert_same_values(np.frombuffer(next(iter(seen))[1], dtype=np.uint16).reshape(xb.shape), ref["dx"], dtype, "dx alias")


def test_uninitialised_workspace_is_loud():
    x = to_dev(wl.random_bits(9, "u", (4, 64), "f16"), "f16")
    junk = torch.full((1 << 16,), 0x5A, dtype=torch.uint8, device="cuda")
    ds = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.sasq_fakequant_bwd(x, x, dev_scalar(0.1), None, ds, junk, 8)
    torch.cuda.synchronize()
    assert torch.isnan(ds).item()


def test_scale_sgd_and_absmax(ws):
    for dtype in ("f16", "bf16"):
        for shape in ((1, 3), (64, 256), (129, 1001)):
            xb = wl.random_bits(10, f"am{shape}{dtype}", shape, dtype, gain=5.0)
            s = torch.zeros(1, dtype=torch.float32, device="cuda")
            for bits in (8, 4):
                B.sasq_absmax_scale(to_dev(xb, dtype), s, ws, bits)
                assert np.float32(s.item()) == oracle.absmax_scale(xb, bits, dtype)
    s = dev_scalar(0.5)
    ds = dev_scalar(126.212890625)
    B.sasq_scale_sgd(s, ds, 2e-4)
    assert np.float32(s.item()) == oracle.scale_sgd(0.5, 126.212890625, 2e-4)


# ---------------------------------------------------------------- weight quantizer
@pytest.mark.parametrize("fmt", ["int8", "int4"])
@pytest.mark.parametrize("shape", [(1, 2), (5, 34), (33, 130), (256, 4096), (7, 11008)])
def test_quantize_weight(fmt, shape):
    w = wl.random_f32(11, f"w{shape}", shape, 0.02)
    if shape[0] > 4:
        w[3] = 0.0
    wq_ref, sw_ref = oracle.quantize_weight(w, fmt)
    wd = torch.from_numpy(w).cuda()
    N, K = shape
    wq = torch.zeros((N, K if fmt == "int8" else K // 2), dtype=torch.int8 if fmt == "int8" else torch.uint8, device="cuda")
    sw = torch.zeros(N, dtype=torch.float32, device="cuda")
    B.sasq_quantize_weight(wd, wq, sw, B.SASQ_W_INT8 if fmt == "int8" else B.SASQ_W_INT4_PACKED)
    assert np.array_equal(sw.cpu().numpy(), sw_ref)
    assert np.array_equal(wq.cpu().numpy(), wq_ref)


# ---------------------------------------------------------------- static linear
def pack_on_device(wq, fmt):
    """Row-major codes (numpy) -> the library's blocked arrangement (device uint8 tensor)."""
    N = wq.shape[0]
    K = wq.shape[1] * (1 if fmt == "int8" else 2)
    src = B.SASQ_W_INT8 if fmt == "int8" else B.SASQ_W_INT4_PACKED
    dst = B.SASQ_W_INT8_BLOCKED if fmt == "int8" else B.SASQ_W_INT4_BLOCKED
    packed = torch.full((B.sasq_packed_weight_bytes(N, K, dst),), 0xA5, dtype=torch.uint8, device="cuda")
    B.sasq_pack_weight(torch.from_numpy(wq).cuda(), packed, N, K, src)
    return packed, dst


def run_linear(xb, s, wq, s_w, bias, fmt, dtype, want_debug=True, path=None, tile=None, blocked=False, a_bits=8, mfma=None):
    """path: None (library's choice by shape), "twopass" or "fused" (activation quantize in a
    separate pass / on load inside the GEMM).  tile: None (by shape), "256", "128x256", "128".
    mfma: None (library's choice), "32x32x32" or "16x16x64" (the int8 GEMM kernel).
    blocked: hand the weights over in the pre-arranged format made by sasq_pack_weight."""
    set_tuning(path=path, tile=tile, mfma=mfma)
    M, K = xb.shape
    N = wq.shape[0]
    wf = B.SASQ_W_INT8 if fmt == "int8" else B.SASQ_W_INT4_PACKED
    if blocked:
        wdev, wf = pack_on_device(wq, fmt)
    else:
        wdev = torch.from_numpy(wq).cuda()
    x = to_dev(xb, dtype)
    y = torch.empty((M, N), dtype=TDT[dtype], device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda") if want_debug else None
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda") if want_debug else None
    wsl = B.new_workspace(B.sasq_static_linear_workspace(M, N, K, wf))
    B.sasq_static_linear(x, dev_scalar(s), wdev, torch.from_numpy(s_w).cuda(),
                         None if bias is None else torch.from_numpy(bias).cuda(), y, wf, wsl, acc, xq, a_bits)
    torch.cuda.synchronize()
    set_tuning()
    return to_bits(y), (acc.cpu().numpy() if want_debug else None), (xq.cpu().numpy() if want_debug else None)


LINEAR_SHAPES = [
    (1, 1, 2), (3, 5, 8), (19, 23, 70),              # scalar path: K not a multiple of 128
    (64, 256, 256),                                   # config 1
    (1, 1, 128), (33, 47, 128), (256, 256, 128),      # MFMA path: single K step, ragged / exact tile
    (300, 520, 384), (257, 255, 1024), (512, 768, 512), (40, 300, 64), (260, 70, 192),
]


@pytest.mark.parametrize("tile", ["256", "128x256", "128"])
@pytest.mark.parametrize("path", ["twopass", "twopass-32x32x32", "fused"])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int8"), ("bf16", "int4"), ("f16", "int4")])
@pytest.mark.parametrize("shape", LINEAR_SHAPES)
def test_static_linear(shape, dtype, fmt, path, tile):
    M, N, K = shape
    mfma = None
    if path == "twopass-32x32x32":          # the int8 GEMM's other kernel (int4 weights have one kernel only)
        if fmt == "int4":
            pytest.skip("one GEMM kernel for int4 weights")
        path, mfma = "twopass", "32x32x32"
    xb = wl.random_bits(12, f"lx{shape}{dtype}", (M, K), dtype, gain=2.0)
    w = wl.random_f32(12, f"lw{shape}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, fmt)
    bias = wl.random_f32(12, f"lb{shape}", (N,), 0.3)
    s = np.float32(oracle.absmax_scale(xb, 8, dtype) / 3)
    for b in (None, bias):
        ref = oracle.static_linear(xb, s, wq, s_w, b, 8, fmt, dtype)
        y, acc, xq = run_linear(xb, s, wq, s_w, b, fmt, dtype, path=path, tile=tile, mfma=mfma)
        assert np.array_equal(xq, ref["xq"]), "activation codes"
        assert np.array_equal(acc, ref["acc"]), "int32 accumulators"
        assert_same_values(y, ref["y"], dtype, "Y")
        y2, _, _ = run_linear(xb, s, wq, s_w, b, fmt, dtype, want_debug=False, path=path, tile=tile, mfma=mfma)
        assert np.array_equal(y2, y)


def blocked_layout_reference(wq, fmt):
    """The documented blocked arrangements, written out index by index in numpy."""
    N = wq.shape[0]
    if fmt == "int8":
        K = wq.shape[1]
        KT = K // 64
        out = np.zeros(((N + 15) // 16 * 16) * K, dtype=np.uint8)
        src = wq.view(np.uint8)
        for n in range(N):
            r = n % 16
            sw = ((r >> 1) & 3) ^ ((r >> 3) & 1)
            for kb in range(KT):
                base = ((n // 16) * KT + kb) * 1024
                for c in range(4):
                    o = base + 16 * (4 * r + (c ^ sw))
                    out[o:o + 16] = src[n, kb * 64 + c * 16: kb * 64 + c * 16 + 16]
        return out
    K = wq.shape[1] * 2
    KT = K // 64
    codes = np.empty((N, K), dtype=np.uint8)
    codes[:, 0::2] = wq & 15
    codes[:, 1::2] = wq >> 4
    out = np.zeros(((N + 31) // 32 * 32) * (K // 2), dtype=np.uint8)
    for n in range(N):
        r = n % 32
        for kb in range(KT):
            base = ((n // 32) * KT + kb) * 1024
            for kk in range(2):
                for g in range(2):
                    c = codes[n, kb * 64 + 32 * kk + 16 * g: kb * 64 + 32 * kk + 16 * g + 16]
                    o = base + 512 * kk + 256 * g + 8 * r
                    for b in range(4):
                        out[o + b] = c[b] | (c[4 + b] << 4)
                        out[o + 4 + b] = c[8 + b] | (c[12 + b] << 4)
    return out


@pytest.mark.parametrize("fmt", ["int8", "int4"])
@pytest.mark.parametrize("shape", [(1, 64), (16, 64), (33, 192), (70, 128), (256, 256)])
def test_pack_weight_layout(fmt, shape):
    """sasq_pack_weight is the permutation the header documents, rows past N zero."""
    N, K = shape
    wq = (wl.random_codes(21, f"pk{shape}", (N, K), -128, 127) if fmt == "int8"
          else wl.random_codes(21, f"pk4{shape}", (N, K // 2), -128, 127).view(np.uint8))
    packed, _ = pack_on_device(wq, fmt)
    assert np.array_equal(packed.cpu().numpy(), blocked_layout_reference(wq, fmt))


def test_pack_weight_rejects_bad_shapes():
    wq = torch.zeros((4, 96), dtype=torch.int8, device="cuda")
    assert B.sasq_packed_weight_bytes(4, 96, B.SASQ_W_INT8_BLOCKED) == 0
    with pytest.raises(B.SasqError):
        B._check(B._lib().sasq_pack_weight(B._ptr(wq), B._ptr(wq), 4, 96, B.SASQ_W_INT8, None), "pack")
    x = torch.zeros((4, 96), dtype=torch.float16, device="cuda")
    y = torch.zeros((4, 4), dtype=torch.float16, device="cuda")
    one = torch.ones(4, dtype=torch.float32, device="cuda")
    rc = B._lib().sasq_static_linear(B._ptr(x), B._ptr(one), B._ptr(wq), B._ptr(one), None, B._ptr(y), None, None,
                                     4, 4, 96, 8, B.SASQ_W_INT8_BLOCKED, B.SASQ_F16, B._ptr(wq), 384, None)
    assert rc == 2


@pytest.mark.parametrize("tile", ["256", "128x256", "128"])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int8"), ("bf16", "int4"), ("f16", "int4")])
@pytest.mark.parametrize("shape", [sh for sh in LINEAR_SHAPES if sh[2] % 64 == 0])
def test_static_linear_blocked_weights(shape, dtype, fmt, tile):
    """Pre-arranged weights give the oracle's accumulators and outputs bit for bit."""
    M, N, K = shape
    xb = wl.random_bits(12, f"lx{shape}{dtype}", (M, K), dtype, gain=2.0)
    w = wl.random_f32(12, f"lw{shape}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, fmt)
    bias = wl.random_f32(12, f"lb{shape}", (N,), 0.3)
    s = np.float32(oracle.absmax_scale(xb, 8, dtype) / 3)
    for b in (None, bias):
        ref = oracle.static_linear(xb, s, wq, s_w, b, 8, fmt, dtype)
        y, acc, xq = run_linear(xb, s, wq, s_w, b, fmt, dtype, tile=tile, blocked=True)
        assert np.array_equal(xq, ref["xq"]), "activation codes"
        assert np.array_equal(acc, ref["acc"]), "int32 accumulators"
        assert_same_values(y, ref["y"], dtype, "Y")
        y2, _, _ = run_linear(xb, s, wq, s_w, b, fmt, dtype, want_debug=False, tile=tile, blocked=True)
        assert np.array_equal(y2, y)
        # the other GEMM kernel on the same pre-arranged weights
        y3, acc3, _ = run_linear(xb, s, wq, s_w, b, fmt, dtype, tile=tile, blocked=True, mfma="32x32x32")
        assert np.array_equal(acc3, ref["acc"]) and np.array_equal(y3, y), "32x32x32 kernel"


@pytest.mark.parametrize("tile", ["256", "128x256", "128"])
@pytest.mark.parametrize("k_tiles", [5, 7, 9, 10, 11, 13, 14, 15, 17, 22])
def test_static_linear_every_k_loop_remainder(k_tiles, tile):
    """The GEMM's K loop has a steady part of whole trips and a remainder of one to seven 64-channel
    tiles: every remainder, with and without a steady part, on row-major and pre-arranged weights of
    both widths (the other shapes in this file all leave a remainder of four)."""
    M, N, K = 150, 275, 64 * k_tiles
    for dtype, fmt, blocked in (("f16", "int8", True), ("bf16", "int8", False), ("bf16", "int4", True), ("f16", "int4", False)):
        xb = wl.random_bits(16, f"kx{k_tiles}{dtype}", (M, K), dtype, gain=2.0)
        w = wl.random_f32(16, f"kw{k_tiles}", (N, K), 0.02)
        wq, s_w = oracle.quantize_weight(w, fmt)
        s = np.float32(oracle.absmax_scale(xb, 8, dtype) / 3)
        ref = oracle.static_linear(xb, s, wq, s_w, None, 8, fmt, dtype)
        y, acc, xq = run_linear(xb, s, wq, s_w, None, fmt, dtype, tile=tile, blocked=blocked)
        assert np.array_equal(xq, ref["xq"]), "activation codes"
        assert np.array_equal(acc, ref["acc"]), "int32 accumulators"
        assert_same_values(y, ref["y"], dtype, "Y")


@pytest.mark.parametrize("a_bits", [4, 6, 2])
@pytest.mark.parametrize("path,blocked", [("twopass", False), ("fused", False), (None, True)])
def test_static_linear_low_bit_activations(a_bits, path, blocked):
    """Activation widths below 8 (codes still travel as int8): W8A4-style and W4A4-style linears."""
    M, N, K = 70, 90, 256
    for dtype, fmt in (("f16", "int8"), ("bf16", "int4")):
        xb = wl.random_bits(15, f"lbx{dtype}", (M, K), dtype, gain=2.0)
        w = wl.random_f32(15, "lbw", (N, K), 0.02)
        wq, s_w = oracle.quantize_weight(w, fmt)
        s = np.float32(oracle.absmax_scale(xb, a_bits, dtype) / 2)
        ref = oracle.static_linear(xb, s, wq, s_w, None, a_bits, fmt, dtype)
        y, acc, xq = run_linear(xb, s, wq, s_w, None, fmt, dtype, path=path, blocked=blocked, a_bits=a_bits)
        assert np.array_equal(xq, ref["xq"]) and np.array_equal(acc, ref["acc"])
        assert np.abs(xq.astype(np.int32)).max() <= 1 << (a_bits - 1)
        assert_same_values(y, ref["y"], dtype, "Y")


def test_static_linear_extreme_codes():
    """All-extreme codes at a long K: signs and int32 headroom through the MFMA path."""
    K = 28672
    xv = np.tile(np.array([[-128.0], [127.0], [-128.0]], dtype=np.float32), (1, K))
    xv[2, ::2] = 127.0
    xb = wl.f32_to_storage_bits(xv, "bf16")
    wq = np.stack([np.full(K, -128), np.full(K, 127), np.full(K, -127), np.where(np.arange(K) % 2, 127, -128)]).astype(np.int8)
    ref = oracle.static_linear(xb, np.float32(1.0), wq, np.ones(4, np.float32), None, 8, "int8", "bf16")
    assert ref["acc"][0, 0] == 128 * 128 * K
    for path in ("twopass", "fused"):
        y, acc, xq = run_linear(xb, np.float32(1.0), wq, np.ones(4, np.float32), None, "int8", "bf16", path=path)
        assert np.array_equal(acc, ref["acc"]) and np.array_equal(xq, ref["xq"])
        assert_same_values(y, ref["y"], "bf16", "Y")
    # int4 weights at their extremes (-8 and 7): the x16 in-register form must not overflow either
    w4 = np.stack([np.full(K // 2, 0x88), np.full(K // 2, 0x77), np.full(K // 2, 0x78)]).astype(np.uint8)
    ref4 = oracle.static_linear(xb, np.float32(1.0), w4, np.ones(3, np.float32), None, 8, "int4", "bf16")
    assert ref4["acc"][0, 0] == 128 * 8 * K
    for path in ("twopass", "fused"):
        y, acc, xq = run_linear(xb, np.float32(1.0), w4, np.ones(3, np.float32), None, "int4", "bf16", path=path)
        assert np.array_equal(acc, ref4["acc"])
        assert_same_values(y, ref4["y"], "bf16", "Y int4")
    # and through the pre-arranged formats
    y, acc, _ = run_linear(xb, np.float32(1.0), wq, np.ones(4, np.float32), None, "int8", "bf16", blocked=True)
    assert np.array_equal(acc, ref["acc"])
    y, acc, _ = run_linear(xb, np.float32(1.0), w4, np.ones(3, np.float32), None, "int4", "bf16", blocked=True)
    assert np.array_equal(acc, ref4["acc"])
    assert_same_values(y, ref4["y"], "bf16", "Y int4 blocked")


@pytest.mark.parametrize("K", [131008, 131070, 131071])
def test_static_linear_maximum_K(K):
    """The longest contraction the library accepts (K <= 131071 keeps K * 128 * 128 inside int32),
    all codes at the extremes: 131008 runs the MFMA kernels (and the x16 in-register form of int4
    weights ends 1 MiB short of 2^31), 131070 / 131071 the scalar kernel.  One more is refused."""
    xv = np.tile(np.array([[-128.0], [127.0]], dtype=np.float32), (1, K))
    xb = wl.f32_to_storage_bits(xv, "f16")
    ones = np.ones(2, np.float32)
    wq = np.stack([np.full(K, -128), np.full(K, 127)]).astype(np.int8)
    ref = oracle.static_linear(xb, np.float32(1.0), wq, ones, None, 8, "int8", "f16")
    assert ref["acc"][0, 0] == 128 * 128 * K and ref["acc"][0, 0] < 2 ** 31
    variants = [dict(path="twopass"), dict(path="fused")] + ([dict(blocked=True)] if K % 64 == 0 else [])
    for kw in variants:
        y, acc, xq = run_linear(xb, np.float32(1.0), wq, ones, None, "int8", "f16", **kw)
        assert np.array_equal(acc, ref["acc"]) and np.array_equal(xq, ref["xq"]), kw
        assert_same_values(y, ref["y"], "f16", f"Y {kw}")
    if K % 2 == 0:
        w4 = np.stack([np.full(K // 2, 0x88), np.full(K // 2, 0x77)]).astype(np.uint8)
        ref4 = oracle.static_linear(xb, np.float32(1.0), w4, ones, None, 8, "int4", "f16")
        assert ref4["acc"][0, 0] == 128 * 8 * K
        for kw in variants:
            y, acc, _ = run_linear(xb, np.float32(1.0), w4, ones, None, "int4", "f16", **kw)
            assert np.array_equal(acc, ref4["acc"]), kw
            assert_same_values(y, ref4["y"], "f16", f"Y int4 {kw}")
    x = to_dev(xb, "f16")
    ws = B.new_workspace(1 << 20)
    with pytest.raises(B.SasqError) as e:
        B._check(B._lib().sasq_static_linear(B._ptr(x), B._ptr(dev_scalar(1.0)), B._ptr(x), B._ptr(x), None, B._ptr(x), None, None,
                                             2, 2, 131072, 8, 0, 0, B._ptr(ws), 1 << 20, None), "K too long")
    assert e.value.status == 2


def test_cross_export_identity():
    """xq of the linear == codes of fake-quant, and Y ~ fakequant(x) . (Wq*s_w)^T (Eq. 2 <=> Eq. 5)."""
    dtype = "f16"
    M, N, K = 96, 80, 256
    xb = wl.random_bits(13, "cx", (M, K), dtype, gain=2.0)
    w = wl.random_f32(13, "cw", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, "int8")
    s = np.float32(0.05)
    y, acc, xq = run_linear(xb, s, wq, s_w, None, "int8", dtype)
    yfq, codes = run_fwd(xb, s, 8, dtype)
    assert np.array_equal(xq, codes)
    exact = (codes.astype(np.float64) * float(s)) @ (wq.astype(np.float64) * s_w[:, None].astype(np.float64)).T
    yv = val(y, dtype)
    assert (np.abs(yv - exact) <= 2.0 ** -10 * np.abs(exact) + 1e-6).all()


def test_scale_adamw():
    rng = np.random.default_rng(31)
    for n in (1, 7, 4096, 11008):
        p = rng.uniform(0.01, 2.0, n).astype(np.float32)
        m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
        pd, md, vd = (torch.from_numpy(a.copy()).cuda() for a in (p, m, v))
        for step in range(1, 5):
            g = (rng.standard_normal(n) * 30).astype(np.float32)
            B.sasq_scale_adamw(pd, torch.from_numpy(g).cuda(), md, vd, step, 2e-4)
            p, m, v = oracle.scale_adamw(p, g, m, v, step, 2e-4)
            # fp32 kernel against the fp64-evaluated oracle: a handful of fp32 roundings
            assert np.allclose(pd.cpu().numpy(), p, rtol=2e-6, atol=0)
            # the moments are sums of two terms that may cancel: absolute slack scaled by the terms
            assert np.allclose(md.cpu().numpy(), m, rtol=2e-6, atol=2e-7 * float(np.abs(g).max()))
            assert np.allclose(vd.cpu().numpy(), v, rtol=2e-6, atol=1e-30)
            # keep both sides on the same state so that differences do not accumulate
            pd.copy_(torch.from_numpy(p)); md.copy_(torch.from_numpy(m)); vd.copy_(torch.from_numpy(v))


def test_mfma_probe_runs_and_validates():
    """The register-only MFMA loop the benchmark times (its own small library, not part of the C ABI):
    runs, writes its sink, rejects bad arguments."""
    import bench
    probe = bench.load_probe()
    stream = None
    sink = torch.full((65536,), 7, dtype=torch.int32, device="cuda")
    ptr = sink.data_ptr()
    torch.cuda.synchronize()
    assert probe(0, 3, ptr, stream) == 0                   # zero operands: every accumulator stays zero
    torch.cuda.synchronize()
    assert int(sink.abs().max()) == 0
    sink.fill_(7)
    assert probe(5, 3, ptr, stream) == 0                   # the 16x16x64 form on zero operands
    torch.cuda.synchronize()
    assert int(sink.abs().max()) == 0
    for kind in (1, 2, 3, 4):
        assert probe(kind, 2, ptr, stream) == 0
    torch.cuda.synchronize()
    # kind 2, 2 iterations: each accumulator element is 2 * sum_k a*b with |a| <= 1, |b| <= 32 over 32 k: bounded
    assert probe(2, 2, ptr, stream) == 0
    torch.cuda.synchronize()
    assert int(sink.abs().max()) <= 2 * 32 * 32 * 256
    assert probe(9, 2, ptr, stream) != 0
    assert probe(0, 0, ptr, stream) != 0
