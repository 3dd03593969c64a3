"""Pins for the CPU oracle (no GPU): each check ties an oracle function to something that is
not the oracle's own formula -- hand-derived tables, exact rational arithmetic, library float
conversions, int64 matmul, autograd of the straight-through surrogate, closed forms."""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import workloads as wl
from tests import exact_ref as ex

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _bits(vals, dtype):
    return wl.f32_to_storage_bits(np.asarray(vals, dtype=np.float32), dtype)


def _val(bits, dtype):
    return wl.storage_bits_to_f32(bits, dtype).astype(np.float64)


# ------------------------------------------------------------------ converters vs libraries
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_decode_matches_library(dtype):
    bits = wl.all_finite_patterns(dtype)
    got = oracle.decode16(bits, dtype)
    if dtype == "f16":
        ref = bits.view(np.float16).astype(np.float64)
    else:
        ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    assert np.array_equal(got, ref)
    assert np.array_equal(np.signbit(got), np.signbit(ref))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_encode_matches_library(dtype):
    rng = np.random.default_rng(1)
    # random bit patterns (all exponents), exact ties between neighbours, overflow edge, subnormals
    v = rng.integers(0, 1 << 32, size=400000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    v = v[np.isfinite(v)]
    pats = wl.all_finite_patterns(dtype)
    pats = pats[(pats & 0x7FFF) < (0x7C00 if dtype == "f16" else 0x7F80)]
    lo = _val(pats, dtype)
    hi = _val((pats + 1).astype(np.uint16), dtype)
    mids = ((lo + np.where(np.isfinite(hi), hi, lo)) / 2).astype(np.float32)
    extra = np.array([65504, 65519.99, 65520, 65536, 1e-8, 2.98e-8, 5.96e-8, 3.3895314e38, 3.4e38,
                      -65520, 0.0, -0.0, np.inf, -np.inf], dtype=np.float32)
    v = np.concatenate([v, mids, np.nextafter(mids, np.float32(np.inf)),
                        np.nextafter(mids, np.float32(-np.inf)), extra])
    got = oracle.encode16(v, dtype)
    if dtype == "f16":
        with np.errstate(over="ignore"):
            ref = v.astype(np.float16).view(np.uint16)
    else:
        ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)


def test_reciprocal_is_fp32_division():
    assert oracle.inv_scale(np.float32(0.1)).view(np.uint32) == 0x41200000   # fl32(1/0.1f) = 10.0f
    assert oracle.inv_scale(np.float32(0.5)) == np.float32(2.0)
    rng = np.random.default_rng(2)
    for s in np.exp(rng.uniform(np.log(1e-4), np.log(1e2), 500)).astype(np.float32):
        assert oracle.inv_scale(s) == np.float32(1.0) / s
        # correctly rounded: the fp32 result is the closest fp32 to the rational 1/s
        r = Fraction(float(oracle.inv_scale(s)))
        exact = 1 / Fraction(float(s))
        up = Fraction(float(np.nextafter(np.float32(r), np.float32(np.inf))))
        dn = Fraction(float(np.nextafter(np.float32(r), np.float32(-np.inf))))
        assert abs(r - exact) <= abs(up - exact) and abs(r - exact) <= abs(dn - exact)


# ------------------------------------------------------------------ hand tables
def _read_table(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        head = f.readline()
        meta = dict(kv.split("=") for kv in head.lstrip("# ").split() if "=" in kv)
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([float(t) for t in line.split()])
    return meta, np.array(rows, dtype=np.float64)


@pytest.mark.parametrize("name,ds_expected", [("handtable_b8_s0p5.txt", 126.212890625),
                                              ("handtable_b4_sneg2.txt", 0.25)])
def test_hand_table(name, ds_expected):
    meta, t = _read_table(name)
    bits, s, dtype = int(meta["bits"]), float(meta["s"]), meta["dtype"]
    Qn, Qp = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    x = _bits(t[:, 0], dtype)
    assert np.array_equal(_val(x, dtype), t[:, 1]), "fixture's own rounding of x"
    y, codes = oracle.fakequant_fwd(x, s, bits, dtype)
    assert np.array_equal(codes.astype(np.float64), t[:, 5])
    assert np.array_equal(_val(y, dtype), t[:, 6])
    dy = _bits(np.ones(len(t)), dtype)
    b = oracle.fakequant_bwd(x, dy, s, bits, dtype)
    assert np.array_equal(_val(b["dx"], dtype), t[:, 4])
    assert b["ds64"] == ds_expected == t[:, 7].sum()
    assert b["ds"] == np.float32(ds_expected)
    # the fixture is self-consistent with the rules it cites
    assert np.array_equal(np.clip(t[:, 3], Qn, Qp), t[:, 5])
    assert np.array_equal(((t[:, 3] >= Qn) & (t[:, 3] <= Qp)).astype(float), t[:, 4])
    # per-element terms: feed one-hot dy
    for i in range(len(t)):
        one = np.zeros(len(t), dtype=np.float32)
        one[i] = 1.0
        assert oracle.fakequant_bwd(x, _bits(one, dtype), s, bits, dtype)["ds64"] == t[i, 7]


def test_hand_table_discriminates_alternative_readings():
    """The rows that separate readings really do: the oracle's own switch for the STE-on-v
    reading changes exactly the half-unit-band row."""
    meta, t = _read_table("handtable_b8_s0p5.txt")
    x = _bits(t[:, 0], "f16")
    dy = _bits(np.ones(len(t)), "f16")
    alt = oracle.fakequant_bwd(x, dy, 0.5, 8, "f16", flags=oracle.STE_ON_V)
    base = oracle.fakequant_bwd(x, dy, 0.5, 8, "f16")
    diff = _val(alt["dx"], "f16") != _val(base["dx"], "f16")
    # v in (127, 127.5): rows 63.6 (127.1875) and 63.7 (127.375); v = -128.375, -128.5 on the low side
    assert list(np.nonzero(diff)[0]) == [4, 5, 8, 9]


# ------------------------------------------------------------------ exhaustive, exact rational
SCALES_EXACT = [0.5, 0.0123456789, -3.0e-3]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("s", SCALES_EXACT)
def test_codes_and_mask_vs_exact_rational(dtype, s):
    bits_all = wl.all_finite_patterns(dtype)
    # every 3rd pattern plus every pattern whose product lies within the clamp range +-2
    v = _val(bits_all, dtype) / float(np.float32(s))
    sel = (np.arange(bits_all.size) % 3 == 0) | (np.abs(v) < 131)
    bits = bits_all[sel] if dtype == "bf16" else bits_all[sel][::2]
    s32 = np.float32(s)
    y, codes = oracle.fakequant_fwd(bits, s32, 8, dtype)
    dy = _bits(np.ones(bits.size), dtype)
    dx = oracle.fakequant_bwd(bits, dy, s32, 8, dtype)["dx"]
    one = _bits([1.0], dtype)[0]
    n_ideal_diff = 0
    for i, b in enumerate(bits.tolist()):
        r, m, q, p = ex.quantize_exact(b, dtype, s32, 8)
        assert int(codes[i]) == q, (hex(b), s)
        assert (dx[i] == one) == bool(m), (hex(b), s)
        # forward value: one fp32 multiply then one RNE to the storage type
        yf = np.float32(q) * s32
        assert y[i] == wl.f32_to_storage_bits(np.array([yf]), dtype)[0] or \
            (_val(y[i:i + 1], dtype)[0] == 0 and float(yf) == 0)
        qi = ex.quantize_ideal(b, dtype, s32, 8)
        if qi is not None:
            assert abs(qi - q) <= 1
            n_ideal_diff += int(qi != q)
    # the reciprocal form is the real-number quantizer except at boundary cases
    assert n_ideal_diff <= max(1, int(2e-3 * bits.size)), n_ideal_diff


def test_ds_terms_vs_exact_rational():
    rng = np.random.default_rng(3)
    for dtype in ("f16", "bf16"):
        for s in (np.float32(0.037), np.float32(-1.7), np.float32(2.0 ** -6)):
            x = _bits(rng.standard_normal(300) * 6 * abs(float(s)) * 40, dtype)
            dy = _bits(rng.standard_normal(300), dtype)
            got = oracle.fakequant_bwd(x, dy, s, 8, dtype)
            total = Fraction(0)
            for xb, gb in zip(x.tolist(), dy.tolist()):
                r, m, q, p = ex.quantize_exact(xb, dtype, s, 8)
                total += ex.frac_of(gb, dtype) * (q - (p if m else 0))
            assert abs(Fraction(got["ds64"]) - total) <= abs(total) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 12)
            assert got["ds"] == np.float32(got["ds64"])


# ------------------------------------------------------------------ autograd second opinion
def _torch_x(bits, dtype):
    t = torch.from_numpy(bits.view(np.int16).copy())
    return t.view(torch.float16 if dtype == "f16" else torch.bfloat16).double()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("s", [0.25, 0.0371, -0.11])
def test_backward_vs_autograd_of_ste_surrogate(dtype, s):
    """d/ds and d/dx of  s * clamp(v + stopgrad(round(v) - v), Qn, Qp)  (Sec. 4.2, Eq. 4), by
    PyTorch autograd in fp64.  v = x * inv(s) with inv(s) entered as the first-order expansion of
    the reciprocal around the current scale, inv32 * (2 - s/s0): its value is exactly fl32(1/s0)
    (the reading adopted for x/s) and its derivative is -inv32/s0."""
    x = wl.random_bits(5, f"ag_x_{dtype}", (37, 129), dtype, gain=30 * abs(s))
    dy = wl.random_bits(5, f"ag_dy_{dtype}", (37, 129), dtype)
    s32 = np.float32(s)
    inv32 = float(np.float32(1.0) / s32)
    xt = _torch_x(x, dtype).requires_grad_(True)
    st = torch.tensor(float(s32), dtype=torch.float64, requires_grad=True)
    v = xt * (inv32 * (2.0 - st / float(s32)))
    u = v + (torch.round(v) - v).detach()          # torch.round is half-to-even
    yhat = st * torch.clamp(u, -128, 127)
    yhat.backward(_torch_x(dy, dtype))
    got = oracle.fakequant_bwd(x, dy, s32, 8, dtype)
    # dx: autograd multiplies dy by s * m * inv32 (= m up to the rounding of inv32); compare masks
    assert np.array_equal(xt.grad.numpy() != 0, _val(got["dx"], dtype) != 0) or \
        np.array_equal((xt.grad.numpy() != 0) | (_val(dy, dtype) == 0), (_val(got["dx"], dtype) != 0) | (_val(dy, dtype) == 0))
    assert np.allclose(xt.grad.numpy(), _val(got["dx"], dtype), rtol=1e-6, atol=0)
    assert abs(st.grad.item() - got["ds64"]) <= 1e-12 * got["sum_abs"]
    if s == 0.25:   # power of two: the plain quotient x/s is the same function, no expansion needed
        xt2 = _torch_x(x, dtype).requires_grad_(True)
        st2 = torch.tensor(0.25, dtype=torch.float64, requires_grad=True)
        v2 = xt2 / st2
        y2 = st2 * torch.clamp(v2 + (torch.round(v2) - v2).detach(), -128, 127)
        y2.backward(_torch_x(dy, dtype))
        assert np.array_equal(xt2.grad.numpy(), _val(got["dx"], dtype))
        assert abs(st2.grad.item() - got["ds64"]) <= 1e-12 * got["sum_abs"]


def test_backward_closed_forms():
    dtype = "f16"
    x = wl.random_bits(7, "cf_x", (64, 96), dtype, gain=3.0)
    xv = _val(x, dtype)
    # (i) s = absmax/Qp: nothing clips, dx == dy bit for bit, ds = sum dy*(r - p)
    s0 = oracle.absmax_scale(x, 8, dtype)
    assert s0 == np.float32(np.float32(np.abs(xv).max()) / np.float32(127.0))
    dy = wl.random_bits(7, "cf_dy", (64, 96), dtype)
    b = oracle.fakequant_bwd(x, dy, s0, 8, dtype)
    assert np.array_equal(b["dx"], dy)
    p = xv * float(np.float32(1.0) / s0)
    assert abs(b["ds64"] - (_val(dy, dtype) * (np.rint(p) - p)).sum()) < 1e-9
    # (ii) everything clips: dx == 0, ds = sum dy * (+-Q), exact with integer dy
    big = _bits(np.where(xv >= 0, 1.0, -1.0) * 500.0, dtype)
    dyi = _bits(np.rint(_val(dy, dtype) * 4), dtype)
    b = oracle.fakequant_bwd(big, dyi, np.float32(1.0), 8, dtype)
    assert not b["dx"].any()
    assert b["ds64"] == (_val(dyi, dtype) * np.where(xv >= 0, 127.0, -128.0)).sum()
    # (iii) on-grid inputs: x = k*s reproduces itself and contributes nothing to ds
    k = np.arange(-128, 128, dtype=np.float32)
    g = _bits(k * 0.125, dtype)
    y, codes = oracle.fakequant_fwd(g, np.float32(0.125), 8, dtype)
    assert np.array_equal(y, g) and np.array_equal(codes, k.astype(np.int8))
    assert oracle.fakequant_bwd(g, _bits(np.ones(256), dtype), np.float32(0.125), 8, dtype)["ds64"] == 0.0


# ------------------------------------------------------------------ invariants (Eq. 1)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantizer_invariants(dtype, bits):
    Qn, Qp = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    pats = wl.all_finite_patterns(dtype)
    xv = _val(pats, dtype)
    for s in (np.float32(0.5), np.float32(0.0173), np.float32(3.1)):
        y, codes = oracle.fakequant_fwd(pats, s, bits, dtype)
        c = codes.astype(np.int64)
        assert c.min() >= Qn and c.max() <= Qp
        order = np.argsort(xv, kind="stable")
        assert (np.diff(c[order]) >= 0).all(), "monotone in x for s > 0"
        fin = np.isfinite(xv)
        unclipped = fin & (np.abs(xv / float(s)) < Qp)
        err = np.abs(c * float(s) - xv)
        assert (err[unclipped] <= abs(float(s)) / 2 * (1 + 1e-6)).all()
        # idempotence: quantizing the fake-quantized tensor gives the same codes
        _, codes2 = oracle.fakequant_fwd(y, s, bits, dtype)
        assert np.array_equal(codes, codes2)
        # odd symmetry away from the asymmetric end
        neg = (pats ^ 0x8000).astype(np.uint16)
        _, cneg = oracle.fakequant_fwd(neg, s, bits, dtype)
        inner = (c > Qn) & (c < Qp)
        assert np.array_equal(cneg[inner].astype(np.int64), -c[inner])
        # negative scale: codes flip sign (inside the symmetric part), values agree
        yn, cn = oracle.fakequant_fwd(pats, -s, bits, dtype)
        assert np.array_equal(cn[inner].astype(np.int64), -c[inner])
        assert np.array_equal(_val(yn, dtype)[inner], _val(y, dtype)[inner])
    # infinities saturate and are masked out
    inf = _bits([np.inf, -np.inf], dtype)
    _, ci = oracle.fakequant_fwd(inf, np.float32(1.0), bits, dtype)
    assert list(ci) == [Qp, Qn]
    assert not oracle.fakequant_bwd(inf, _bits([1, 1], dtype), np.float32(1.0), bits, dtype)["dx"].any()


def test_ablation_switches():
    """Table 3's "w/o round" and "w/o clamp" variants as invariants."""
    dtype = "bf16"
    x = wl.random_bits(9, "abl", (50, 64), dtype, gain=2.0)
    xv = _val(x, dtype)
    s = np.float32(0.03125)
    y, _ = oracle.fakequant_fwd(x, s, 8, dtype, flags=oracle.NO_ROUND)
    unclipped = np.abs(xv / float(s)) <= 127
    assert np.array_equal(_val(y, dtype)[unclipped], xv[unclipped])   # power-of-two s: exact
    assert (np.abs(_val(y, dtype)[~unclipped]) <= 128 * float(s)).all()
    b = oracle.fakequant_bwd(x, x, s, 8, dtype, flags=oracle.NO_CLAMP)
    assert np.array_equal(b["dx"], x)                                 # m == 1 everywhere
    s2 = np.float32(0.1)
    y2 = oracle.encode16  # noqa: F841  (converter already pinned above)
    v = xv * float(np.float32(1.0) / s2)
    b2 = oracle.fakequant_bwd(x, _bits(np.ones(x.shape), dtype), s2, 8, dtype, flags=oracle.NO_CLAMP)
    assert abs(b2["ds64"] - (np.rint(v) - v).sum()) < 1e-9 and abs(b2["ds64"]) <= 0.5 * x.size


# ------------------------------------------------------------------ static linear (Eq. 2)
def test_int4_pack_and_hand_matmul():
    with open(os.path.join(GOLD, "int4_pack.txt")) as f:
        lines = [l.split() for l in f if not l.startswith("#") and l.strip()]
    d = {l[0]: l[1:] for l in lines}
    wq = np.array([int(b, 16) for b in d["bytes"]], dtype=np.uint8).reshape(2, 2)
    xcodes = np.array([int(v) for v in d["x"]], dtype=np.float32).reshape(2, 4)
    acc = np.array([int(v) for v in d["acc"]], dtype=np.int32).reshape(2, 2)
    x = _bits(xcodes, "f16")
    out = oracle.static_linear(x, np.float32(1.0), wq, np.ones(2, np.float32), None, 8, "int4", "f16")
    assert np.array_equal(out["xq"], xcodes.astype(np.int8))
    assert np.array_equal(out["acc"], acc)
    assert np.array_equal(_val(out["y"], "f16"), acc.astype(np.float64))
    # the weight quantizer packs the same way
    w = np.array([[7, -8, 1, -1], [-3, 0, 5, -6]], dtype=np.float32)
    w[0] *= 1.0  # row absmax 8 -> s_w = 8/7, codes round(w*7/8): not the table; use a scale-free row
    wq2, sw2 = oracle.quantize_weight(np.array([[7, -7, 1, -1], [-3.5, 0, 7, -7]], np.float32), "int4")
    assert np.array_equal(sw2, np.array([1.0, 1.0], np.float32))
    assert wq2.tolist() == [[0x97, 0xF1], [0x0C, 0x97]]   # -3.5 ties to even -> -4 = 0xC


@pytest.mark.parametrize("dtype,w_fmt", [("f16", "int8"), ("bf16", "int8"), ("bf16", "int4")])
def test_static_linear_vs_int64_matmul_and_fp64(dtype, w_fmt):
    M, N, K = 19, 23, 70
    x = wl.random_bits(11, f"sl_x_{dtype}", (M, K), dtype, gain=2.0)
    w = wl.random_f32(11, f"sl_w_{dtype}{w_fmt}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, w_fmt)
    bias = wl.random_f32(11, "sl_b", (N,), 0.5)
    s = np.float32(0.043)
    out = oracle.static_linear(x, s, wq, s_w, bias, 8, w_fmt, dtype)
    _, codes = oracle.fakequant_fwd(x, s, 8, dtype)
    assert np.array_equal(out["xq"], codes), "static linear quantizes exactly like fake-quant"
    if w_fmt == "int4":
        lo = (wq & 15).astype(np.int64)
        hi = (wq >> 4).astype(np.int64)
        w8 = np.empty((N, K), dtype=np.int64)
        w8[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
        w8[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    else:
        w8 = wq.astype(np.int64)
    ref_acc = codes.astype(np.int64) @ w8.T
    assert np.array_equal(out["acc"].astype(np.int64), ref_acc)
    # Eq. 2 in real arithmetic: Y = (s*q) . (Wq*s_w)^T + b, to half an output ulp (+ fp32 slack)
    exact = ref_acc.astype(np.float64) * float(s) * s_w.astype(np.float64)[None, :] + bias.astype(np.float64)
    yv = _val(out["y"], dtype)
    ulp = np.abs(_val((out["y"] + 1).astype(np.uint16), dtype) - yv)
    assert (np.abs(yv - exact) <= 0.5 * ulp * (1 + 2.0 ** -9) + 1e-30).all()
    # without bias and with the pinned operation order the result is reproducible by numpy fp32
    out2 = oracle.static_linear(x, s, wq, s_w, None, 8, w_fmt, dtype, want_acc=False, want_xq=False)
    c = (s * s_w).astype(np.float32)
    yf = ref_acc.astype(np.float32) * c[None, :]
    assert np.array_equal(out2["y"], wl.f32_to_storage_bits(yf, dtype)) or \
        np.array_equal(_val(out2["y"], dtype), _val(wl.f32_to_storage_bits(yf, dtype), dtype))


def test_static_linear_extremes_and_identity():
    # all-extreme codes: sign handling and int32 headroom at the largest K of the workloads
    K = 28672
    x = _bits(np.array([[-128.0] * K, [127.0] * K]), "bf16")
    wq = np.array([[-128] * K, [127] * K, [-127] * K], dtype=np.int8)
    out = oracle.static_linear(x, np.float32(1.0), wq, np.ones(3, np.float32), None, 8, "int8", "bf16")
    assert out["acc"].tolist() == [[128 * 128 * K, -128 * 127 * K, 128 * 127 * K],
                                   [-127 * 128 * K, 127 * 127 * K, -127 * 127 * K]]
    # W = 127*I, s_w = 1/127  =>  Y == fake-quant(x) up to the extra fp32 roundings
    Kd = 64
    xb = wl.random_bits(13, "id_x", (8, Kd), "f16", gain=1.5)
    s = np.float32(0.02)
    wI = (127 * np.eye(Kd)).astype(np.int8)
    out = oracle.static_linear(xb, s, wI, np.full(Kd, 1 / 127, np.float32), None, 8, "int8", "f16")
    yfq, _ = oracle.fakequant_fwd(xb, s, 8, "f16")
    a, b = _val(out["y"], "f16"), _val(yfq, "f16")
    assert (np.abs(a - b) <= 2.0 ** -10 * np.abs(b) + 1e-12).all()


# ------------------------------------------------------------------ weight quantizer, scale rule, SGD
def test_weight_quantizer_properties():
    w = wl.random_f32(17, "wq", (33, 130), 0.02)
    w[5] = 0.0                                             # zero row
    for fmt, Qp in (("int8", 127), ("int4", 7)):
        wq, s_w = oracle.quantize_weight(w, fmt)
        amax = np.abs(w).max(axis=1)
        ref_sw = np.where(amax == 0, np.float32(1.0), amax / np.float32(Qp)).astype(np.float32)
        assert np.array_equal(s_w, ref_sw)
        if fmt == "int4":
            lo, hi = (wq & 15).astype(np.int64), (wq >> 4).astype(np.int64)
            c = np.empty(w.shape, dtype=np.int64)
            c[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
            c[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
        else:
            c = wq.astype(np.int64)
        assert c.min() >= -Qp - 1 and c.max() <= Qp
        assert (np.abs(c).max(axis=1)[amax > 0] == Qp).all()
        assert not c[5].any()
        assert (np.abs(c * s_w[:, None].astype(np.float64) - w) <= s_w[:, None] / 2 * (1 + 1e-5)).all()
        # numpy fp64 evaluation of the same reading
        inv = (np.float32(1.0) / s_w).astype(np.float64)
        assert np.array_equal(c, np.clip(np.rint(w.astype(np.float64) * inv[:, None]), -Qp - 1, Qp).astype(np.int64))


def test_scale_sgd():
    assert oracle.scale_sgd(0.5, 126.212890625, 2e-4) == np.float32(0.5) - np.float32(2e-4) * np.float32(126.212890625)
    assert oracle.scale_sgd(1.0, 0.0, 0.1) == np.float32(1.0)


def test_oracle_independent_of_thread_count():
    x = wl.random_bits(19, "thr_x", (200, 64), "f16", gain=4.0)
    dy = wl.random_bits(19, "thr_dy", (200, 64), "f16")
    a = oracle.fakequant_bwd(x, dy, np.float32(0.05), 8, "f16")
    b = oracle.fakequant_bwd(x.reshape(200, 64), dy.reshape(200, 64), np.float32(0.05), 8, "f16")
    assert a["ds64"] == b["ds64"]


def test_epilogue_rounding_order_is_pinned():
    """Y = fl32(fl32(acc) * fl32(s * s_w[n])): find (by numpy fp32 arithmetic) accumulator / scale
    triples for which multiplying in the other order lands on a different fp16 value, build inputs
    that produce exactly those accumulators, and require the pinned order."""
    rng = np.random.default_rng(23)
    A = rng.integers(-60000, 60000, size=400000).astype(np.int64)
    s = np.float32(0.0437)
    sw = np.exp(rng.uniform(np.log(1e-4), np.log(1e-2), A.size)).astype(np.float32)
    af = A.astype(np.float32)
    pinned = (af * (s * sw).astype(np.float32)).astype(np.float32)
    other = ((af * s).astype(np.float32) * sw).astype(np.float32)
    hp, ho = wl.f32_to_storage_bits(pinned, "f16"), wl.f32_to_storage_bits(other, "f16")
    pick = np.flatnonzero(hp != ho)[:24]
    assert pick.size >= 8, "search found too few discriminating cases"
    # one output channel per case: N = len(pick), K = 8, a single token
    K = 8
    xcodes = np.array([127, -128, 90, -77, 64, 33, -5, 1], dtype=np.int64)
    N = pick.size
    wq = np.zeros((N, K), dtype=np.int8)
    for j, i in enumerate(pick):
        # greedy integer solve of sum_k xcodes[k] * w[k] = A[i] with |w| <= 127
        rest = int(A[i])
        for k in range(K):
            w = int(np.clip(round(rest / xcodes[k]), -127, 127)) if k < K - 1 else int(rest // xcodes[k])
            wq[j, k] = w
            rest -= w * int(xcodes[k])
        assert rest == 0 and -127 <= wq[j, K - 1] <= 127
    x = _bits((xcodes.astype(np.float32) * s)[None, :], "f16")
    out = oracle.static_linear(x, s, wq, sw[pick], None, 8, "int8", "f16")
    assert np.array_equal(out["xq"][0], xcodes.astype(np.int8))
    assert np.array_equal(out["acc"][0].astype(np.int64), A[pick])
    assert np.array_equal(out["y"][0], hp[pick])
    assert not np.array_equal(out["y"][0], ho[pick])


def test_adamw_matches_torch_optimizer():
    """The oracle's AdamW step against torch.optim.AdamW on fp64 CPU parameters (library routine)."""
    rng = np.random.default_rng(29)
    n = 17
    p0 = rng.uniform(0.01, 2.0, n).astype(np.float32)
    grads = [rng.standard_normal(n).astype(np.float32) * 50 for _ in range(4)]
    pt = torch.nn.Parameter(torch.tensor(p0.astype(np.float64)))
    opt = torch.optim.AdamW([pt], lr=2e-4, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for step, g in enumerate(grads, start=1):
        pt.grad = torch.tensor(g.astype(np.float64))
        opt.step()
        p, m, v = oracle.scale_adamw(p, g, m, v, step, 2e-4)
        assert np.allclose(p, pt.detach().numpy(), rtol=3e-7, atol=0), step   # fp32 state rounding only
    # first step from zero state moves every scale by ~lr against the gradient's sign
    p1, _, _ = oracle.scale_adamw(p0, grads[0], np.zeros(n, np.float32), np.zeros(n, np.float32), 1, 2e-4, wd=0.0)
    assert np.allclose(p1 - p0, -2e-4 * np.sign(grads[0]), rtol=1e-3, atol=1e-7)
