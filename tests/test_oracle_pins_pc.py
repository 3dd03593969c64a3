"""Pins for the per-channel oracle functions (no GPU): a hand-derived table, PyTorch autograd with
a broadcast scale vector, and the reduction to the (independently pinned) per-tensor functions,
column by column -- which is what catches a wrong scale-to-column assignment or a transposed loop."""
from __future__ import annotations

import os

import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _bits(v, dtype):
    return wl.f32_to_storage_bits(np.asarray(v, dtype=np.float32), dtype)


def _val(b, dtype):
    return wl.storage_bits_to_f32(b, dtype).astype(np.float64)


def test_hand_table_per_channel():
    d = {}
    with open(os.path.join(GOLD, "handtable_pc.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d.setdefault(k, []).append([float(t) for t in v])
    s = np.array(d["s"][0], dtype=np.float32)
    x = _bits(np.array(d["x"]), "f16")
    y, codes = oracle.fakequant_fwd_pc(x, s, 8, "f16")
    assert np.array_equal(codes, np.array(d["q"], dtype=np.int8))
    assert np.array_equal(_val(y, "f16"), np.array(d["xhat"]))
    b = oracle.fakequant_bwd_pc(x, _bits(np.ones((3, 3)), "f16"), s, 8, "f16")
    assert np.array_equal(_val(b["dx"], "f16"), np.array(d["dx"]))
    assert np.array_equal(b["ds64"], np.array(d["ds"][0]))
    assert np.array_equal(b["ds"], np.array(d["ds"][0], dtype=np.float32))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_per_channel_reduces_to_per_tensor_columnwise(dtype):
    rows, cols = 37, 21
    x = wl.random_bits(31, f"pcx{dtype}", (rows, cols), dtype, gain=3.0)
    dy = wl.random_bits(31, f"pcg{dtype}", (rows, cols), dtype)
    s = (np.abs(wl.random_f32(31, "pcs", (cols,), 0.05)) + 0.003).astype(np.float32)
    s[3] = -s[3]
    y, codes = oracle.fakequant_fwd_pc(x, s, 8, dtype)
    b = oracle.fakequant_bwd_pc(x, dy, s, 8, dtype)
    for k in range(cols):
        xc, gc = np.ascontiguousarray(x[:, k:k + 1]), np.ascontiguousarray(dy[:, k:k + 1])
        yk, ck = oracle.fakequant_fwd(xc, s[k], 8, dtype)
        assert np.array_equal(y[:, k:k + 1], yk) and np.array_equal(codes[:, k:k + 1], ck)
        bk = oracle.fakequant_bwd(xc, gc, s[k], 8, dtype)
        assert np.array_equal(b["dx"][:, k:k + 1], bk["dx"])
        assert b["ds64"][k] == bk["ds64"] and b["ds"][k] == bk["ds"]
    # equal scales everywhere: the column sums add up to the per-tensor gradient
    s1 = np.full(cols, 0.04, np.float32)
    assert abs(oracle.fakequant_bwd_pc(x, dy, s1, 8, dtype)["ds64"].sum()
               - oracle.fakequant_bwd(x, dy, np.float32(0.04), 8, dtype)["ds64"]) < 1e-9


def test_per_channel_backward_vs_autograd():
    dtype = "bf16"
    rows, cols = 29, 17
    x = wl.random_bits(33, "pcax", (rows, cols), dtype, gain=2.0)
    dy = wl.random_bits(33, "pcag", (rows, cols), dtype)
    s = np.array([2.0 ** -(3 + (k % 4)) for k in range(cols)], dtype=np.float32)   # powers of two: x/s exact
    xt = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).double().requires_grad_(True)
    st = torch.tensor(s.astype(np.float64), requires_grad=True)
    v = xt / st[None, :]
    yhat = st[None, :] * torch.clamp(v + (torch.round(v) - v).detach(), -128, 127)
    yhat.backward(torch.from_numpy(dy.view(np.int16).copy()).view(torch.bfloat16).double())
    b = oracle.fakequant_bwd_pc(x, dy, s, 8, dtype)
    assert np.array_equal(xt.grad.numpy(), _val(b["dx"], dtype))
    assert np.allclose(st.grad.numpy(), b["ds64"], rtol=0, atol=1e-10)
