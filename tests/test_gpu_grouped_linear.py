"""GPU parity of sasq_static_linear_grouped (Sec. 3, Eq. 3) against the CPU oracle: activation
codes and the fp32 group sums f bit for bit, Y equal by value; every weight format, both tiles,
the scalar fallback for shapes the MFMA kernel does not take; config-3 shapes on sampled rows."""
from __future__ import annotations


import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import binding as B
from paper_2512_14481_amd import workloads as wl
from tests.gpu_util import TDT, assert_same_values, set_tuning, to_bits, to_dev

pytestmark = pytest.mark.gpu

WF = {("int8", False): B.SASQ_W_INT8, ("int4", False): B.SASQ_W_INT4_PACKED,
      ("int8", True): B.SASQ_W_INT8_BLOCKED, ("int4", True): B.SASQ_W_INT4_BLOCKED}


def device_weights(wq, fmt, blocked):
    wd = torch.from_numpy(wq).cuda()
    if not blocked:
        return wd
    N = wq.shape[0]
    K = wq.shape[1] * (1 if fmt == "int8" else 2)
    packed = torch.empty(B.sasq_packed_weight_bytes(N, K, WF[(fmt, True)]), dtype=torch.uint8, device="cuda")
    B.sasq_pack_weight(wd, packed, N, K, WF[(fmt, False)])
    return packed


def run_grouped(xb, s_g, wq, s_w, bias, group, fmt, dtype, blocked, want_debug=True, tile=None):
    set_tuning(tile=tile)
    M, K = xb.shape
    N = wq.shape[0]
    wf = WF[(fmt, blocked)]
    x = to_dev(xb, dtype)
    y = torch.empty((M, N), dtype=TDT[dtype], device="cuda")
    f = torch.empty((M, N), dtype=torch.float32, device="cuda") if want_debug else None
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda") if want_debug else None
    ws = B.new_workspace(B.sasq_static_linear_workspace(M, N, K, wf))
    B.sasq_static_linear_grouped(x, torch.from_numpy(s_g).cuda(), device_weights(wq, fmt, blocked),
                                 torch.from_numpy(s_w).cuda(), None if bias is None else torch.from_numpy(bias).cuda(),
                                 y, group, wf, ws, f, xq)
    torch.cuda.synchronize()
    set_tuning()
    return to_bits(y), (f.cpu().numpy() if want_debug else None), (xq.cpu().numpy() if want_debug else None)


def problem(seed, shape, group, dtype, fmt):
    M, N, K = shape
    xb = wl.random_bits(seed, f"gx{shape}{dtype}", (M, K), dtype, gain=2.0)
    w = wl.random_f32(seed, f"gw{shape}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, fmt)
    bias = wl.random_f32(seed, f"gb{shape}", (N,), 0.3)
    s0 = float(oracle.absmax_scale(xb, 8, dtype))
    s_g = (s0 * (0.2 + 0.8 * wl.random_f32(seed, f"gs{shape}{group}", (K // group,), 1.0) ** 2)).astype(np.float32)
    return xb, wq, s_w, bias, s_g


MFMA_CASES = [((33, 47, 128), 64), ((256, 256, 128), 128), ((300, 520, 384), 128), ((257, 255, 1024), 256),
              ((130, 700, 512), 64), ((40, 300, 64), 64)]


@pytest.mark.parametrize("tile", ["128x256", "128"])
@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int4")])
@pytest.mark.parametrize("shape,group", MFMA_CASES)
def test_grouped_linear_mfma(shape, group, dtype, fmt, blocked, tile):
    xb, wq, s_w, bias, s_g = problem(51, shape, group, dtype, fmt)
    for b in (None, bias):
        ref = oracle.static_linear_grouped(xb, s_g, wq, s_w, b, group, 8, fmt, dtype)
        y, f, xq = run_grouped(xb, s_g, wq, s_w, b, group, fmt, dtype, blocked, tile=tile)
        assert np.array_equal(xq, ref["xq"]), "activation codes"
        assert np.array_equal(f.view(np.uint32), ref["f"].view(np.uint32)) or np.array_equal(f, ref["f"]), "fp32 group sums"
        assert_same_values(y, ref["y"], dtype, "Y")
        y2, _, _ = run_grouped(xb, s_g, wq, s_w, b, group, fmt, dtype, blocked, want_debug=False, tile=tile)
        assert np.array_equal(y2, y)


@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int4"), ("bf16", "int8")])
@pytest.mark.parametrize("shape", [(33, 47, 128), (256, 256, 64), (300, 520, 384), (257, 255, 1024), (130, 700, 320),
                                   (140, 150, 576), (140, 150, 704), (70, 260, 960)])   # K loop remainders of 5, 7, 7 tiles
def test_grouped_linear_groups_of_32(shape, dtype, fmt, blocked):
    """Groups of 32 channels, two per 64-byte K tile: the matrix-unit path multiplies every K tile twice, one half
    of the channels at a time.  Row-major int4 weights stay on the scalar kernel and are compared all the same."""
    xb, wq, s_w, bias, s_g = problem(53, shape, 32, dtype, fmt)
    ref = oracle.static_linear_grouped(xb, s_g, wq, s_w, bias, 32, 8, fmt, dtype)
    y, f, xq = run_grouped(xb, s_g, wq, s_w, bias, 32, fmt, dtype, blocked)
    assert np.array_equal(xq, ref["xq"]), "activation codes"
    assert np.array_equal(f.view(np.uint32), ref["f"].view(np.uint32)) or np.array_equal(f, ref["f"]), "fp32 group sums"
    assert_same_values(y, ref["y"], dtype, "Y")
    y2, _, _ = run_grouped(xb, s_g, wq, s_w, bias, 32, fmt, dtype, blocked, want_debug=False)
    assert np.array_equal(y2, y)


@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int4"), ("f16", "int4")])
@pytest.mark.parametrize("shape,group", [((3, 5, 8), 1), ((19, 23, 70), 7), ((19, 23, 70), 70), ((33, 47, 128), 1),
                                         ((33, 47, 128), 16), ((64, 256, 256), 32), ((1, 1, 2), 2)])
def test_grouped_linear_scalar_path(shape, group, dtype, fmt):
    xb, wq, s_w, bias, s_g = problem(52, shape, group, dtype, fmt)
    for b in (None, bias):
        ref = oracle.static_linear_grouped(xb, s_g, wq, s_w, b, group, 8, fmt, dtype)
        y, f, xq = run_grouped(xb, s_g, wq, s_w, b, group, fmt, dtype, False)
        assert np.array_equal(xq, ref["xq"])
        assert np.array_equal(f, ref["f"])
        assert_same_values(y, ref["y"], dtype, "Y")


def test_grouped_linear_rejects():
    x = torch.zeros((4, 128), dtype=torch.float16, device="cuda")
    y = torch.zeros((4, 4), dtype=torch.float16, device="cuda")
    one = torch.ones(128, dtype=torch.float32, device="cuda")
    wq = torch.zeros((16 * 128,), dtype=torch.uint8, device="cuda")
    ws = B.new_workspace(B.sasq_static_linear_workspace(4, 4, 128, 0))
    call = lambda group, wf: B._lib().sasq_static_linear_grouped(
        B._ptr(x), B._ptr(one), B._ptr(wq), B._ptr(one), None, B._ptr(y), None, None, 4, 4, 128, group, 8, wf, 0,
        B._ptr(ws), ws.numel(), None)
    assert call(3, 0) == 2          # group does not divide K
    assert call(0, 0) == 2
    assert call(16, 2) == 2         # pre-arranged weights need whole K tiles per group, or groups of 32
    assert call(64, 7) == 4


@pytest.mark.parametrize("proj_name,group", [("gate", 128), ("down", 256), ("up", 32)])
def test_grouped_linear_config3_sampled(proj_name, group):
    """Config-3 shapes in the configuration the benchmark times (pre-arranged int8 weights, no debug
    outputs); rows and columns sampled for the oracle, including tile edges."""
    cfg = wl.CONFIGS["c3_mlp7b"]
    dtype, fmt = cfg.dtype, cfg.w_fmt
    proj = next(p for p in cfg.projs if p.name == proj_name)
    xb = wl.activation(cfg, proj.x)
    M, K, N = cfg.M, cfg.K_of(proj), proj.N
    w = wl.weight_fp32(cfg, proj.name)
    wq, s_w = oracle.quantize_weight(w, fmt)
    del w
    G = K // group
    # one factor per group from that group's own absmax (what a per-channel calibration would give), shrunk so some clip
    xv = np.abs(wl.storage_bits_to_f32(xb, dtype)).reshape(M, G, group).max(axis=(0, 2))
    s_g = (np.maximum(xv, 1e-3) / 127.0 / 2.0).astype(np.float32)
    y, _, _ = run_grouped(xb, s_g, wq, s_w, None, group, fmt, dtype, True, want_debug=False)
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[0, M - 1, 127, 128, 255, 256], rng.integers(0, M, 10)]))
    cols = np.unique(np.concatenate([[0, N - 1, 127, 128, 255, 256, (N // 256) * 256 - 1], rng.integers(0, N, 10)]))
    ref_r = oracle.static_linear_grouped(np.ascontiguousarray(xb[rows]), s_g, wq, s_w, None, group, 8, fmt, dtype)
    assert_same_values(y[rows], ref_r["y"], dtype, "Y rows")
    ref_c = oracle.static_linear_grouped(xb, s_g, np.ascontiguousarray(wq[cols]), np.ascontiguousarray(s_w[cols]),
                                         None, group, 8, fmt, dtype)
    assert_same_values(np.ascontiguousarray(y[:, cols]), ref_c["y"], dtype, "Y columns")
