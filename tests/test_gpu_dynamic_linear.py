"""GPU parity of sasq_dynamic_linear (per-token factors computed on the fly) against the CPU
oracle: row factors, activation codes and int32 accumulators bit for bit, Y equal by value."""
from __future__ import annotations


import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import binding as B
from paper_2512_14481_amd import workloads as wl
from tests.gpu_util import TDT, assert_same_values, set_tuning, to_bits, to_dev
from tests.test_gpu_grouped_linear import WF, device_weights

pytestmark = pytest.mark.gpu


def run_dynamic(xb, wq, s_w, bias, fmt, dtype, blocked, want_debug=True, tile=None, mfma=None):
    set_tuning(tile=tile, mfma=mfma)
    M, K = xb.shape
    N = wq.shape[0]
    wf = WF[(fmt, blocked)]
    x = to_dev(xb, dtype)
    y = torch.empty((M, N), dtype=TDT[dtype], device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda") if want_debug else None
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda") if want_debug else None
    srow = torch.empty((M,), dtype=torch.float32, device="cuda") if want_debug else None
    ws = B.new_workspace(B.sasq_dynamic_linear_workspace(M, N, K, wf))
    B.sasq_dynamic_linear(x, device_weights(wq, fmt, blocked), torch.from_numpy(s_w).cuda(),
                          None if bias is None else torch.from_numpy(bias).cuda(), y, wf, ws, acc, xq, srow)
    torch.cuda.synchronize()
    set_tuning()
    if not want_debug:
        return to_bits(y), None, None, None
    return to_bits(y), acc.cpu().numpy(), xq.cpu().numpy(), srow.cpu().numpy()


def problem(seed, shape, dtype, fmt):
    M, N, K = shape
    xb = wl.random_bits(seed, f"dx{shape}{dtype}", (M, K), dtype, gain=2.0)
    if M > 2:
        xb[M // 2] = 0                         # an all-zero token
    w = wl.random_f32(seed, f"dw{shape}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, fmt)
    bias = wl.random_f32(seed, f"db{shape}", (N,), 0.3)
    return xb, wq, s_w, bias


SHAPES = [(1, 1, 2), (3, 5, 8), (19, 23, 70), (64, 256, 256), (1, 1, 128), (33, 47, 128), (300, 520, 384),
          (257, 255, 1024), (40, 300, 64)]


@pytest.mark.parametrize("tile", ["256", "128x256", "128"])
@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int4")])
@pytest.mark.parametrize("shape", SHAPES)
def test_dynamic_linear(shape, dtype, fmt, blocked, tile):
    if blocked and shape[2] % 64:
        pytest.skip("pre-arranged weights need K % 64 == 0")
    if shape[2] % 64 and tile != "256":
        pytest.skip("scalar path has no tiles")
    xb, wq, s_w, bias = problem(71, shape, dtype, fmt)
    for b in (None, bias):
        ref = oracle.dynamic_linear(xb, wq, s_w, b, 8, fmt, dtype)
        y, acc, xq, srow = run_dynamic(xb, wq, s_w, b, fmt, dtype, blocked, tile=tile)
        assert np.array_equal(srow, ref["s_row"]), "row factors"
        assert np.array_equal(xq, ref["xq"]), "activation codes"
        assert np.array_equal(acc, ref["acc"]), "int32 accumulators"
        assert_same_values(y, ref["y"], dtype, "Y")
        y2, _, _, _ = run_dynamic(xb, wq, s_w, b, fmt, dtype, blocked, want_debug=False, tile=tile)
        assert np.array_equal(y2, y)
        if fmt == "int8" and shape[2] % 64 == 0:       # the int8 GEMM's other kernel
            y3, acc3, _, _ = run_dynamic(xb, wq, s_w, b, fmt, dtype, blocked, tile=tile, mfma="32x32x32")
            assert np.array_equal(acc3, ref["acc"]) and np.array_equal(y3, y), "32x32x32 kernel"


def test_dynamic_linear_config3_sampled():
    """Config-3 down projection in the timed configuration; sampled rows against the oracle (a row's
    output depends on that row only) and sampled columns on all rows."""
    cfg = wl.CONFIGS["c3_mlp7b"]
    dtype, fmt = cfg.dtype, cfg.w_fmt
    proj = next(p for p in cfg.projs if p.name == "down")
    xb = wl.activation(cfg, proj.x)
    M, K, N = cfg.M, cfg.K_of(proj), proj.N
    wq, s_w = oracle.quantize_weight(wl.weight_fp32(cfg, proj.name), fmt)
    y, _, _, _ = run_dynamic(xb, wq, s_w, None, fmt, dtype, True, want_debug=False)
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([[0, M - 1, 255, 256], rng.integers(0, M, 12)]))
    cols = np.unique(np.concatenate([[0, N - 1, 255, 256], rng.integers(0, N, 12)]))
    ref_r = oracle.dynamic_linear(np.ascontiguousarray(xb[rows]), wq, s_w, None, 8, fmt, dtype)
    assert_same_values(y[rows], ref_r["y"], dtype, "Y rows")
    ref_c = oracle.dynamic_linear(xb, np.ascontiguousarray(wq[cols]), np.ascontiguousarray(s_w[cols]), None, 8, fmt, dtype)
    assert_same_values(np.ascontiguousarray(y[:, cols]), ref_c["y"], dtype, "Y columns")
