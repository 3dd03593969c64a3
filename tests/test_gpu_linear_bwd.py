"""GPU parity of the backward of the frozen quantized linear (sasq_prepare_bwd_weight,
sasq_linear_bwd_input) against the CPU oracle: the prepared 16-bit weight bit for bit, dX within
the fp32 accumulation bound of the exactly rounded result."""
from __future__ import annotations


import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import binding as B
from paper_2512_14481_amd import workloads as wl
from tests.gpu_util import TDT, set_tuning, to_bits, to_dev, val

pytestmark = pytest.mark.gpu

WF = {"int8": B.SASQ_W_INT8, "int4": B.SASQ_W_INT4_PACKED}


def unblock(raw: np.ndarray, N: int, K: int) -> np.ndarray:
    """Prepared weight bytes -> B[k][n] as uint16 [Kpad, Npad], following the layout the header states."""
    Kpad, Npad = (K + 15) // 16 * 16, (N + 31) // 32 * 32
    blocks = raw.view(np.uint16).reshape(Kpad // 16, Npad // 32, 16, 4, 8)   # kb, nb, row, position, element
    out = np.empty((Kpad, Npad), dtype=np.uint16)
    view = out.reshape(Kpad // 16, 16, Npad // 32, 32)
    for r in range(16):
        swz = ((r >> 1) & 3) ^ ((r >> 3) & 1)
        for c in range(4):
            view[:, r, :, 8 * c:8 * c + 8] = blocks[:, :, r, c ^ swz, :]
    return out


def prepare(wq, s_w, fmt, dtype):
    N = wq.shape[0]
    K = wq.shape[1] * (1 if fmt == "int8" else 2)
    wt = torch.empty(B.sasq_bwd_weight_bytes(N, K), dtype=torch.uint8, device="cuda")
    B.sasq_prepare_bwd_weight(torch.from_numpy(wq).cuda(), torch.from_numpy(s_w).cuda(), wt, N, K, WF[fmt], TDT[dtype])
    return wt, K


def run_bwd(dyb, wt, K, dtype, tile=None, want_acc=False, mfma=None):
    set_tuning(bwd_tile=tile, mfma=mfma)
    M = dyb.shape[0]
    dx = torch.empty((M, K), dtype=TDT[dtype], device="cuda")
    acc = torch.empty((M, K), dtype=torch.float32, device="cuda") if want_acc else None
    B.sasq_linear_bwd_input(to_dev(dyb, dtype), wt, dx, K, acc)
    torch.cuda.synchronize()
    set_tuning()
    if want_acc:
        return to_bits(dx), acc.cpu().numpy()
    return to_bits(dx)


def check_dx(got_bits, ref, dtype, N, what):
    """|dX_gpu - exact| <= half a 16-bit ulp of dX_gpu + N 2^-24 sum|terms| (fp32 accumulation in any
    order), and nearly all outputs are the exactly rounded ones."""
    g = val(got_bits, dtype)
    assert np.isfinite(g).all(), what
    ulp = np.abs(val((got_bits + 1).astype(np.uint16), dtype) - g)
    ulp = np.maximum(ulp, np.abs(val((got_bits - 1).astype(np.uint16), dtype) - g))
    bound = 0.5 * ulp * (1 + 2.0 ** -9) + N * 2.0 ** -24 * ref["sum_abs"] + 1e-45
    err = np.abs(g - ref["exact"])
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside the bound; worst {err[bad].max()} at {np.argwhere(bad)[0]}"
    same = (g == val(ref["dx"], dtype)).mean()
    assert same >= 0.95, f"{what}: only {same:.3f} of the outputs are the exactly rounded ones"


def problem(seed, shape, dtype, fmt):
    M, N, K = shape
    dyb = wl.random_bits(seed, f"bdy{shape}{dtype}", (M, N), dtype, gain=0.02)
    w = wl.random_f32(seed, f"bw{shape}", (N, K), 0.02)
    wq, s_w = oracle.quantize_weight(w, fmt)
    return dyb, wq, s_w


# (M, N = contraction, K = input channels): MFMA kernel when N is a multiple of 32 (M and K ragged),
# scalar kernel otherwise
SHAPES = [(1, 32, 2), (3, 32, 6), (19, 64, 70), (64, 256, 256), (33, 96, 48), (300, 384, 520),
          (257, 1024, 250), (130, 2048, 264), (513, 160, 136),
          (4, 1, 2), (5, 8, 4), (7, 40, 20), (33, 100, 18), (20, 250, 130)]


@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int8"), ("bf16", "int4"), ("f16", "int4")])
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("seed", [81, 82])
def test_prepared_weight_matches_oracle(seed, shape, dtype, fmt):
    # (seed 82, (64, 256, 256), f16, int8) holds a weight whose fp32 product w_int * s_w is an exact
    # fp16 tie while the exact product is not: the fp32 rounding must come first
    _, wq, s_w = problem(seed, shape, dtype, fmt)
    N, K = shape[1], shape[2]
    wt, K2 = prepare(wq, s_w, fmt, dtype)
    assert K2 == K
    got = unblock(wt.cpu().numpy(), N, K)
    ref = oracle.linear_bwd_input(np.zeros((1, N), np.uint16), wq, s_w, fmt, dtype)["wq16"]
    assert np.array_equal(got[:K, :N], ref.T)
    assert not got[K:].any() and not got[:, N:].any()


@pytest.mark.parametrize("mfma", ["16x16x64", "32x32x32"])      # the two GEMM kernels (16x16x32 and 32x32x16 MFMA tiles)
@pytest.mark.parametrize("tile", ["256", "128"])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int4")])
@pytest.mark.parametrize("shape", SHAPES)
def test_linear_bwd_matches_oracle(shape, dtype, fmt, tile, mfma):
    dyb, wq, s_w = problem(82, shape, dtype, fmt)
    wt, K = prepare(wq, s_w, fmt, dtype)
    ref = oracle.linear_bwd_input(dyb, wq, s_w, fmt, dtype)
    got, acc = run_bwd(dyb, wt, K, dtype, tile, want_acc=True, mfma=mfma)
    check_dx(got, ref, dtype, shape[1], f"{shape} {dtype} {fmt} tile {tile} {mfma}")
    # the fp32 sums before the 16-bit rounding: N fp32 additions in any order
    err = np.abs(acc.astype(np.float64) - ref["exact"])
    assert (err <= shape[1] * 2.0 ** -24 * ref["sum_abs"] + 1e-45).all(), err.max()
    # and dX is the rounding of exactly those sums
    assert np.array_equal(got, wl.f32_to_storage_bits(acc, dtype))
    assert np.array_equal(run_bwd(dyb, wt, K, dtype, tile), got)          # same without the inspection output


def test_linear_bwd_exact_on_small_integers():
    """Integer-valued dY and power-of-two weight factors: every product and partial sum is exact in
    fp32 whatever the order, so dX must equal the oracle bit for bit."""
    M, N, K = 70, 512, 200
    dyb = wl.f32_to_storage_bits(wl.random_codes(83, "idy", (M, N), -4, 4).astype(np.float32), "bf16")
    wq = wl.random_codes(83, "iw", (N, K), -7, 7).astype(np.int8)
    s_w = (np.float32(2.0) ** -wl.random_codes(83, "is", (N,), 0, 3).astype(np.float32)).astype(np.float32)
    wt, _ = prepare(wq, s_w, "int8", "bf16")
    ref = oracle.linear_bwd_input(dyb, wq, s_w, "int8", "bf16")
    for tile in ("256", "128"):
        got = run_bwd(dyb, wt, K, "bf16", tile)
        assert np.array_equal(val(got, "bf16"), val(ref["dx"], "bf16")), tile


@pytest.mark.parametrize("cfg_name,proj", [("c3_mlp7b", "gate"), ("c3_mlp7b", "down"), ("c5_layer70b", "o"),
                                           ("c4_w4a8_13b", "down")])
def test_linear_bwd_full_size_sampled_rows(cfg_name, proj):
    """Full LLaMA-2 projection sizes in the default launch configuration; the oracle computes a
    sample of dX rows (a row of dX depends on that row of dY only)."""
    cfg = wl.CONFIGS[cfg_name]
    p = next(q for q in cfg.projs if q.name == proj)
    M, N, K = cfg.M, p.N, cfg.K_of(p)
    dtype, fmt = cfg.dtype, cfg.w_fmt
    dyb = wl.random_bits(cfg.seed + 7, f"bwd{cfg_name}{proj}", (M, N), dtype, gain=0.01)
    wq, s_w = oracle.quantize_weight(wl.weight_fp32(cfg, proj), fmt)
    wt, _ = prepare(wq, s_w, fmt, dtype)
    got = run_bwd(dyb, wt, K, dtype)
    rows = np.array([0, 1, 255, 256, M // 2 + 1, M - 129, M - 2, M - 1])
    ref = oracle.linear_bwd_input(dyb[rows], wq, s_w, fmt, dtype)
    check_dx(got[rows], ref, dtype, N, f"{cfg_name}/{proj}")


def test_linear_bwd_output_beyond_2_31_elements():
    """dX with 2.3e9 elements (flat indices beyond 2^31), short contraction: sampled token rows on
    both sides of the 32-bit boundary against the oracle."""
    dtype, fmt = "bf16", "int8"
    M, N, K = 70000, 32, 32768
    assert M * K > 2 ** 31
    dyb = wl.random_bits(29, "bigdy", (M, N), dtype, gain=0.02)
    wq, s_w = oracle.quantize_weight(wl.random_f32(29, "bigwb", (N, K), 0.02), fmt)
    wt, _ = prepare(wq, s_w, fmt, dtype)
    dx = torch.empty((M, K), dtype=TDT[dtype], device="cuda")
    B.sasq_linear_bwd_input(to_dev(dyb, dtype), wt, dx, K)
    torch.cuda.synchronize()
    edge = 2 ** 31 // K
    rows = np.array([0, 1, edge - 1, edge, edge + 1, M - 2, M - 1])
    ref = oracle.linear_bwd_input(dyb[rows], wq, s_w, fmt, dtype)
    check_dx(to_bits(dx[torch.from_numpy(rows).cuda()]), ref, dtype, N, "rows across the boundary")
