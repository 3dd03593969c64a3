"""GPU parity at the full sizes of the five workload configurations, in the launch configuration
the benchmark times (MFMA path, no debug outputs for Y; int32 accumulators requested separately).

Fake-quant forward/backward and the activation codes are compared over the WHOLE tensor (the
oracle handles 2e8 elements in seconds).  The linear is compared on sampled output rows and
columns that the oracle computes one by one (all N outputs of a sampled token, all M outputs of a
sampled channel, always including the first/last row and column and tile-edge neighbours).
"""
from __future__ import annotations

import functools

import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import binding as B
from paper_2512_14481_amd import workloads as wl
from tests.gpu_util import TDT, assert_same_values, dev_scalar, set_tuning, to_bits, to_dev

pytestmark = pytest.mark.gpu

CASES_ACT = [(c.name, a.name) for c in wl.CONFIGS.values() for a in c.acts]
CASES_PROJ = [(c.name, p.name) for c in wl.CONFIGS.values() for p in c.projs]


@functools.lru_cache(maxsize=2)
def activation_bits(cfg_name: str, act_name: str) -> np.ndarray:
    return wl.activation(wl.CONFIGS[cfg_name], act_name)


@pytest.fixture(scope="module")
def ws():
    return B.new_workspace(1 << 20)


@pytest.mark.parametrize("cfg_name,act_name", CASES_ACT)
def test_fakequant_full_tensor(cfg_name, act_name, ws):
    cfg = wl.CONFIGS[cfg_name]
    dtype = cfg.dtype
    xb = activation_bits(cfg_name, act_name)
    proj = next(p for p in cfg.projs if p.x == act_name)
    dyb = wl.upstream_grad(cfg, proj.name)
    x, dy = to_dev(xb, dtype), to_dev(dyb, dtype)
    s_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.sasq_absmax_scale(x, s_dev, ws, 8)
    s0 = oracle.absmax_scale(xb, 8, dtype)
    assert np.float32(s_dev.item()) == s0, "absmax initial scale"
    y = torch.empty_like(x)
    dx = torch.empty_like(x)
    codes = torch.empty(x.shape, dtype=torch.int8, device="cuda")
    ds = torch.zeros(1, dtype=torch.float32, device="cuda")
    for s in (s0, np.float32(s0 / 4)):           # the init scale (nothing clips) and a trained-like one
        sd = dev_scalar(s)
        B.sasq_fakequant_fwd(x, sd, y, codes, 8)
        B.sasq_fakequant_bwd(x, dy, sd, dx, ds, ws, 8)
        torch.cuda.synchronize()
        y_ref, c_ref = oracle.fakequant_fwd(xb, s, 8, dtype)
        assert np.array_equal(codes.cpu().numpy(), c_ref), f"codes s={s}"
        assert_same_values(to_bits(y), y_ref, dtype, f"y s={s}", rel=1e-3)
        assert_same_values(to_bits(y), y_ref, dtype, f"y (exact) s={s}")
        ref = oracle.fakequant_bwd(xb, dyb, s, 8, dtype)
        assert_same_values(to_bits(dx), ref["dx"], dtype, f"dx s={s}")
        got = float(ds.item())
        assert abs(got - ref["ds64"]) <= 1e-4 * abs(ref["ds64"]), (s, got, ref["ds64"], ref["sum_abs"])
        if s == s0:
            assert np.array_equal(to_bits(dx), dyb), "nothing clips at the absmax scale: dx == dy"
        # the timed configuration: no codes output
        y2 = torch.empty_like(x)
        B.sasq_fakequant_fwd(x, sd, y2, None, 8)
        assert torch.equal(y2.view(torch.int16), y.view(torch.int16))
        ds2 = torch.zeros(1, dtype=torch.float32, device="cuda")
        B.sasq_fakequant_bwd(x, dy, sd, dx, ds2, ws, 8)
        assert ds2.view(torch.int32).item() == ds.view(torch.int32).item(), "ds is run-to-run reproducible"


def sample_indices(n: int, tile: int, count: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    fixed = [0, n - 1, min(tile - 1, n - 1), min(tile, n - 1), (n // tile) * tile - 1 if n >= tile else 0,
             min((n // tile) * tile, n - 1), n // 2]
    rnd = rng.integers(0, n, size=max(count - len(fixed), 0))
    return np.unique(np.array(fixed + rnd.tolist(), dtype=np.int64))


@pytest.mark.parametrize("cfg_name,proj_name", CASES_PROJ)
def test_static_linear_full_size(cfg_name, proj_name, ws):
    cfg = wl.CONFIGS[cfg_name]
    dtype, fmt = cfg.dtype, cfg.w_fmt
    proj = next(p for p in cfg.projs if p.name == proj_name)
    xb = activation_bits(cfg_name, proj.x)
    M, K, N = cfg.M, cfg.K_of(proj), proj.N
    wf = B.SASQ_W_INT8 if fmt == "int8" else B.SASQ_W_INT4_PACKED

    # frozen weights: quantized by the library on the device and by the oracle on the host
    w = wl.weight_fp32(cfg, proj.name)
    wq_ref, sw_ref = oracle.quantize_weight(w, fmt)
    wd = torch.from_numpy(w).cuda()
    wq = torch.empty(wq_ref.shape, dtype=torch.int8 if fmt == "int8" else torch.uint8, device="cuda")
    s_w = torch.empty(N, dtype=torch.float32, device="cuda")
    B.sasq_quantize_weight(wd, wq, s_w, wf)
    del wd, w
    assert np.array_equal(s_w.cpu().numpy(), sw_ref), "per-channel weight scales"
    assert np.array_equal(wq.cpu().numpy(), wq_ref), "weight codes"

    s = np.float32(oracle.absmax_scale(xb, 8, dtype) / 4)
    x = to_dev(xb, dtype)
    sd = dev_scalar(s)
    y = torch.empty((M, N), dtype=TDT[dtype], device="cuda")
    wsl = B.new_workspace(B.sasq_static_linear_workspace(M, N, K, wf))
    set_tuning()
    B.sasq_static_linear(x, sd, wq, s_w, None, y, wf, wsl)            # the timed configuration
    torch.cuda.synchronize()
    for path, mfma in (("twopass", None), ("twopass", "32x32x32"), ("fused", None)):   # every activation path and GEMM kernel agrees bit for bit
        set_tuning(path=path, mfma=mfma)
        y_alt = torch.empty_like(y)
        B.sasq_static_linear(x, sd, wq, s_w, None, y_alt, wf, wsl)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_alt.view(torch.int16)), (path, mfma)
    for tile in ("256", "128x256", "128"):                            # and every tile size
        set_tuning(tile=tile)
        B.sasq_static_linear(x, sd, wq, s_w, None, y_alt, wf, wsl)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_alt.view(torch.int16)), tile
    set_tuning()
    # the pre-arranged weight format (what the benchmark times): bit-identical at every tile size
    wfb = B.SASQ_W_INT8_BLOCKED if fmt == "int8" else B.SASQ_W_INT4_BLOCKED
    wpk = torch.empty(B.sasq_packed_weight_bytes(N, K, wfb), dtype=torch.uint8, device="cuda")
    B.sasq_pack_weight(wq, wpk, N, K, wf)
    for tile, mfma in ((None, None), ("256", None), ("128x256", None), ("128", None), (None, "32x32x32")):
        set_tuning(tile=tile, mfma=mfma)
        y_alt.fill_(0)
        B.sasq_static_linear(x, sd, wpk, s_w, None, y_alt, wfb, wsl)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_alt.view(torch.int16)), f"blocked weights, tile {tile}, mfma {mfma}"
    set_tuning()
    del y_alt, wpk
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    y_dbg = torch.empty_like(y)
    B.sasq_static_linear(x, sd, wq, s_w, None, y_dbg, wf, wsl, acc, xq)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_dbg.view(torch.int16))

    # every activation code
    _, c_ref = oracle.fakequant_fwd(xb, s, 8, dtype)
    assert np.array_equal(xq.cpu().numpy(), c_ref), "activation codes of the linear"
    del xq, c_ref

    rows = sample_indices(M, 256, 24, seed=1)
    cols = sample_indices(N, 256, 24, seed=2)
    ref_r = oracle.static_linear(np.ascontiguousarray(xb[rows]), s, wq_ref, sw_ref, None, 8, fmt, dtype, want_xq=False)
    assert np.array_equal(acc[torch.from_numpy(rows).cuda()].cpu().numpy(), ref_r["acc"]), "int32 accumulators (rows)"
    assert_same_values(to_bits(y[torch.from_numpy(rows).cuda()]), ref_r["y"], dtype, "Y rows", rel=1e-3)
    assert_same_values(to_bits(y[torch.from_numpy(rows).cuda()]), ref_r["y"], dtype, "Y rows (exact)")
    ref_c = oracle.static_linear(xb, s, np.ascontiguousarray(wq_ref[cols]), np.ascontiguousarray(sw_ref[cols]),
                                 None, 8, fmt, dtype, want_xq=False)
    ci = torch.from_numpy(cols).cuda()
    assert np.array_equal(acc[:, ci].cpu().numpy(), ref_c["acc"]), "int32 accumulators (columns)"
    assert_same_values(to_bits(y[:, ci].contiguous()), ref_c["y"], dtype, "Y columns (exact)")
    assert torch.isfinite(y.float()).all()


@pytest.mark.parametrize("cfg_name", ["c2_attn7b", "c3_mlp7b", "c4_w4a8_13b", "c5_layer70b"])
def test_batched_layer_calls_match_single_calls_full_size(cfg_name):
    """The launch configuration the benchmark times: every projection of the config through the
    batched fake-quant and batched linear entry points, against the single-tensor calls (which the
    tests above tie to the oracle): y, dx and Y bit-identical, ds within the reduction-order tolerance."""
    cfg = wl.CONFIGS[cfg_name]
    dt = TDT[cfg.dtype]
    wf_rm = B.SASQ_W_INT8 if cfg.w_fmt == "int8" else B.SASQ_W_INT4_PACKED
    wf = B.SASQ_W_INT8_BLOCKED if cfg.w_fmt == "int8" else B.SASQ_W_INT4_BLOCKED
    g = torch.Generator(device="cuda").manual_seed(17)
    M = cfg.M
    fq_fwd, fq_bwd, lin, singles = [], [], [], []
    n = len(cfg.projs)
    s_all = torch.empty(n, dtype=torch.float32, device="cuda")
    ds_all = torch.zeros(n, dtype=torch.float32, device="cuda")
    acts = {}                                           # projections on the same activation share the tensor, as in the benchmark
    for i, p in enumerate(cfg.projs):
        K, N = cfg.K_of(p), p.N
        if p.x not in acts:
            acts[p.x] = (torch.randn((M, K), device="cuda", generator=g) * 1.5).to(dt)
            acts[p.x][:, 7] *= 30                       # an outlier channel that clips
        x = acts[p.x]
        dy = torch.randn((M, K), device="cuda", generator=g).to(dt)
        s_all[i] = float(x.abs().max()) / 127 / (3 + 0.5 * i)     # a different factor for every projection
        if cfg.w_fmt == "int8":
            wq = torch.randint(-127, 128, (N, K), device="cuda", generator=g, dtype=torch.int8)
        else:
            wq = torch.randint(0, 256, (N, K // 2), device="cuda", generator=g, dtype=torch.uint8)
        pk = torch.empty(B.sasq_packed_weight_bytes(N, K, wf), dtype=torch.uint8, device="cuda")
        B.sasq_pack_weight(wq, pk, N, K, wf_rm)
        del wq
        s_w = torch.rand(N, device="cuda", generator=g) * 1e-3 + 1e-4
        y_b, dx_b = torch.empty_like(x), torch.empty_like(x)
        Y_b = torch.empty((M, N), dtype=dt, device="cuda")
        fq_fwd.append((x, s_all[i:i + 1], y_b))
        fq_bwd.append((x, dy, s_all[i:i + 1], dx_b, ds_all[i:i + 1]))
        lin.append((x, s_all[i:i + 1], pk, s_w, None, Y_b))
    ws_b = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(n))
    ws_l = B.new_workspace(B.sasq_static_linear_batch_workspace(lin, wf))
    B.sasq_fakequant_fwd_batch(fq_fwd, 8)
    B.sasq_fakequant_bwd_batch(fq_bwd, ws_b, 8)
    B.sasq_static_linear_batch(lin, wf, ws_l)
    torch.cuda.synchronize()
    ws1 = B.new_workspace(B.sasq_fakequant_bwd_workspace(1, 1))
    ds1 = torch.zeros(1, dtype=torch.float32, device="cuda")
    for i, p in enumerate(cfg.projs):
        x, s, y_b = fq_fwd[i]
        _, dy, _, dx_b, _ = fq_bwd[i]
        y1, dx1 = torch.empty_like(x), torch.empty_like(x)
        B.sasq_fakequant_fwd(x, s, y1, None, 8)
        B.sasq_fakequant_bwd(x, dy, s, dx1, ds1, ws1, 8)
        assert torch.equal(y1.view(torch.int16), y_b.view(torch.int16)), (p.name, "y")
        assert torch.equal(dx1.view(torch.int16), dx_b.view(torch.int16)), (p.name, "dx")
        a, b = float(ds1.item()), float(ds_all[i].item())
        assert abs(a - b) <= 1e-4 * abs(a) + 1e-2, (p.name, a, b)
        del y1, dx1
        _, _, pk, s_w, _, Y_b = lin[i]
        Y1 = torch.empty_like(Y_b)
        wsl = B.new_workspace(B.sasq_static_linear_workspace(M, p.N, cfg.K_of(p), wf))
        B.sasq_static_linear(x, s, pk, s_w, None, Y1, wf, wsl)
        torch.cuda.synchronize()
        assert torch.equal(Y1.view(torch.int16), Y_b.view(torch.int16)), (p.name, "Y")
        assert torch.isfinite(Y_b.float()).all()
        del Y1, wsl


@pytest.mark.parametrize("cfg_name", ["c3_mlp7b", "c4_w4a8_13b"])
def test_batched_layer_calls_against_the_oracle_full_size(cfg_name):
    """The configuration the benchmark times, tied to the oracle in one step: the config's own
    workload (seeded activations, gradients and weights, pre-arranged weight format) through the
    batched fake-quant and batched linear entry points; forward values and dx on sampled rows, ds of
    every operator, and Y on sampled rows and sampled columns against the oracle."""
    cfg = wl.CONFIGS[cfg_name]
    dtype, fmt = cfg.dtype, cfg.w_fmt
    dt = TDT[dtype]
    wf_rm = B.SASQ_W_INT8 if fmt == "int8" else B.SASQ_W_INT4_PACKED
    wf = B.SASQ_W_INT8_BLOCKED if fmt == "int8" else B.SASQ_W_INT4_BLOCKED
    M, n = cfg.M, len(cfg.projs)
    set_tuning()
    acts_b = {a.name: activation_bits(cfg_name, a.name) for a in cfg.acts}
    acts = {name: to_dev(b, dtype) for name, b in acts_b.items()}
    s_host = [np.float32(oracle.absmax_scale(acts_b[p.x], 8, dtype) / (3 + 0.5 * i)) for i, p in enumerate(cfg.projs)]
    s_all = torch.from_numpy(np.array(s_host, dtype=np.float32)).cuda()
    ds_all = torch.zeros(n, dtype=torch.float32, device="cuda")
    fq_fwd, fq_bwd, lin, dys, wrefs = [], [], [], [], []
    for i, p in enumerate(cfg.projs):
        K, N = cfg.K_of(p), p.N
        x = acts[p.x]
        dyb = wl.upstream_grad(cfg, p.name)
        dys.append(dyb)
        w = wl.weight_fp32(cfg, p.name)
        wq_ref, sw_ref = oracle.quantize_weight(w, fmt)
        wrefs.append((wq_ref, sw_ref))
        pk = torch.empty(B.sasq_packed_weight_bytes(N, K, wf), dtype=torch.uint8, device="cuda")
        B.sasq_pack_weight(torch.from_numpy(wq_ref).cuda(), pk, N, K, wf_rm)
        fq_fwd.append((x, s_all[i:i + 1], torch.empty_like(x)))
        fq_bwd.append((x, to_dev(dyb, dtype), s_all[i:i + 1], torch.empty_like(x), ds_all[i:i + 1]))
        lin.append((x, s_all[i:i + 1], pk, torch.from_numpy(sw_ref).cuda(), None, torch.empty((M, N), dtype=dt, device="cuda")))
        del w
    ws_b = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(n))
    ws_l = B.new_workspace(B.sasq_static_linear_batch_workspace(lin, wf))
    B.sasq_fakequant_fwd_batch(fq_fwd, 8)
    B.sasq_fakequant_bwd_batch(fq_bwd, ws_b, 8)
    B.sasq_static_linear_batch(lin, wf, ws_l)
    torch.cuda.synchronize()
    rows = sample_indices(M, 256, 16, seed=5)
    ri = torch.from_numpy(rows).cuda()
    for i, p in enumerate(cfg.projs):
        xb, s = acts_b[p.x], s_host[i]
        # fake-quant forward and backward: sampled rows element by element, ds over the whole tensor
        y_ref, _ = oracle.fakequant_fwd(np.ascontiguousarray(xb[rows]), s, 8, dtype)
        assert_same_values(to_bits(fq_fwd[i][2][ri]), y_ref, dtype, f"{p.name}: x' rows")
        b_all = oracle.fakequant_bwd(xb, dys[i], s, 8, dtype)
        assert_same_values(to_bits(fq_bwd[i][3][ri]), np.ascontiguousarray(b_all["dx"][rows]), dtype, f"{p.name}: dx rows")
        got, ref = float(ds_all[i].item()), float(b_all["ds64"])
        assert abs(got - ref) <= 1e-4 * abs(ref), (p.name, got, ref)
        del b_all
        # static linear: sampled rows against all columns, sampled columns against all rows
        wq_ref, sw_ref = wrefs[i]
        Y = lin[i][5]
        ref_r = oracle.static_linear(np.ascontiguousarray(xb[rows]), s, wq_ref, sw_ref, None, 8, fmt, dtype, want_xq=False)
        assert_same_values(to_bits(Y[ri]), ref_r["y"], dtype, f"{p.name}: Y rows")
        cols = sample_indices(p.N, 256, 12, seed=6 + i)
        ref_c = oracle.static_linear(xb, s, np.ascontiguousarray(wq_ref[cols]), np.ascontiguousarray(sw_ref[cols]),
                                     None, 8, fmt, dtype, want_xq=False)
        assert_same_values(to_bits(Y[:, torch.from_numpy(cols).cuda()].contiguous()), ref_c["y"], dtype, f"{p.name}: Y columns")


@pytest.mark.parametrize("per_channel", [False, True])
def test_fakequant_beyond_2_31_elements(per_channel, ws):
    """A tensor of 2.6e9 elements (flat indices beyond 2^31): forward and dx against the oracle on
    row slices at the start, across the 2^31-element boundary and at the end; ds against the sum
    of the same operator over eight row blocks (each below 2^31 elements)."""
    dtype = "bf16"
    rows, cols = 40000, 65544
    assert rows * cols > 2 ** 31
    g = torch.Generator(device="cuda").manual_seed(17)
    x = torch.empty((rows, cols), dtype=TDT[dtype], device="cuda")
    dy = torch.empty((rows, cols), dtype=TDT[dtype], device="cuda")
    step = 5000
    for r in range(0, rows, step):                     # filled block-wise: no fp32 copy of the whole tensor
        x[r:r + step] = (torch.randn((step, cols), device="cuda", generator=g) * 2).to(TDT[dtype])
        dy[r:r + step] = torch.randn((step, cols), device="cuda", generator=g).to(TDT[dtype])
    y, dx = torch.empty_like(x), torch.empty_like(x)
    if per_channel:
        s_np = (np.abs(wl.random_f32(17, "bigs", (cols,), 0.02)) + np.float32(0.02)).astype(np.float32)
        s = torch.from_numpy(s_np).cuda()
        ds = torch.empty(cols, dtype=torch.float32, device="cuda")
        wsp = B.new_workspace(B.sasq_fakequant_bwd_pc_workspace(rows, cols))
        B.sasq_fakequant_fwd_pc(x, s, y, None, 8)
        B.sasq_fakequant_bwd_pc(x, dy, s, dx, ds, wsp, 8)
    else:
        s_np = np.float32(0.03)
        s = dev_scalar(s_np)
        ds = torch.empty(1, dtype=torch.float32, device="cuda")
        B.sasq_fakequant_fwd(x, s, y, None, 8)
        B.sasq_fakequant_bwd(x, dy, s, dx, ds, ws, 8)
    torch.cuda.synchronize()
    edge = 2 ** 31 // cols                              # the row that holds flat index 2^31
    for r0 in (0, edge - 1, 2 ** 32 // cols // 2, rows - 3):
        sl = slice(r0, r0 + 3)
        xb, dyb = to_bits(x[sl]), to_bits(dy[sl])
        if per_channel:
            y_ref, _ = oracle.fakequant_fwd_pc(xb, s_np, 8, dtype)
            ref = oracle.fakequant_bwd_pc(xb, dyb, s_np, 8, dtype)
        else:
            y_ref, _ = oracle.fakequant_fwd(xb, s_np, 8, dtype)
            ref = oracle.fakequant_bwd(xb, dyb, s_np, 8, dtype)
        assert_same_values(to_bits(y[sl]), y_ref, dtype, f"y rows {r0}")
        assert_same_values(to_bits(dx[sl]), ref["dx"], dtype, f"dx rows {r0}")
    # ds: the whole-tensor reduction against eight separate reductions over row blocks
    total = np.zeros(ds.numel(), dtype=np.float64)
    for r in range(0, rows, step):
        part = torch.empty_like(ds)
        if per_channel:
            B.sasq_fakequant_bwd_pc(x[r:r + step], dy[r:r + step], s, None, part, wsp, 8)
        else:
            B.sasq_fakequant_bwd(x[r:r + step], dy[r:r + step], s, None, part, ws, 8)
        torch.cuda.synchronize()
        total += part.cpu().numpy().astype(np.float64)
    got = ds.cpu().numpy().astype(np.float64)
    # the two differ by summation order only: 1e-4 relative plus fp32 rounding noise scaled by an upper
    # bound of the sum of |terms| (every term is at most 128 |dy|); an indexing mistake is off by ~|ds|
    abs_dy = torch.zeros(cols, dtype=torch.float64, device="cuda")
    for r in range(0, rows, step):
        abs_dy += dy[r:r + step].abs().sum(dim=0, dtype=torch.float64)
    bound = 128.0 * (abs_dy.cpu().numpy() if per_channel else float(abs_dy.sum().item()))
    assert (np.abs(got - total) <= 1e-4 * np.abs(total) + 1e-6 * bound).all(), (np.abs(got - total).max(), np.abs(total).min())


@pytest.mark.parametrize("blocked", [False, True])
def test_static_linear_output_beyond_2_31_elements(blocked):
    """Y with 2.3e9 elements (flat output indices beyond 2^31), short K: sampled token rows on both
    sides of the 32-bit boundary against the oracle."""
    dtype = "f16"
    M, N, K = 70000, 32768, 64
    assert M * N > 2 ** 31
    xb = wl.random_bits(19, "bigx", (M, K), dtype, gain=2.0)
    wq, s_w = oracle.quantize_weight(wl.random_f32(19, "bigw", (N, K), 0.02), "int8")
    bias = wl.random_f32(19, "bigb", (N,), 0.3)
    s = np.float32(0.04)
    wf = B.SASQ_W_INT8
    wd = torch.from_numpy(wq).cuda()
    if blocked:
        packed = torch.empty(B.sasq_packed_weight_bytes(N, K, B.SASQ_W_INT8_BLOCKED), dtype=torch.uint8, device="cuda")
        B.sasq_pack_weight(wd, packed, N, K, B.SASQ_W_INT8)
        wd, wf = packed, B.SASQ_W_INT8_BLOCKED
    y = torch.empty((M, N), dtype=TDT[dtype], device="cuda")
    wsl = B.new_workspace(B.sasq_static_linear_workspace(M, N, K, wf))
    B.sasq_static_linear(to_dev(xb, dtype), dev_scalar(s), wd, torch.from_numpy(s_w).cuda(), torch.from_numpy(bias).cuda(),
                         y, wf, wsl)
    torch.cuda.synchronize()
    edge = 2 ** 31 // N
    rows = np.array([0, 1, edge - 1, edge, edge + 1, M - 2, M - 1])
    ref = oracle.static_linear(xb[rows], s, wq, s_w, bias, 8, "int8", dtype)
    assert_same_values(to_bits(y[torch.from_numpy(rows).cuda()]), ref["y"], dtype, "Y rows")


@pytest.mark.parametrize("blocked", [False, True])
def test_static_linear_activations_beyond_2_31_elements(blocked):
    """X (and the library's staged int8 copy of it) with 2.3e9 elements, few output channels: sampled
    token rows on both sides of the 32-bit boundary against the oracle."""
    dtype = "bf16"
    M, N, K = 70000, 64, 32768
    assert M * K > 2 ** 31
    g = torch.Generator(device="cuda").manual_seed(23)
    x = torch.empty((M, K), dtype=TDT[dtype], device="cuda")
    for r in range(0, M, 10000):
        x[r:r + 10000] = (torch.randn((10000, K), device="cuda", generator=g) * 2).to(TDT[dtype])
    wq, s_w = oracle.quantize_weight(wl.random_f32(23, "bigw2", (N, K), 0.02), "int8")
    s = np.float32(0.05)
    wf = B.SASQ_W_INT8
    wd = torch.from_numpy(wq).cuda()
    if blocked:
        packed = torch.empty(B.sasq_packed_weight_bytes(N, K, B.SASQ_W_INT8_BLOCKED), dtype=torch.uint8, device="cuda")
        B.sasq_pack_weight(wd, packed, N, K, B.SASQ_W_INT8)
        wd, wf = packed, B.SASQ_W_INT8_BLOCKED
    y = torch.empty((M, N), dtype=TDT[dtype], device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    wsl = B.new_workspace(B.sasq_static_linear_workspace(M, N, K, wf))
    B.sasq_static_linear(x, dev_scalar(s), wd, torch.from_numpy(s_w).cuda(), None, y, wf, wsl, acc, None)
    torch.cuda.synchronize()
    edge = 2 ** 31 // K
    rows = np.array([0, 1, edge - 1, edge, edge + 1, M - 2, M - 1])
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.static_linear(to_bits(x[idx]), s, wq, s_w, None, 8, "int8", dtype)
    assert np.array_equal(acc[idx].cpu().numpy(), ref["acc"])
    assert_same_values(to_bits(y[idx]), ref["y"], dtype, "Y rows")
