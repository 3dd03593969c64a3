"""GPU parity of the batched fake-quant entry points: outputs bit-identical to the single-tensor
calls (and so to the oracle), ds within the single-tensor tolerance of the oracle, deterministic."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import binding as B
from paper_2512_14481_amd import workloads as wl
from tests.gpu_util import TDT, dev_scalar, rel_err, to_bits, to_dev

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1), (3, 5), (17, 33), (64, 256), (257, 1031), (512, 4096), (1, 8192), (300, 7)]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("count", [1, 3, 8])
def test_batch_matches_single_calls_and_oracle(dtype, count):
    shapes = SHAPES[:count]
    xs = [wl.random_bits(81, f"bx{sh}{dtype}", sh, dtype, gain=2.0) for sh in shapes]
    dys = [wl.random_bits(81, f"bd{sh}{dtype}", sh, dtype, gain=1.0) for sh in shapes]
    ss = [np.float32(oracle.absmax_scale(x, 8, dtype) / (2 + i)) for i, x in enumerate(xs)]
    xd = [to_dev(x, dtype) for x in xs]
    dyd = [to_dev(d, dtype) for d in dys]
    sd = torch.tensor([float(s) for s in ss], dtype=torch.float32, device="cuda")
    yd = [torch.empty_like(x) for x in xd]
    dxd = [torch.empty_like(x) if i != 1 else None for i, x in enumerate(xd)]      # one item without dx
    dsd = torch.full((count,), float("nan"), dtype=torch.float32, device="cuda")
    ws = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(count))
    B.sasq_fakequant_fwd_batch([(xd[i], sd[i:i + 1], yd[i]) for i in range(count)], 8)
    items = [(xd[i], dyd[i], sd[i:i + 1], dxd[i], dsd[i:i + 1]) for i in range(count)]
    B.sasq_fakequant_bwd_batch(items, ws, 8)
    ds1 = dsd.cpu().numpy().copy()
    B.sasq_fakequant_bwd_batch(items, ws, 8)                                       # same workspace, second call
    torch.cuda.synchronize()
    assert np.array_equal(dsd.cpu().numpy(), ds1), "ds is deterministic and the tickets were reset"
    for i in range(count):
        y_ref, _ = oracle.fakequant_fwd(xs[i], ss[i], 8, dtype)
        ref = oracle.fakequant_bwd(xs[i], dys[i], ss[i], 8, dtype)
        assert np.array_equal(wl.storage_bits_to_f32(to_bits(yd[i]), dtype), wl.storage_bits_to_f32(y_ref, dtype)), i
        if dxd[i] is not None:
            assert np.array_equal(wl.storage_bits_to_f32(to_bits(dxd[i]), dtype), wl.storage_bits_to_f32(ref["dx"], dtype)), i
        tol = 1e-4 * abs(ref["ds64"]) + 1e-7 * ref["sum_abs"] + 1e-30
        assert abs(float(ds1[i]) - ref["ds64"]) <= tol, (i, ds1[i], ref["ds64"])


def test_batch_sgd_vec_and_errors():
    s = torch.tensor([0.5, 0.25, 2.0], dtype=torch.float32, device="cuda")
    ds = torch.tensor([126.212890625, -3.0, 0.0], dtype=torch.float32, device="cuda")
    B.sasq_scale_sgd_vec(s, ds, 2e-4)
    ref = [oracle.scale_sgd(a, b, 2e-4) for a, b in ((0.5, 126.212890625), (0.25, -3.0), (2.0, 0.0))]
    assert np.array_equal(s.cpu().numpy(), np.array(ref, dtype=np.float32))
    x = torch.zeros((4, 8), dtype=torch.float16, device="cuda")
    with pytest.raises(ValueError):
        B.sasq_fakequant_fwd_batch([], 8)
    arr, dt = B._fq_items([(x, s[:1], x)], False)
    assert B._lib().sasq_fakequant_fwd_batch(arr, 0, 8, dt, None) == 2
    assert B._lib().sasq_fakequant_fwd_batch(arr, 9, 8, dt, None) == 2
    assert B._lib().sasq_fakequant_fwd_batch(arr, 1, 9, dt, None) == 4
    assert B._lib().sasq_fakequant_bwd_batch(arr, 1, 8, dt, None, 0, None) == 1     # dy / ds missing


def test_batch_larger_than_one_launch_matches_single_calls():
    """Seven tensors of config 4's sizes (365 MB of inputs: the library cuts the batch into several
    launches): outputs bit-identical to the single-tensor calls, ds equal to theirs within the
    reduction-order tolerance, every item's ticket reset for the next call."""
    dtype = "bf16"
    shapes = [(4096, 5120)] * 6 + [(4096, 13824)]
    g = torch.Generator(device="cuda").manual_seed(5)
    xd = [(torch.randn(sh, device="cuda", generator=g) * 2).to(TDT[dtype]) for sh in shapes]
    dyd = [torch.randn(sh, device="cuda", generator=g).to(TDT[dtype]) for sh in shapes]
    sd = torch.tensor([0.02 + 0.01 * i for i in range(7)], dtype=torch.float32, device="cuda")
    y_b = [torch.empty_like(x) for x in xd]
    dx_b = [torch.empty_like(x) for x in xd]
    ds_b = torch.zeros(7, dtype=torch.float32, device="cuda")
    ws = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(7))
    items = [(xd[i], dyd[i], sd[i:i + 1], dx_b[i], ds_b[i:i + 1]) for i in range(7)]
    B.sasq_fakequant_fwd_batch([(xd[i], sd[i:i + 1], y_b[i]) for i in range(7)], 8)
    B.sasq_fakequant_bwd_batch(items, ws, 8)
    first = ds_b.clone()
    B.sasq_fakequant_bwd_batch(items, ws, 8)
    assert torch.equal(first, ds_b)
    ws1 = B.new_workspace(B.sasq_fakequant_bwd_workspace(1, 1))
    y1, dx1 = torch.empty_like(xd[6]), torch.empty_like(xd[6])
    ds1 = torch.zeros(1, dtype=torch.float32, device="cuda")
    for i in range(7):
        y1, dx1 = torch.empty_like(xd[i]), torch.empty_like(xd[i])
        B.sasq_fakequant_fwd(xd[i], sd[i:i + 1], y1, None, 8)
        B.sasq_fakequant_bwd(xd[i], dyd[i], sd[i:i + 1], dx1, ds1, ws1, 8)
        assert torch.equal(y1.view(torch.int16), y_b[i].view(torch.int16)), i
        assert torch.equal(dx1.view(torch.int16), dx_b[i].view(torch.int16)), i
        a, b = float(ds1.item()), float(first[i].item())
        assert abs(a - b) <= 1e-4 * abs(a) + 1e-3, (i, a, b)


# ---------------------------------------------------------------- batched static linear
from tests.test_gpu_grouped_linear import WF, device_weights  # noqa: E402
from tests.gpu_util import assert_same_values  # noqa: E402

LIN_BATCHES = [
    [(33, 47, 128)],
    [(300, 520, 384), (300, 260, 1024), (300, 520, 64)],
    [(257, 255, 1024), (40, 300, 64), (512, 768, 512), (64, 256, 256), (1, 1, 128), (260, 70, 192), (130, 700, 512), (256, 256, 128)],
    # more than 256 tiles of 256x256 with a short last round: its tiles are handed out as 128-row halves.  The
    # first M leaves 204 rows in the last row of tiles (a full upper half, a ragged lower one), the second 100
    # rows (the lower halves have nothing to do)
    [(250, 200, 128), (4300, 4090, 64)],
    [(4196, 4096, 64)],
]


@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int4")])
@pytest.mark.parametrize("batch", LIN_BATCHES, ids=["one", "three", "eight", "split-tail", "split-tail-short"])
def test_linear_batch_matches_oracle(batch, dtype, fmt, blocked):
    wf = WF[(fmt, blocked)]
    items, refs = [], []
    for j, (M, N, K) in enumerate(batch):
        xb = wl.random_bits(91, f"lbx{j}{(M, N, K)}{dtype}", (M, K), dtype, gain=2.0)
        w = wl.random_f32(91, f"lbw{j}{(M, N, K)}", (N, K), 0.02)
        wq, s_w = oracle.quantize_weight(w, fmt)
        bias = wl.random_f32(91, f"lbb{j}", (N,), 0.3) if j % 2 else None
        s = np.float32(oracle.absmax_scale(xb, 8, dtype) / 3)
        refs.append(oracle.static_linear(xb, s, wq, s_w, bias, 8, fmt, dtype, want_acc=False, want_xq=False)["y"])
        y = torch.full((M, N), float("nan"), dtype=TDT[dtype], device="cuda")
        items.append((to_dev(xb, dtype), dev_scalar(s), device_weights(wq, fmt, blocked), torch.from_numpy(s_w).cuda(),
                      None if bias is None else torch.from_numpy(bias).cuda(), y))
    ws = B.new_workspace(B.sasq_static_linear_batch_workspace(items, wf))
    B.sasq_static_linear_batch(items, wf, ws)
    torch.cuda.synchronize()
    for j, it in enumerate(items):
        assert_same_values(to_bits(it[5]), refs[j], dtype, f"Y of item {j}")


@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("dtype,fmt", [("f16", "int8"), ("bf16", "int4")])
def test_linear_batch_with_projections_sharing_inputs(dtype, fmt, blocked):
    """q/k/v-like and gate/up-like projections on shared activation tensors (the pre-pass reads a
    shared X once and stages one code buffer per projection), interleaved with one on its own X;
    ragged M; every weight format (row-major int4 stores its codes in the permuted K order)."""
    wf = WF[(fmt, blocked)]
    M = 70
    xa = wl.random_bits(93, f"sha{dtype}", (M, 256), dtype, gain=2.0)
    xb = wl.random_bits(93, f"shb{dtype}", (M, 128), dtype, gain=2.0)
    xc = wl.random_bits(93, f"shc{dtype}", (M, 256), dtype, gain=2.0)
    dev = {"a": to_dev(xa, dtype), "b": to_dev(xb, dtype), "c": to_dev(xc, dtype)}
    bits = {"a": xa, "b": xb, "c": xc}
    plan = [("a", 96), ("b", 40), ("a", 33), ("c", 64), ("b", 300), ("a", 128)]      # (input, N): a x3, b x2, c alone
    items, refs = [], []
    for j, (name, N) in enumerate(plan):
        K = bits[name].shape[1]
        wq, s_w = oracle.quantize_weight(wl.random_f32(93, f"shw{j}", (N, K), 0.02), fmt)
        s = np.float32(oracle.absmax_scale(bits[name], 8, dtype) / (2 + j))          # a different factor per projection
        refs.append(oracle.static_linear(bits[name], s, wq, s_w, None, 8, fmt, dtype, want_acc=False, want_xq=False)["y"])
        y = torch.full((M, N), float("nan"), dtype=TDT[dtype], device="cuda")
        items.append((dev[name], dev_scalar(s), device_weights(wq, fmt, blocked), torch.from_numpy(s_w).cuda(), None, y))
    ws = B.new_workspace(B.sasq_static_linear_batch_workspace(items, wf))
    B.sasq_static_linear_batch(items, wf, ws)
    torch.cuda.synchronize()
    for j, it in enumerate(items):
        assert_same_values(to_bits(it[5]), refs[j], dtype, f"Y of item {j} ({plan[j]})")


def test_linear_batch_rejects():
    x = torch.zeros((4, 96), dtype=torch.float16, device="cuda")
    y = torch.zeros((4, 4), dtype=torch.float16, device="cuda")
    wq = torch.zeros((4, 96), dtype=torch.int8, device="cuda")
    one = torch.ones(4, dtype=torch.float32, device="cuda")
    arr, dt = B._lin_items([(x, one[:1], wq, one, None, y)], B.SASQ_W_INT8)
    ws = B.new_workspace(4096)
    call = lambda count, bits, wf: B._lib().sasq_static_linear_batch(arr, count, bits, wf, dt, B._ptr(ws), ws.numel(), None)
    assert call(1, 8, 0) == 2            # K not a multiple of 64
    assert call(0, 8, 0) == 2
    assert call(1, 9, 0) == 4
    assert call(1, 8, 5) == 4


# ------------------------------------------------------------------ per-channel factors, batched
PC_SHAPES = [(1, 8), (3, 16), (17, 40), (64, 256), (257, 1032), (512, 4096), (5, 8192), (300, 520)]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("count", [1, 3, 8])
def test_pc_batch_matches_single_calls_and_oracle(dtype, count):
    shapes = PC_SHAPES[:count]
    xs = [wl.random_bits(85, f"px{sh}{dtype}", sh, dtype, gain=2.0) for sh in shapes]
    dys = [wl.random_bits(85, f"pd{sh}{dtype}", sh, dtype, gain=1.0) for sh in shapes]
    ss = [(np.abs(wl.random_f32(85, f"ps{sh}", (sh[1],), 0.02)) + np.float32(0.005)).astype(np.float32) for sh in shapes]
    xd = [to_dev(x, dtype) for x in xs]
    dyd = [to_dev(d, dtype) for d in dys]
    sd = [torch.from_numpy(s).cuda() for s in ss]
    yd = [torch.empty_like(x) for x in xd]
    dxd = [torch.empty_like(x) if i != 1 else None for i, x in enumerate(xd)]      # one item without dx
    dsd = [torch.full((sh[1],), float("nan"), dtype=torch.float32, device="cuda") for sh in shapes]
    B.sasq_fakequant_fwd_pc_batch([(xd[i], sd[i], yd[i]) for i in range(count)], 8)
    items = [(xd[i], dyd[i], sd[i], dxd[i], dsd[i]) for i in range(count)]
    ws = B.new_workspace(B.sasq_fakequant_bwd_pc_batch_workspace(items))
    B.sasq_fakequant_bwd_pc_batch(items, ws, 8)
    ds1 = [d.cpu().numpy().copy() for d in dsd]
    B.sasq_fakequant_bwd_pc_batch(items, ws, 8)                                    # same workspace, second call
    torch.cuda.synchronize()
    for i in range(count):
        assert np.array_equal(dsd[i].cpu().numpy(), ds1[i]), "ds is deterministic and the tickets were reset"
        # single-tensor calls: everything bit-identical (an item's reduction does not depend on the batch)
        y1 = torch.empty_like(xd[i])
        dx1 = torch.empty_like(xd[i])
        ds_single = torch.empty_like(dsd[i])
        ws1 = B.new_workspace(B.sasq_fakequant_bwd_pc_workspace(*shapes[i]))
        B.sasq_fakequant_fwd_pc(xd[i], sd[i], y1, None, 8)
        B.sasq_fakequant_bwd_pc(xd[i], dyd[i], sd[i], dx1, ds_single, ws1, 8)
        torch.cuda.synchronize()
        assert torch.equal(y1.view(torch.int16), yd[i].view(torch.int16)), i
        if dxd[i] is not None:
            assert torch.equal(dx1.view(torch.int16), dxd[i].view(torch.int16)), i
        assert np.array_equal(ds_single.cpu().numpy(), ds1[i]), i
        # and the oracle
        y_ref, _ = oracle.fakequant_fwd_pc(xs[i], ss[i], 8, dtype)
        ref = oracle.fakequant_bwd_pc(xs[i], dys[i], ss[i], 8, dtype)
        assert np.array_equal(wl.storage_bits_to_f32(to_bits(yd[i]), dtype), wl.storage_bits_to_f32(y_ref, dtype)), i
        if dxd[i] is not None:
            assert np.array_equal(wl.storage_bits_to_f32(to_bits(dxd[i]), dtype), wl.storage_bits_to_f32(ref["dx"], dtype)), i
        tol = 1e-4 * np.abs(ref["ds64"]) + 1e-6 * ref["sum_abs"] + 1e-30
        assert (np.abs(ds1[i].astype(np.float64) - ref["ds64"]) <= tol).all(), i


def test_pc_batch_errors_and_layer_sizes():
    x = torch.zeros((4, 12), dtype=torch.float16, device="cuda")          # cols % 8 != 0
    s = torch.ones(12, dtype=torch.float32, device="cuda")
    arr, dt = B._fq_items([(x, s, x)], False)
    assert B._lib().sasq_fakequant_fwd_pc_batch(arr, 1, 8, dt, None) == 2
    assert B._lib().sasq_fakequant_fwd_pc_batch(arr, 0, 8, dt, None) == 2
    # the four activation tensors of config 3 / a LLaMA-2-7B layer (x_qkv, x_o, x_mlp, x_down), batched,
    # against the single-tensor calls
    dtype = "f16"
    shapes = [(2048, 4096)] * 3 + [(2048, 11008)]
    g = torch.Generator(device="cuda").manual_seed(6)
    xd = [(torch.randn(sh, device="cuda", generator=g) * 2).to(TDT[dtype]) for sh in shapes]
    dyd = [torch.randn(sh, device="cuda", generator=g).to(TDT[dtype]) for sh in shapes]
    sd = [torch.rand(sh[1], device="cuda", generator=g) * 0.05 + 0.01 for sh in shapes]
    yb = [torch.empty_like(t) for t in xd]
    dxb = [torch.empty_like(t) for t in xd]
    dsb = [torch.empty(sh[1], dtype=torch.float32, device="cuda") for sh in shapes]
    items = [(xd[i], dyd[i], sd[i], dxb[i], dsb[i]) for i in range(4)]
    ws = B.new_workspace(B.sasq_fakequant_bwd_pc_batch_workspace(items))
    B.sasq_fakequant_fwd_pc_batch([(xd[i], sd[i], yb[i]) for i in range(4)], 8)
    B.sasq_fakequant_bwd_pc_batch(items, ws, 8)
    torch.cuda.synchronize()
    for i in range(4):
        y1, dx1, ds1 = torch.empty_like(xd[i]), torch.empty_like(xd[i]), torch.empty_like(dsb[i])
        ws1 = B.new_workspace(B.sasq_fakequant_bwd_pc_workspace(*shapes[i]))
        B.sasq_fakequant_fwd_pc(xd[i], sd[i], y1, None, 8)
        B.sasq_fakequant_bwd_pc(xd[i], dyd[i], sd[i], dx1, ds1, ws1, 8)
        torch.cuda.synchronize()
        assert torch.equal(y1.view(torch.int16), yb[i].view(torch.int16)), i
        assert torch.equal(dx1.view(torch.int16), dxb[i].view(torch.int16)), i
        assert torch.equal(ds1, dsb[i]), i


@pytest.fixture
def force_sharing():
    """The library groups operators on one x only from 12 M elements up; this lifts the threshold."""
    from tests.gpu_util import set_tuning
    set_tuning(share=3)
    yield
    set_tuning()


def test_batch_sharing_at_its_natural_size():
    """Two operators on one 4096 x 4096 input (grouped by the library's own rule) and one on another:
    against the single-tensor calls, bit for bit (ds within the reduction-order tolerance)."""
    dtype = "f16"
    g = torch.Generator(device="cuda").manual_seed(9)
    xa = (torch.randn((4096, 4096), device="cuda", generator=g) * 2).to(TDT[dtype])
    xb = (torch.randn((4096, 4096), device="cuda", generator=g) * 2).to(TDT[dtype])
    xd = [xa, xb, xa]
    dyd = [torch.randn((4096, 4096), device="cuda", generator=g).to(TDT[dtype]) for _ in range(3)]
    sd = torch.tensor([0.05, 0.03, 0.011], dtype=torch.float32, device="cuda")
    yb = [torch.empty_like(xa) for _ in range(3)]
    dxb = [torch.empty_like(xa) for _ in range(3)]
    dsb = torch.zeros(3, dtype=torch.float32, device="cuda")
    ws = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(3))
    B.sasq_fakequant_fwd_batch([(xd[i], sd[i:i + 1], yb[i]) for i in range(3)], 8)
    B.sasq_fakequant_bwd_batch([(xd[i], dyd[i], sd[i:i + 1], dxb[i], dsb[i:i + 1]) for i in range(3)], ws, 8)
    torch.cuda.synchronize()
    ws1 = B.new_workspace(B.sasq_fakequant_bwd_workspace(4096, 4096))
    for i in range(3):
        y1, dx1 = torch.empty_like(xa), torch.empty_like(xa)
        ds1 = torch.zeros(1, dtype=torch.float32, device="cuda")
        B.sasq_fakequant_fwd(xd[i], sd[i:i + 1], y1, None, 8)
        B.sasq_fakequant_bwd(xd[i], dyd[i], sd[i:i + 1], dx1, ds1, ws1, 8)
        torch.cuda.synchronize()
        assert torch.equal(y1.view(torch.int16), yb[i].view(torch.int16)), i
        assert torch.equal(dx1.view(torch.int16), dxb[i].view(torch.int16)), i
        assert rel_err(float(dsb[i].item()), float(ds1.item())) <= 1e-5, i


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(3, 5), (64, 256), (257, 1031), (700, 4099)])
def test_batch_operators_sharing_one_input(dtype, shape, force_sharing):
    """Five operators, three of them (not adjacent in the batch) on the same x with different factors,
    two on another x: the library reads a shared x once.  Everything must equal the single-tensor
    calls bit for bit (ds within the reduction-order tolerance) and the oracle."""
    xa = wl.random_bits(87, f"sxa{shape}{dtype}", shape, dtype, gain=2.0)
    xb = wl.random_bits(87, f"sxb{shape}{dtype}", shape, dtype, gain=3.0)
    xs = [xa, xb, xa, xb, xa]
    dys = [wl.random_bits(87, f"sd{i}{shape}{dtype}", shape, dtype, gain=1.0 + i) for i in range(5)]
    s0 = float(oracle.absmax_scale(xa, 8, dtype))
    ss = [np.float32(s0 / d) for d in (1.0, 2.0, 3.5, 5.0, 9.0)]
    xad, xbd = to_dev(xa, dtype), to_dev(xb, dtype)
    xd = [xad, xbd, xad, xbd, xad]                                   # the same device tensors: same pointers
    dyd = [to_dev(d, dtype) for d in dys]
    sd = torch.tensor([float(s) for s in ss], dtype=torch.float32, device="cuda")
    yd = [torch.empty_like(xad) for _ in range(5)]
    dxd = [torch.empty_like(xad) if i != 2 else None for i in range(5)]  # one member of the group without dx
    dsd = torch.full((5,), float("nan"), dtype=torch.float32, device="cuda")
    ws = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(5))
    B.sasq_fakequant_fwd_batch([(xd[i], sd[i:i + 1], yd[i]) for i in range(5)], 8)
    items = [(xd[i], dyd[i], sd[i:i + 1], dxd[i], dsd[i:i + 1]) for i in range(5)]
    B.sasq_fakequant_bwd_batch(items, ws, 8)
    ds1 = dsd.cpu().numpy().copy()
    B.sasq_fakequant_bwd_batch(items, ws, 8)                          # same workspace again: tickets were reset
    torch.cuda.synchronize()
    assert np.array_equal(dsd.cpu().numpy(), ds1)
    for i in range(5):
        y_ref, _ = oracle.fakequant_fwd(xs[i], ss[i], 8, dtype)
        ref = oracle.fakequant_bwd(xs[i], dys[i], ss[i], 8, dtype)
        assert np.array_equal(wl.storage_bits_to_f32(to_bits(yd[i]), dtype), wl.storage_bits_to_f32(y_ref, dtype)), i
        if dxd[i] is not None:
            assert np.array_equal(wl.storage_bits_to_f32(to_bits(dxd[i]), dtype), wl.storage_bits_to_f32(ref["dx"], dtype)), i
        tol = 1e-4 * abs(ref["ds64"]) + 1e-7 * ref["sum_abs"] + 1e-30
        assert abs(float(ds1[i]) - ref["ds64"]) <= tol, (i, ds1[i], ref["ds64"])


def test_instrumented_build_computes_the_same_and_stamps_in_order():
    """The benchmark's instrumented build of the library (per-tile timestamps in the batched GEMM, bench.py
    --tile-timestamps) against the product library on one batch: same Y bit for bit; every workgroup that ran a tile
    left five non-decreasing cycle stamps and its K."""
    import ctypes
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(B.__file__)), "libsasq_ts.so")
    assert os.path.exists(path), "libsasq_ts.so missing: python -m paper_2512_14481_amd.build"
    ts = ctypes.CDLL(path)
    ts.sasq_ts_set_buffer.argtypes = [ctypes.c_void_p]
    wf = WF[("int8", True)]
    batch = [(300, 520, 384), (257, 255, 1024)]
    items = []
    for j, (M, N, K) in enumerate(batch):
        xb = wl.random_bits(97, f"tsx{j}", (M, K), "f16", gain=2.0)
        wq, s_w = oracle.quantize_weight(wl.random_f32(97, f"tsw{j}", (N, K), 0.02), "int8")
        s = np.float32(oracle.absmax_scale(xb, 8, "f16") / 3)
        items.append((to_dev(xb, "f16"), dev_scalar(s), device_weights(wq, "int8", True), torch.from_numpy(s_w).cuda(), None,
                      torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")))
    ws = B.new_workspace(B.sasq_static_linear_batch_workspace(items, wf))
    B.sasq_static_linear_batch(items, wf, ws)
    torch.cuda.synchronize()
    want = [it[5].clone() for it in items]
    for it in items:
        it[5].fill_(float("nan"))
    arr, dt = B._lin_items(items, wf)
    stamps = torch.zeros(64 * 16, dtype=torch.int64, device="cuda")
    assert ts.sasq_ts_set_buffer(stamps.data_ptr()) == 0
    rc = ts.sasq_static_linear_batch(arr, len(items), 8, wf, dt, ctypes.c_void_p(ws.data_ptr()),
                                     ctypes.c_size_t(ws.numel() * ws.element_size()), None)
    assert rc == 0
    torch.cuda.synchronize()
    assert ts.sasq_ts_set_buffer(None) == 0
    for j, it in enumerate(items):
        assert torch.equal(it[5].view(torch.int16), want[j].view(torch.int16)), j
    t = stamps.cpu().numpy().reshape(64, 16)
    ran = t[t[:, 0] != 0]
    assert len(ran) == 6 + 2                               # 2 x 3 tiles of the first item, 2 x 1 of the second
    assert (np.diff(ran[:, [0, 2, 4, 6, 8]], axis=1) >= 0).all()
    assert sorted(set(ran[:, 14].tolist())) == [384, 1024]

