"""One scale-training step of a quantized linear layer, every stage on the GPU, each stage checked
against the CPU oracle on the same inputs (Sec. 4.2: only the quantization factor is trained):

    x' = fakequant(x; s)                  sasq_fakequant_fwd           (Eq. 5)
    Y  = static_linear(x; s, Wq, s_w)     sasq_static_linear           (Eq. 2; equals x' . Wq^T)
    dx'= dY . Wq                          sasq_linear_bwd_input        (frozen weight, upstream dY synthetic)
    dx, ds = fakequant_bwd(x, dx'; s)     sasq_fakequant_bwd           (Eq. 4 and the STE)
    s <- AdamW(s, ds)                     sasq_scale_adamw
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_2512_14481_amd import binding as B
from paper_2512_14481_amd import workloads as wl
from tests.gpu_util import TDT, assert_same_values, rel_err, to_bits, to_dev, val

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,fmt,shape", [("f16", "int8", (64, 256, 256)), ("bf16", "int4", (200, 96, 320)),
                                             ("bf16", "int8", (1000, 1024, 512))])
def test_scale_training_step_stage_by_stage(dtype, fmt, shape):
    M, N, K = shape
    xb = wl.random_bits(91, f"lx{shape}", (M, K), dtype, gain=2.0)
    dyb = wl.random_bits(91, f"ldy{shape}", (M, N), dtype, gain=0.01)
    wq, s_w = oracle.quantize_weight(wl.random_f32(91, f"lw{shape}", (N, K), 0.02), fmt)
    s = np.float32(oracle.absmax_scale(xb, 8, dtype) * 0.6)           # some clipping: ds has both kinds of terms
    wf = B.SASQ_W_INT8 if fmt == "int8" else B.SASQ_W_INT4_PACKED

    x, dy_out = to_dev(xb, dtype), to_dev(dyb, dtype)
    s_d = torch.tensor([float(s)], dtype=torch.float32, device="cuda")
    wq_d, sw_d = torch.from_numpy(wq).cuda(), torch.from_numpy(s_w).cuda()
    wt = torch.empty(B.sasq_bwd_weight_bytes(N, K), dtype=torch.uint8, device="cuda")
    B.sasq_prepare_bwd_weight(wq_d, sw_d, wt, N, K, wf, TDT[dtype])
    ws_lin = B.new_workspace(B.sasq_static_linear_workspace(M, N, K, wf))
    ws_bwd = B.new_workspace(B.sasq_fakequant_bwd_workspace(M, K))

    xhat = torch.empty_like(x)
    y = torch.empty((M, N), dtype=TDT[dtype], device="cuda")
    dxp = torch.empty_like(x)
    dx = torch.empty_like(x)
    ds = torch.zeros(1, dtype=torch.float32, device="cuda")
    m1 = torch.zeros(1, dtype=torch.float32, device="cuda")
    v1 = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.sasq_fakequant_fwd(x, s_d, xhat, None, 8)
    B.sasq_static_linear(x, s_d, wq_d, sw_d, None, y, wf, ws_lin)
    B.sasq_linear_bwd_input(dy_out, wt, dxp, K)
    B.sasq_fakequant_bwd(x, dxp, s_d, dx, ds, ws_bwd, 8)
    s_new = s_d.clone()
    B.sasq_scale_adamw(s_new, ds, m1, v1, 1, 1e-3)
    torch.cuda.synchronize()

    # forward stages: bit for bit
    xhat_ref, _ = oracle.fakequant_fwd(xb, s, 8, dtype)
    assert_same_values(to_bits(xhat), xhat_ref, dtype, "x'")
    lin = oracle.static_linear(xb, s, wq, s_w, None, 8, fmt, dtype)
    assert_same_values(to_bits(y), lin["y"], dtype, "Y")
    # backward through the frozen weight: within the fp32 accumulation bound of the exact sums
    ref = oracle.linear_bwd_input(dyb, wq, s_w, fmt, dtype)
    g = val(to_bits(dxp), dtype)
    ulp = np.maximum(np.abs(val((to_bits(dxp) + 1).astype(np.uint16), dtype) - g),
                     np.abs(val((to_bits(dxp) - 1).astype(np.uint16), dtype) - g))
    assert (np.abs(g - ref["exact"]) <= 0.5 * ulp * (1 + 2.0 ** -9) + N * 2.0 ** -24 * ref["sum_abs"] + 1e-45).all()
    # fake-quant backward on the GPU's own dx': dx bit for bit, ds within 1e-4
    fq = oracle.fakequant_bwd(xb, to_bits(dxp), s, 8, dtype)
    assert_same_values(to_bits(dx), fq["dx"], dtype, "dx")
    assert rel_err(float(ds.item()), fq["ds64"]) <= 1e-4
    # ... and end to end against the oracle-only chain (dx' differs in a few last bits)
    fq_chain = oracle.fakequant_bwd(xb, ref["dx"], s, 8, dtype)
    assert abs(float(ds.item()) - fq_chain["ds64"]) <= 1e-3 * fq_chain["sum_abs"]
    # optimizer step on the scale
    upd = oracle.scale_adamw(np.array([s], np.float32), np.array([ds.item()], np.float32),
                             np.zeros(1, np.float32), np.zeros(1, np.float32), 1, 1e-3)
    assert np.allclose(s_new.cpu().numpy(), upd[0], rtol=2e-6, atol=0)     # fp32 kernel, fp64-evaluated oracle
    assert float(s_new.item()) != float(s)


def test_batched_step_replays_from_a_hip_graph():
    """The library allocates nothing, copies nothing and clears nothing on its own, so the whole batched pass
    (fake-quant forward and backward of every input, SGD on the scales, static linears) can be captured into a
    HIP graph.  Three replays, with eager library calls and synchronisations between them, must leave exactly
    what three eager passes leave: outputs, ds and the trained scales, bit for bit (the scales change with
    every pass, so a replay that reused stale state would show)."""
    dtype, tdt = "f16", TDT["f16"]
    shapes = [(300, 384, 256), (300, 256, 256), (200, 520, 192)]       # (M, N, K); the first two share their input
    xb = [wl.random_bits(95, "gx0", (300, 256), dtype, gain=2.0), None, wl.random_bits(95, "gx2", (200, 192), dtype, gain=2.0)]
    xb[1] = xb[0]
    x_d = [to_dev(xb[0], dtype), None, to_dev(xb[2], dtype)]
    x_d[1] = x_d[0]
    dy_d = [to_dev(wl.random_bits(95, f"gdy{i}", (sh[0], sh[2]), dtype, gain=0.01), dtype) for i, sh in enumerate(shapes)]
    s0 = [np.float32(oracle.absmax_scale(xb[i], 8, dtype) * (0.5 + 0.1 * i)) for i in range(3)]
    wq_d, sw_d = [], []
    for i, (M, N, K) in enumerate(shapes):
        wq, s_w = oracle.quantize_weight(wl.random_f32(95, f"gw{i}", (N, K), 0.02), "int8")
        wq_d.append(torch.from_numpy(wq).cuda()); sw_d.append(torch.from_numpy(s_w).cuda())
    s_all = torch.zeros(3, dtype=torch.float32, device="cuda")
    ds_all = torch.zeros(3, dtype=torch.float32, device="cuda")
    xhat = [torch.empty_like(x) for x in x_d]
    dx = [torch.empty_like(x) for x in x_d]
    y = [torch.empty((M, N), dtype=tdt, device="cuda") for (M, N, K) in shapes]
    fwd_items = [(x_d[i], s_all[i:i + 1], xhat[i]) for i in range(3)]
    bwd_items = [(x_d[i], dy_d[i], s_all[i:i + 1], dx[i], ds_all[i:i + 1]) for i in range(3)]
    lin_items = [(x_d[i], s_all[i:i + 1], wq_d[i], sw_d[i], None, y[i]) for i in range(3)]
    ws_bwd = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(3))
    ws_lin = B.new_workspace(B.sasq_static_linear_batch_workspace(lin_items, B.SASQ_W_INT8))

    def one_pass():
        B.sasq_fakequant_fwd_batch(fwd_items, 8)
        B.sasq_fakequant_bwd_batch(bwd_items, ws_bwd, 8)
        B.sasq_scale_sgd_vec(s_all, ds_all, 2e-4)
        B.sasq_static_linear_batch(lin_items, B.SASQ_W_INT8, ws_lin)

    def reset():
        s_all.copy_(torch.tensor([float(v) for v in s0]))
        for t in xhat + dx + y:
            t.fill_(float("nan"))
        ds_all.fill_(float("nan"))
        torch.cuda.synchronize()

    def snapshot():
        torch.cuda.synchronize()
        return [to_bits(t).copy() for t in xhat + dx + y] + [s_all.cpu().numpy().copy(), ds_all.cpu().numpy().copy()]

    reset()
    eager = []
    for _ in range(3):
        one_pass()
        eager.append(snapshot())
    assert not np.array_equal(eager[0][-2], eager[1][-2]), "the scales move from pass to pass"

    reset()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        one_pass()                                  # warm-up on the capture stream (PyTorch's capture protocol)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            one_pass()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    scratch = torch.empty_like(x_d[2])
    ws1 = B.new_workspace(B.sasq_fakequant_bwd_workspace(200, 192))
    ds1 = torch.zeros(1, dtype=torch.float32, device="cuda")
    reset()
    for k in range(3):
        graph.replay()
        got = snapshot()
        for a, b in zip(got, eager[k]):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), f"replay {k + 1} differs from eager pass {k + 1}"
        # the program's own eager work between replays
        B.sasq_fakequant_fwd(x_d[2], s_all[2:3], scratch, None, 8)
        B.sasq_fakequant_bwd(x_d[2], dy_d[2], s_all[2:3], scratch, ds1, ws1, 8)
        torch.cuda.synchronize()
