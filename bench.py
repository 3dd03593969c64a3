#!/usr/bin/env python3
"""Benchmark of the SASQ hot path on one MI355X.

A "step" is one pass of the whole hot path over the LLaMA-2-7B MLP workload (M = 4096 tokens;
gate, up: K 4096 -> N 11008; down: K 11008 -> N 4096; fp16 activations, int8 weights): for every
projection, fake-quant forward, straight-through backward with the grid-wide ds reduction, one SGD
update of the scale, and the static-inference W8A8 linear.  Inputs are seeded synthetic tensors
already resident in HBM; weights are quantized once, outside the timed region, by the library.

Prints ONE JSON line.  `value` is the linear-layer integer throughput of the whole step
(2*M*N*K summed over the projections, divided by the full step time, fake-quant kernels included).
`roofline` is the static linear alone, timed with HIP events on the launch stream inside the timed
region; `fakequant` is the fake-quant forward+backward pair against HBM bandwidth; `cpu_baseline`
is the CPU oracle on a bounded row sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2512_14481_amd import binding as B          # noqa: E402
from paper_2512_14481_amd import workloads as wl       # noqa: E402

INT8_MFMA_PEAK_TOPS = 5000.0      # MI355X dense int8, published
F16_MFMA_PEAK_TFLOPS = 2500.0    # MI355X dense fp16 / bf16, published
# what a register-only v_mfma_i32_32x32x32_i8 loop sustains on this part with GEMM-like operand codes (the part is
# power-limited under MFMA load; profiles/mfma_peak_and_clock.txt) -- context for `frac`, not the roofline's peak
INT8_MFMA_SUSTAINED_TOPS = 3700.0    # 3613-3750 across boxes (python bench.py --mfma-peak)
# HBM-side bytes per sasq_static_linear call (both kernels), averaged over gate/up/down of config 3:
# rocprofv3 FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 (factors from a plain 1 GiB copy), see
# profiles/bench_c3_mlp7b_counters.txt.  Algorithmic bytes are 221.2 MB.
C3_LINEAR_TRAFFIC_BYTES = 450654 * 1024          # one call per projection, average
C3_LINEAR_BATCH_TRAFFIC_BYTES = 1364068 * 1024   # the batched call (all three projections)
HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E, published
LR = 2e-4
TDT = {"f16": torch.float16, "bf16": torch.bfloat16}


def dev16(bits: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dtype])


class Projection:
    def __init__(self, cfg, proj, x, ws_small):
        self.name, self.x = proj.name, x
        self.M, self.K, self.N = x.shape[0], x.shape[1], proj.N
        wf = B.SASQ_W_INT8 if cfg.w_fmt == wl.W_INT8 else B.SASQ_W_INT4_PACKED
        self.wf = wf
        w = torch.from_numpy(wl.weight_fp32(cfg, proj.name)).cuda()
        kq = self.K if wf == B.SASQ_W_INT8 else self.K // 2
        self.wq = torch.empty((self.N, kq), dtype=torch.int8 if wf == B.SASQ_W_INT8 else torch.uint8, device="cuda")
        self.s_w = torch.empty(self.N, dtype=torch.float32, device="cuda")
        B.sasq_quantize_weight(w, self.wq, self.s_w, wf)
        del w
        # the dequantized weight for the backward GEMM, prepared once from the row-major codes
        self.wt_bwd = None
        if self.N % 32 == 0:
            self.wt_bwd = torch.empty(B.sasq_bwd_weight_bytes(self.N, self.K), dtype=torch.uint8, device="cuda")
            B.sasq_prepare_bwd_weight(self.wq, self.s_w, self.wt_bwd, self.N, self.K, wf, x.dtype)
        # frozen weights are re-arranged once at set-up into the GEMM's blocked format (SASQ_BENCH_ROWMAJOR=1
        # keeps the row-major interchange format instead)
        if self.K % 64 == 0 and not os.environ.get("SASQ_BENCH_ROWMAJOR"):
            wfb = B.SASQ_W_INT8_BLOCKED if wf == B.SASQ_W_INT8 else B.SASQ_W_INT4_BLOCKED
            packed = torch.empty(B.sasq_packed_weight_bytes(self.N, self.K, wfb), dtype=torch.uint8, device="cuda")
            B.sasq_pack_weight(self.wq, packed, self.N, self.K, wf)
            self.wq, self.wf = packed, wfb
        self.dy = dev16(wl.upstream_grad(cfg, proj.name), cfg.dtype)
        self.s = torch.empty(1, dtype=torch.float32, device="cuda")
        B.sasq_absmax_scale(x, self.s, ws_small, 8)           # s0 = absmax / 127
        self.s0 = self.s.clone()
        self.ds = torch.zeros(1, dtype=torch.float32, device="cuda")
        self.xhat = torch.empty_like(x)
        self.dx = torch.empty_like(x)
        self.y = torch.empty((self.M, self.N), dtype=x.dtype, device="cuda")
        self.ws_lin = B.new_workspace(B.sasq_static_linear_workspace(self.M, self.N, self.K, wf))
        self.ops = 2.0 * self.M * self.N * self.K
        self.fq_bytes = 10.0 * self.M * self.K


class Layer:
    """The projections of the workload with their scales in one vector, and the descriptors of
    the batched fake-quant calls (one launch for all fake-quant operators of the layer)."""

    def __init__(self, projs):
        self.projs = projs
        n = len(projs)
        self.s_all = torch.cat([p.s for p in projs]).contiguous()
        self.ds_all = torch.zeros(n, dtype=torch.float32, device="cuda")
        for i, p in enumerate(projs):
            p.s, p.ds = self.s_all[i:i + 1], self.ds_all[i:i + 1]
        self.s0_all = self.s_all.clone()
        self.fwd_items = [(p.x, p.s, p.xhat) for p in projs]
        self.bwd_items = [(p.x, p.dy, p.s, p.dx, p.ds) for p in projs]
        self.ws_batch = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(n))
        self.fq_bytes = sum(p.fq_bytes for p in projs)
        # the linears of the layer in one batched call (needs one weight format and K % 64 == 0 throughout)
        self.wf = projs[0].wf
        self.lin_items = [(p.x, p.s, p.wq, p.s_w, None, p.y) for p in projs]
        self.lin_batched = all(p.wf == self.wf and p.K % 64 == 0 for p in projs)
        if self.lin_batched:
            self.ws_lin = B.new_workspace(B.sasq_static_linear_batch_workspace(self.lin_items, self.wf))
        self.ops = sum(p.ops for p in projs)


def step(layer, ev=None):
    """One pass of the hot path: fake-quant forward and backward (+ds) of every projection input
    (one batched launch each), SGD on the scales, then the static linear of every projection.
    ev: optional dict of event lists for per-call timing."""
    if ev is not None:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
    B.sasq_fakequant_fwd_batch(layer.fwd_items, 8)
    B.sasq_fakequant_bwd_batch(layer.bwd_items, layer.ws_batch, 8)
    if ev is not None:
        e1.record()
        ev["fq"].append((e0, e1))
    B.sasq_scale_sgd_vec(layer.s_all, layer.ds_all, LR)
    if layer.lin_batched:
        if ev is not None:
            e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e2.record()
        B.sasq_static_linear_batch(layer.lin_items, layer.wf, layer.ws_lin)
        if ev is not None:
            e3.record()
            ev["lin_batch"].append((e2, e3))
        return
    for p in layer.projs:
        if ev is not None:
            e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e2.record()
        B.sasq_static_linear(p.x, p.s, p.wq, p.s_w, None, p.y, p.wf, p.ws_lin)
        if ev is not None:
            e3.record()
            ev["lin"].append((e2, e3, p))


def step_unbatched(projs, ws_bwd, ev=None):
    """The same pass with one launch per tensor and call (--unbatched)."""
    for p in projs:
        if ev is not None:
            e0, e1, e2, e3 = (torch.cuda.Event(enable_timing=True) for _ in range(4))
            e0.record()
        B.sasq_fakequant_fwd(p.x, p.s, p.xhat, None, 8)
        B.sasq_fakequant_bwd(p.x, p.dy, p.s, p.dx, p.ds, ws_bwd, 8)
        if ev is not None:
            e1.record()
        B.sasq_scale_sgd(p.s, p.ds, LR)
        if ev is not None:
            e2.record()
        B.sasq_static_linear(p.x, p.s, p.wq, p.s_w, None, p.y, p.wf, p.ws_lin)
        if ev is not None:
            e3.record()
            ev["fq_each"].append((e0, e1, p))
            ev["lin"].append((e2, e3, p))


def cpu_baseline(cfg, rows: int):
    """The CPU oracle, as it stands, on the first `rows` tokens of every projection's input."""
    import oracle
    t_total, ops = 0.0, 0.0
    for proj in cfg.projs:
        x = wl.activation(cfg, proj.x, rows=rows)
        dy = wl.upstream_grad(cfg, proj.name, rows=rows)
        w = wl.weight_fp32(cfg, proj.name)
        wq, s_w = oracle.quantize_weight(w, cfg.w_fmt)       # set-up, not timed (as on the GPU)
        s = oracle.absmax_scale(x, 8, cfg.dtype)
        t0 = time.perf_counter()
        oracle.fakequant_fwd(x, s, 8, cfg.dtype)
        b = oracle.fakequant_bwd(x, dy, s, 8, cfg.dtype)
        s1 = oracle.scale_sgd(s, b["ds"], LR)
        oracle.static_linear(x, s1, wq, s_w, None, 8, cfg.w_fmt, cfg.dtype, want_acc=False, want_xq=False)
        t_total += time.perf_counter() - t0
        ops += 2.0 * rows * proj.N * cfg.K_of(proj)
    return {"value": ops / t_total / 1e12, "unit": "TOPS", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"first {rows} of {cfg.M} tokens of every projection, whole step "
                      f"(fake-quant fwd+bwd, SGD, static linear); {t_total:.1f} s"}


def mfma_peak():
    """What the part's matrix units sustain on their own (register-only loop, GEMM register pattern),
    per operand pattern: TOP/s of each of 80 back-to-back launches (about 0.5 s of load per pattern)."""
    sink = torch.empty(65536, dtype=torch.int32, device="cuda")
    iters, launches = 20000, 80
    out = {"metric": "register-only MFMA loop, sustained", "unit": "TOP/s (TFLOP/s for f16)", "iters_per_launch": iters,
           "launches": launches, "patterns": {}}
    for kind, name, ops in ((0, "i8 zeros", 65536.0), (1, "i8 random bits", 65536.0), (2, "i8 GEMM-like codes", 65536.0),
                            (3, "f16 small random values", 32768.0)):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
        torch.cuda.synchronize()
        ev[0].record()
        for l in range(launches):
            B.sasq_mfma_probe(kind, iters, sink)
            ev[l + 1].record()
        torch.cuda.synchronize()
        tops = [1024.0 * iters * 16 * ops / (ev[l].elapsed_time(ev[l + 1]) * 1e-3) / 1e12 for l in range(launches)]
        settled = sorted(tops[launches // 2:])
        out["patterns"][name] = {"first_launches": [round(v) for v in tops[:4]], "settled_median": round(settled[len(settled) // 2]),
                                 "settled_min": round(settled[0]), "settled_max": round(settled[-1])}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--settle-steps", type=int, default=100,
                    help="untimed steps before the timed region in all, warm-up included (0: only the warm-up steps)")
    ap.add_argument("--config", default="c3_mlp7b")
    ap.add_argument("--cpu-rows", type=int, default=4096)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--unbatched", action="store_true",
                    help="one launch per tensor for the fake-quant operators instead of one per layer")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="instead of the workload: time the library's register-only MFMA loop under sustained load "
                         "(80 back-to-back launches per operand pattern) and print what the matrix units sustain")
    ap.add_argument("--calib", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build is single-GPU; --gpus must be 1 (the path shards by token rows with "
                 "one tiny all-gather for ds, but nothing multi-GPU is implemented)")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if a.mfma_peak:
        torch.cuda.set_device(0)
        mfma_peak()
        return

    cfg = wl.CONFIGS[a.config]
    ws_small = B.new_workspace(max(B.sasq_absmax_scale_workspace(1, 1), B.sasq_fakequant_bwd_workspace(1, 1)))
    acts = {act.name: dev16(wl.activation(cfg, act.name), cfg.dtype) for act in cfg.acts}
    projs = [Projection(cfg, p, acts[p.x], ws_small) for p in cfg.projs]
    layer = Layer(projs)
    run_step = (lambda ev=None: step_unbatched(projs, ws_small, ev)) if a.unbatched else (lambda ev=None: step(layer, ev))
    torch.cuda.synchronize()

    if a.calib:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                                 # 1 GiB read + 1 GiB written by a plain copy kernel
        torch.cuda.synchronize()
        del src, dst
    # The GEMM's time settles only after about 80 steps of continuous load (power management); a caller
    # that asks for a short warm-up still gets the settled state: the same step is run, untimed, until
    # `settle_steps` steps have gone by in all, then the W warm-up steps proper.
    settle = max(0, a.settle_steps - a.warmup)
    for _ in range(settle):
        run_step()
    for _ in range(a.warmup):
        run_step()
    layer.s_all.copy_(layer.s0_all)                   # every timed run starts from the same scales
    torch.cuda.synchronize()
    ev = {"fq": [], "fq_each": [], "lin": [], "lin_batch": []}
    t0 = time.perf_counter()
    for _ in range(a.steps):
        run_step(ev)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if not a.unbatched:
        # per-projection fake-quant figures: the unbatched pass once more, outside the timed region
        layer.s_all.copy_(layer.s0_all)
        for _ in range(3):
            step_unbatched(projs, ws_small, ev)
        torch.cuda.synchronize()
        if not layer.lin_batched:
            ev["lin"] = ev["lin"][:a.steps * len(projs)]

    ms_per_step = dt / a.steps * 1e3
    total_ops = sum(p.ops for p in projs)
    lin_ms = [(e0.elapsed_time(e1), p) for e0, e1, p in ev["lin"]]
    fq_ms = [(e0.elapsed_time(e1), p) for e0, e1, p in ev["fq_each"]]
    if ev["lin_batch"]:
        # the roofline figure is the batched call: the layer's activation pre-pass + one GEMM launch
        lin_ops_per_call = total_ops
        lin_avg_ms = sum(e0.elapsed_time(e1) for e0, e1 in ev["lin_batch"]) / len(ev["lin_batch"])
    else:
        lin_ops_per_call = total_ops / len(projs)     # average over the projections' calls
        lin_avg_ms = sum(t for t, _ in lin_ms) / len(lin_ms)
    lin_tops = lin_ops_per_call / (lin_avg_ms * 1e-3) / 1e12
    # spread over the timed steps (median and fastest call)
    lin_all = sorted(e0.elapsed_time(e1) for e0, e1 in ev["lin_batch"]) if ev["lin_batch"] else sorted(t for t, _ in lin_ms)
    fq_all = sorted(e0.elapsed_time(e1) for e0, e1 in ev["fq"]) if ev["fq"] else []
    med = lambda v: v[len(v) // 2] if v else None
    if a.unbatched:
        fq_gbps = sum(p.fq_bytes for _, p in fq_ms) / (sum(t for t, _ in fq_ms) * 1e-3) / 1e9
    else:
        fq_gbps = layer.fq_bytes * len(ev["fq"]) / (sum(e0.elapsed_time(e1) for e0, e1 in ev["fq"]) * 1e-3) / 1e9
    per_proj = {}
    for name in [p.name for p in projs]:
        tl = [t for t, p in lin_ms if p.name == name]
        tf = [t for t, p in fq_ms if p.name == name]
        pp = next(p for p in projs if p.name == name)
        per_proj[name] = {"linear_us": round(1e3 * sum(tl) / len(tl), 2),
                          "linear_tops": round(pp.ops / (sum(tl) / len(tl) * 1e-3) / 1e12, 1),
                          "fakequant_fwd_bwd_us": round(1e3 * sum(tf) / len(tf), 2),
                          "fakequant_gbps": round(pp.fq_bytes / (sum(tf) / len(tf) * 1e-3) / 1e9, 1)}

    # per-channel fake-quant (the granularity of the paper's main runs), measured after the timed
    # region on the same tensors: one scale per column, ds a column reduction
    pc = None
    if cfg.name == "c3_mlp7b":
        tot_b, tot_ms = 0.0, 0.0
        for p in (projs[0], projs[2]):
            sv = p.s.expand(p.K).contiguous()
            dsv = torch.zeros(p.K, dtype=torch.float32, device="cuda")
            wsp = B.new_workspace(B.sasq_fakequant_bwd_pc_workspace(p.M, p.K))
            for _ in range(2):
                B.sasq_fakequant_fwd_pc(p.x, sv, p.xhat, None, 8)
                B.sasq_fakequant_bwd_pc(p.x, p.dy, sv, p.dx, dsv, wsp, 8)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                B.sasq_fakequant_fwd_pc(p.x, sv, p.xhat, None, 8)
                B.sasq_fakequant_bwd_pc(p.x, p.dy, sv, p.dx, dsv, wsp, 8)
            e1.record()
            torch.cuda.synchronize()
            tot_ms += e0.elapsed_time(e1) / 5
            tot_b += p.fq_bytes
        pc = {"achieved": round(tot_b / (tot_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
              "frac": round(tot_b / (tot_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
              "note": "per-channel fwd+bwd on x_mlp and x_down, one launch per tensor, warm repeat of 5"}
        # the same for all three projection inputs of the layer in one launch each way
        svs = [p.s.expand(p.K).contiguous() for p in projs]
        dsvs = [torch.zeros(p.K, dtype=torch.float32, device="cuda") for p in projs]
        fwd_items = [(p.x, svs[i], p.xhat) for i, p in enumerate(projs)]
        bwd_items = [(p.x, p.dy, svs[i], p.dx, dsvs[i]) for i, p in enumerate(projs)]
        wsb = B.new_workspace(B.sasq_fakequant_bwd_pc_batch_workspace(bwd_items))
        for _ in range(2):
            B.sasq_fakequant_fwd_pc_batch(fwd_items, 8)
            B.sasq_fakequant_bwd_pc_batch(bwd_items, wsb, 8)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            B.sasq_fakequant_fwd_pc_batch(fwd_items, 8)
            B.sasq_fakequant_bwd_pc_batch(bwd_items, wsb, 8)
        e1.record()
        torch.cuda.synchronize()
        bms = e0.elapsed_time(e1) / 5
        bb = sum(p.fq_bytes for p in projs)
        pc["batched"] = {"achieved": round(bb / (bms * 1e-3) / 1e9, 1), "unit": "GB/s",
                         "frac": round(bb / (bms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                         "note": "sasq_fakequant_fwd_pc_batch + sasq_fakequant_bwd_pc_batch over the three projection inputs"}

    # static linear with one activation factor per group of 128 / 512 input channels (the grouped form
    # the paper gives for per-channel activation factors), measured after the timed region
    grouped = None
    if cfg.name == "c3_mlp7b":
        grouped = {}
        for group in (128, 512):
            tot_ops, tot_ms, calls = 0.0, 0.0, 0
            for p in projs:
                if p.K % group:
                    continue
                calls += 1
                sg = p.s.expand(p.K // group).contiguous()
                for _ in range(2):
                    B.sasq_static_linear_grouped(p.x, sg, p.wq, p.s_w, None, p.y, group, p.wf, p.ws_lin)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(5):
                    B.sasq_static_linear_grouped(p.x, sg, p.wq, p.s_w, None, p.y, group, p.wf, p.ws_lin)
                e1.record()
                torch.cuda.synchronize()
                tot_ms += e0.elapsed_time(e1) / 5
                tot_ops += p.ops
            grouped[f"group_{group}"] = {"achieved": round(tot_ops / (tot_ms * 1e-3) / 1e12, 1), "unit": "TOP/s",
                                         "frac": round(tot_ops / (tot_ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, 4),
                                         "us_per_call": round(1e3 * tot_ms / calls, 1), "calls": calls}
        grouped["note"] = ("sasq_static_linear_grouped on the projections whose K the group divides "
                           "(gate, up, down for 128; gate, up for 512); warm repeat of 5")

    # dynamic per-token linear (per-row absmax + quantize + the same GEMM + per-row dequantize): the
    # baseline whose online reduction the static scale removes, on the same tensors
    dynamic = None
    if cfg.name == "c3_mlp7b":
        dynamic = {}
        tot_ops, tot_ms = 0.0, 0.0
        for p in projs:
            wsd = B.new_workspace(B.sasq_dynamic_linear_workspace(p.M, p.N, p.K, p.wf))
            for _ in range(2):
                B.sasq_dynamic_linear(p.x, p.wq, p.s_w, None, p.y, p.wf, wsd)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                B.sasq_dynamic_linear(p.x, p.wq, p.s_w, None, p.y, p.wf, wsd)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            e0.record()
            for _ in range(5):
                B.sasq_static_linear(p.x, p.s, p.wq, p.s_w, None, p.y, p.wf, p.ws_lin)
            e1.record()
            torch.cuda.synchronize()
            ms_static = e0.elapsed_time(e1) / 5
            dynamic[p.name] = {"dynamic_us": round(1e3 * ms, 1), "static_us": round(1e3 * ms_static, 1)}
            tot_ms += ms
            tot_ops += p.ops
        dynamic["achieved"] = round(tot_ops / (tot_ms * 1e-3) / 1e12, 1)
        dynamic["unit"] = "TOP/s"
        dynamic["note"] = "sasq_dynamic_linear vs sasq_static_linear, same tensors, warm repeat of 5 each"

    # backward of the frozen linear w.r.t. its input (16-bit MFMA GEMM against the prepared dequantized
    # weight): the step that produces each fake-quant operator's upstream gradient during scale training
    bwd_lin = None
    if cfg.name == "c3_mlp7b":
        bwd_lin = {}
        tot_flops, tot_ms = 0.0, 0.0
        gen = torch.Generator(device="cuda").manual_seed(cfg.seed + 11)
        for p in projs:
            if p.wt_bwd is None:
                continue
            dy_out = (torch.randn((p.M, p.N), device="cuda", generator=gen) * 0.01).to(p.x.dtype)
            dx_lin = torch.empty_like(p.x)
            for _ in range(2):
                B.sasq_linear_bwd_input(dy_out, p.wt_bwd, dx_lin, p.K)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                B.sasq_linear_bwd_input(dy_out, p.wt_bwd, dx_lin, p.K)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            bwd_lin[p.name] = {"us": round(1e3 * ms, 1), "tflops": round(p.ops / (ms * 1e-3) / 1e12, 1)}
            tot_ms += ms
            tot_flops += p.ops
            del dy_out, dx_lin
        bwd_lin["achieved"] = round(tot_flops / (tot_ms * 1e-3) / 1e12, 1)
        bwd_lin["peak"] = F16_MFMA_PEAK_TFLOPS
        bwd_lin["unit"] = "TFLOP/s"
        bwd_lin["frac"] = round(bwd_lin["achieved"] / F16_MFMA_PEAK_TFLOPS, 4)
        bwd_lin["note"] = f"sasq_linear_bwd_input, {cfg.dtype} MFMA with fp32 accumulation, warm repeat of 5 per projection"

    out = {
        "metric": "static-scale W8A8 linear TOPS (% int8 MFMA peak); fake-quant fwd+bwd GB/s",
        "value": round(total_ops / (ms_per_step * 1e-3) / 1e12, 2),
        "unit": "TOPS",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "settle_steps": settle, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: LLaMA-2-7B MLP, M=4096 tokens, gate/up 4096->11008, down 11008->4096, "
                               "fp16 activations, int8 per-channel weights, per-tensor static scale; "
                               "step = fake-quant fwd + STE bwd + ds + SGD + static W8A8 linear per projection"
                   if cfg.name == "c3_mlp7b" else cfg.name},
        "roofline": {"bound": "mfma",
                     "kernel": ("sasq_static_linear_batch: all projections of the layer, one activation-quantize launch + one "
                                "int8 MFMA GEMM launch with fused dequantize" if ev["lin_batch"] else
                                "sasq_static_linear (activation quantize + int8 MFMA GEMM + dequant)"),
                     "achieved": round(lin_tops, 1), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(lin_tops / INT8_MFMA_PEAK_TOPS, 4),
                     "sustained_mfma_only": INT8_MFMA_SUSTAINED_TOPS,
                     "frac_of_sustained": round(lin_tops / INT8_MFMA_SUSTAINED_TOPS, 4),
                     "traffic": (C3_LINEAR_BATCH_TRAFFIC_BYTES if ev["lin_batch"] else C3_LINEAR_TRAFFIC_BYTES) if cfg.name == "c3_mlp7b" else None,
                     "traffic_unit": "bytes per call (rocprofv3 FETCH_SIZE/WRITE_SIZE, copy-calibrated)",
                     "algorithmic_bytes": int(sum(3 * p.M * p.K + p.M * p.K + p.wq.numel() + 2 * p.M * p.N + 4 * p.N
                                                  for p in projs) / (1 if ev["lin_batch"] else len(projs))),
                     "avg_launch_us": round(lin_avg_ms * 1e3, 2),
                     "median_launch_us": round(med(lin_all) * 1e3, 2), "min_launch_us": round(lin_all[0] * 1e3, 2)},
        "fakequant": {"bound": "hbm", "achieved": round(fq_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                      "frac": round(fq_gbps / HBM_PEAK_GBPS, 4),
                      "bytes_per_element": 10,
                      "median_us": round(med(fq_all) * 1e3, 2) if fq_all else None,
                      "min_us": round(fq_all[0] * 1e3, 2) if fq_all else None,
                      "note": ("fwd (2+2 B/el) + bwd (2+2+2 B/el); " +
                               ("events around each tensor's pair of launches" if a.unbatched else
                                "one batched launch each for all projection inputs of the layer, events around the two launches; "
                                "per_projection holds the one-launch-per-tensor figures measured after the timed region"))},
        "per_projection": per_proj,
        "fakequant_per_channel": pc,
        "static_linear_grouped": grouped,
        "dynamic_linear": dynamic,
        "linear_bwd_input": bwd_lin,
    }
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, a.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
