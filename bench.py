#!/usr/bin/env python3
"""Benchmark of the SASQ hot path on one MI355X.

A "step" is one pass of the whole hot path over the LLaMA-2-7B MLP workload (M = 4096 tokens;
gate, up: K 4096 -> N 11008; down: K 11008 -> N 4096; fp16 activations, int8 weights): for every
projection, fake-quant forward, straight-through backward with the grid-wide ds reduction, one SGD
update of the scale, and the static-inference W8A8 linear.  Inputs are seeded synthetic tensors
already resident in HBM; weights are quantized once, outside the timed region, by the library.

Prints ONE JSON line.  `value` is the linear-layer integer throughput of the whole step
(2*M*N*K summed over the projections, divided by the full step time, fake-quant kernels included),
measured after exactly the W warm-up steps asked for; `settled` repeats the measurement after the
part's power management has settled under the load (about 100 steps).  `roofline` is the static
linear alone, timed with HIP events on the launch stream inside the timed region; `fakequant` is
the fake-quant forward+backward pair against HBM bandwidth; `cpu_baseline` is the CPU oracle on a
bounded row sample of the same workload (all host cores, and one thread).

Cold buffers: the activation-sized tensors exist in `--rotate` (default 2) copies per direction and
every step works on the copy that was touched longest ago, so that whatever a kernel reads was last
touched more than 1 GB of traffic earlier and cannot come from the 256 MB Infinity Cache (the copies
hold the same values: results do not depend on the rotation).  `--rotate 1` keeps one copy (warm).
"""
from __future__ import annotations

import argparse
import ctypes
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
# what a register-only v_mfma_i32_16x16x64_i8 loop (the default GEMM's instruction) sustains on this part with GEMM-like
# operand codes (the part is power-limited under MFMA load; profiles/mfma_peak_and_clock.txt) -- context for `frac`, not
# the roofline's peak
INT8_MFMA_SUSTAINED_TOPS = 4400.0    # 4150-4580 across launches and boxes (python bench.py --mfma-peak)
# HBM-side bytes per static linear call (both kernels) on config 3: RECORDED constants, not read in
# this run: rocprofv3 FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 (factors from a plain 1 GiB copy), from
# the counter passes summarised in profiles/bench_c3_mlp7b_counters.txt.
C3_LINEAR_TRAFFIC_BYTES = 449967 * 1024          # one call per projection, average
C3_LINEAR_BATCH_TRAFFIC_BYTES = 1421507 * 1024   # the batched call (all three projections)
TRAFFIC_SOURCE = "recorded constant from profiles/bench_c3_mlp7b_counters.txt (rocprofv3 FETCH_SIZE/WRITE_SIZE, copy-calibrated), not measured in this run"
HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E, published
LR = 2e-4
ROWMAJOR = False
TDT = {"f16": torch.float16, "bf16": torch.bfloat16}


def dev16(bits: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dtype])


class Projection:
    """One projection: frozen weights prepared once, and `rot` copies of every activation-sized
    tensor per direction.  xf[j] / xhat[j] serve the forward fake-quant of steps with j = step % rot,
    xb[j] / dy[j] / dx[j] the backward, and the static linear reads xb[(j + 1) % rot]."""

    def __init__(self, cfg, proj, xf, xb, ws_small, rot):
        x = xf[0]
        self.name, self.x, self.xf, self.xb = proj.name, x, xf, xb
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
        # frozen weights are re-arranged once at set-up into the GEMM's blocked format (--rowmajor keeps the
        # row-major interchange format instead)
        if self.K % 64 == 0 and not ROWMAJOR:
            wfb = B.SASQ_W_INT8_BLOCKED if wf == B.SASQ_W_INT8 else B.SASQ_W_INT4_BLOCKED
            packed = torch.empty(B.sasq_packed_weight_bytes(self.N, self.K, wfb), dtype=torch.uint8, device="cuda")
            B.sasq_pack_weight(self.wq, packed, self.N, self.K, wf)
            self.wq, self.wf = packed, wfb
        dy0 = dev16(wl.upstream_grad(cfg, proj.name), cfg.dtype)
        self.dy = [dy0] + [dy0.clone() for _ in range(rot - 1)]
        self.s = torch.empty(1, dtype=torch.float32, device="cuda")
        B.sasq_absmax_scale(x, self.s, ws_small, 8)           # s0 = absmax / 127
        self.s0 = self.s.clone()
        self.ds = torch.zeros(1, dtype=torch.float32, device="cuda")
        self.xhat = [torch.empty_like(x) for _ in range(rot)]
        self.dx = [torch.empty_like(x) for _ in range(rot)]
        self.y = torch.empty((self.M, self.N), dtype=x.dtype, device="cuda")
        self.ws_lin = B.new_workspace(B.sasq_static_linear_workspace(self.M, self.N, self.K, wf))
        self.ops = 2.0 * self.M * self.N * self.K
        self.fq_bytes = 10.0 * self.M * self.K            # 2+2 forward, 2+2+2 backward, per operator
        e, wbytes = 2, (1.0 if cfg.w_fmt == wl.W_INT8 else 0.5)
        # bytes the static linear has to move at least: X in, W in, Y out, the per-channel factors
        self.lin_bytes = e * self.M * self.K + wbytes * self.N * self.K + e * self.M * self.N + 4 * self.N
        # what this library adds: the int8 activation codes written by the pre-pass and read by the GEMM
        self.lin_staging_bytes = 2 * self.M * self.K


class Layer:
    """The projections of the workload with their scales in one vector, and the descriptors of
    the batched calls (one launch for all fake-quant operators of the layer), one set per rotation slot."""

    def __init__(self, projs, rot):
        self.projs, self.rot = projs, rot
        n = len(projs)
        self.s_all = torch.cat([p.s for p in projs]).contiguous()
        self.ds_all = torch.zeros(n, dtype=torch.float32, device="cuda")
        for i, p in enumerate(projs):
            p.s, p.ds = self.s_all[i:i + 1], self.ds_all[i:i + 1]
        self.s0_all = self.s_all.clone()
        self.fwd_items = [[(p.xf[j], p.s, p.xhat[j]) for p in projs] for j in range(rot)]
        self.bwd_items = [[(p.xb[j], p.dy[j], p.s, p.dx[j], p.ds) for p in projs] for j in range(rot)]
        self.ws_batch = B.new_workspace(B.sasq_fakequant_bwd_batch_workspace(n))
        self.fq_bytes = sum(p.fq_bytes for p in projs)
        # bytes the two batched launches really move: operators in front of projections that share an
        # activation (gate/up, q/k/v) read it once in the forward launch
        shared_reads = sum(2.0 * p.M * p.K for i, p in enumerate(projs)
                           if any(q.xf[0] is p.xf[0] for q in projs[:i]) and p.M * p.K >= (12 << 20))
        self.fq_bytes_moved = self.fq_bytes - shared_reads
        # the linears of the layer in one batched call (needs one weight format and K % 64 == 0 throughout)
        self.wf = projs[0].wf
        self.lin_items = [[(p.xb[(j + 1) % rot], p.s, p.wq, p.s_w, None, p.y) for p in projs] for j in range(rot)]
        self.lin_batched = all(p.wf == self.wf and p.K % 64 == 0 for p in projs)
        if self.lin_batched:
            self.ws_lin = B.new_workspace(B.sasq_static_linear_batch_workspace(self.lin_items[0], self.wf))
        self.ops = sum(p.ops for p in projs)
        self.step_no = 0


def step(layer, ev=None):
    """One pass of the hot path: fake-quant forward and backward (+ds) of every projection input
    (one batched launch each), SGD on the scales, then the static linear of every projection.
    ev: optional dict of event lists for per-call timing."""
    j = layer.step_no % layer.rot
    layer.step_no += 1
    if ev is not None:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
    B.sasq_fakequant_fwd_batch(layer.fwd_items[j], 8)
    B.sasq_fakequant_bwd_batch(layer.bwd_items[j], layer.ws_batch, 8)
    if ev is not None:
        e1.record()
        ev["fq"].append((e0, e1))
    B.sasq_scale_sgd_vec(layer.s_all, layer.ds_all, LR)
    if layer.lin_batched:
        if ev is not None:
            e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e2.record()
        B.sasq_static_linear_batch(layer.lin_items[j], layer.wf, layer.ws_lin)
        if ev is not None:
            e3.record()
            ev["lin_batch"].append((e2, e3))
        return
    for p in layer.projs:
        if ev is not None:
            e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e2.record()
        B.sasq_static_linear(p.xb[(j + 1) % layer.rot], p.s, p.wq, p.s_w, None, p.y, p.wf, p.ws_lin)
        if ev is not None:
            e3.record()
            ev["lin"].append((e2, e3, p))


def step_unbatched(layer, ws_bwd, ev=None):
    """The same pass with one launch per tensor and call (--unbatched)."""
    j = layer.step_no % layer.rot
    layer.step_no += 1
    for p in layer.projs:
        if ev is not None:
            e0, e1, e2, e3 = (torch.cuda.Event(enable_timing=True) for _ in range(4))
            e0.record()
        B.sasq_fakequant_fwd(p.xf[j], p.s, p.xhat[j], None, 8)
        B.sasq_fakequant_bwd(p.xb[j], p.dy[j], p.s, p.dx[j], p.ds, ws_bwd, 8)
        if ev is not None:
            e1.record()
        B.sasq_scale_sgd(p.s, p.ds, LR)
        if ev is not None:
            e2.record()
        B.sasq_static_linear(p.xb[(j + 1) % layer.rot], p.s, p.wq, p.s_w, None, p.y, p.wf, p.ws_lin)
        if ev is not None:
            e3.record()
            ev["fq_each"].append((e0, e1, p))
            ev["lin"].append((e2, e3, p))


def _oracle_step(cfg, rows: int):
    """The CPU oracle, as it stands, on the first `rows` tokens of every projection's input: seconds, operations."""
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
    return t_total, ops


def cpu_baseline(cfg, rows: int):
    """The oracle timed on all host cores (on `rows` tokens) and on one thread (on rows / cores tokens, so
    that both legs take about the same time).  The oracle is not changed or tuned for this; the thread count
    of its OpenMP loops is limited from outside for the second leg."""
    import oracle
    from threadpoolctl import threadpool_limits
    cores = oracle.threads()
    rows = min(rows, cfg.M)
    t_all, ops_all = _oracle_step(cfg, rows)
    rows1 = min(cfg.M, max(16, rows // max(cores, 1)))
    with threadpool_limits(limits=1, user_api="openmp"):
        one = oracle.threads()
        t_one, ops_one = _oracle_step(cfg, rows1)
    return {"value": ops_all / t_all / 1e12, "unit": "TOPS", "cores": cores, "kind": "oracle",
            "sample": f"first {rows} of {cfg.M} tokens of every projection, whole step "
                      f"(fake-quant fwd+bwd, SGD, static linear); {t_all:.1f} s",
            "single_thread": {"value": ops_one / t_one / 1e12, "unit": "TOPS", "cores": one,
                              "sample": f"first {rows1} tokens, same step; {t_one:.1f} s"}}


def tile_timestamps(cfg, layer, run_step, settle: int):
    """Where the cycles of a tile of the batched GEMM go, in the benchmark's steady state: `settle` steps on the
    instrumented library, then one step whose GEMM workgroups stamp s_memtime / s_memrealtime at body start, after the
    pipeline fill, after the K loop, after the stages have drained and after the epilogue."""
    lib = B._lib()
    lib.sasq_ts_set_buffer.argtypes = [ctypes.c_void_p]
    lib.sasq_ts_set_buffer.restype = ctypes.c_int
    if not layer.lin_batched:
        sys.exit("bench.py: --tile-timestamps stamps the batched GEMM; this configuration does not use it")
    for _ in range(settle):
        run_step()
    torch.cuda.synchronize()
    max_wgs = 1 << 16
    buf = torch.zeros(max_wgs * 16, dtype=torch.int64, device="cuda")
    if lib.sasq_ts_set_buffer(buf.data_ptr()) != 0:
        sys.exit("bench.py: could not set the timestamp buffer")
    run_step()
    torch.cuda.synchronize()
    lib.sasq_ts_set_buffer(None)
    t = buf.cpu().numpy().reshape(max_wgs, 16)
    wg_id = np.nonzero(t[:, 0] != 0)[0]
    t = t[t[:, 0] != 0]
    cyc, wall = t[:, [0, 2, 4, 6, 8]].astype(np.float64), t[:, [1, 3, 5, 7, 9]].astype(np.float64)
    K, half = t[:, 14], t[:, 15]
    span_us = (wall[:, 4].max() - wall[:, 0].min()) / 100.0
    total_us = (wall[:, 4] - wall[:, 0]) / 100.0
    out = {"metric": "cycles per tile of the batched int8 GEMM (instrumented build), medians over the tiles of one call",
           "config": cfg.name, "workgroups": int(len(t)), "kernel_span_us": round(span_us, 1),
           "sum_of_tile_times_over_256_us": round(float(total_us.sum()) / 256.0, 1),
           "shader_clock_ghz": round(float(np.median((cyc[:, 4] - cyc[:, 0]) / np.maximum(total_us, 1e-9)) / 1e3), 3), "tiles": []}
    # Between two tiles on one CU: workgroup ids go to the eight XCDs in turn and an XCD holds 32 workgroups of this
    # kernel at a time, so within an XCD the (32 + j)-th workgroup to start took the place of the j-th to end.
    gaps = []
    for x in range(8):
        m = wg_id % 8 == x
        starts, ends = np.sort(wall[m, 0]), np.sort(wall[m, 4])
        if len(starts) > 32:
            gaps.append((starts[32:] - ends[:len(starts) - 32]) / 100.0)
    if gaps:
        g = np.concatenate(gaps)
        out["between_tiles_us"] = {"median": round(float(np.median(g)), 2), "p10": round(float(np.percentile(g, 10)), 2),
                                   "p90": round(float(np.percentile(g, 90)), 2), "count": int(len(g)),
                                   "note": "end of a workgroup's last stamp to the first stamp of the workgroup that took its place "
                                           "(matched by order within each XCD; the realtime counter ticks every 10 ns)"}
    last = np.sort(wall[:, 4])[-256:] if len(wall) >= 256 else wall[:, 4]
    out["idle_at_the_end_us"] = round(float((wall[:, 4].max() - last).mean() / 100.0), 1)   # mean over the CUs' last tiles
    out["xcd_done_before_the_end_us"] = [round(float((wall[:, 4].max() - wall[wg_id % 8 == x, 4].max()) / 100.0), 1) for x in range(8)]
    for k in sorted(set(K.tolist())):
        for h in (0, 1, 2):
            m = (K == k) & (half == h)
            if not m.any():
                continue
            kt = int(k) // 64
            d = np.diff(cyc[m], axis=1)                # fill, K loop, drain, epilogue
            med = np.median(d, axis=0)
            out["tiles"].append({"K": int(k), "shape": "256x256" if h == 0 else "128x256 (split last round)", "count": int(m.sum()),
                                 "fill": int(med[0]), "k_loop": int(med[1]), "per_k_tile": round(float(med[1]) / kt, 1),
                                 "per_k_tile_p10_p90": [round(float(np.percentile(d[:, 1], q)) / kt, 1) for q in (10, 90)],
                                 "mfma_issue_per_k_tile": 1024 if h == 0 else 512,
                                 "drain": int(med[2]), "epilogue": int(med[3]), "total": int(np.median(cyc[m][:, 4] - cyc[m][:, 0])),
                                 "total_us": round(float(np.median(total_us[m])), 1)})
    print(json.dumps(out))


def load_probe():
    """The benchmark's register-only MFMA loop (paper_2512_14481_amd/bench_csrc, built by the package's build step
    into libsasq_bench.so): tooling of this script, not an entry point of the SASQ library."""
    path = os.path.join(ROOT, "paper_2512_14481_amd", "libsasq_bench.so")
    if not os.path.exists(path):
        sys.exit(f"bench.py: {path} is missing: build it with `python -m paper_2512_14481_amd.build`")
    fn = ctypes.CDLL(path).sasq_bench_mfma_probe
    fn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    fn.restype = ctypes.c_int
    return fn


def mfma_peak():
    """What the part's matrix units sustain on their own (register-only loop, GEMM register pattern),
    per operand pattern: TOP/s of each of 80 back-to-back launches (about 0.5 s of load per pattern)."""
    probe = load_probe()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    sink = torch.empty(65536, dtype=torch.int32, device="cuda")
    iters, launches = 20000, 80
    out = {"metric": "register-only MFMA loop, sustained", "unit": "TOP/s (TFLOP/s for f16)", "iters_per_launch": iters,
           "launches": launches, "patterns": {}}
    for kind, name, ops in ((0, "i8 32x32x32 zeros", 65536.0), (1, "i8 32x32x32 random bits", 65536.0),
                            (2, "i8 32x32x32 GEMM-like codes", 65536.0), (5, "i8 16x16x64 zeros", 131072.0),
                            (4, "i8 16x16x64 GEMM-like codes", 131072.0),
                            (3, "f16 32x32x16 small random values", 32768.0)):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
        torch.cuda.synchronize()
        ev[0].record()
        for l in range(launches):
            if probe(kind, iters, ctypes.c_void_p(sink.data_ptr()), stream) != 0:
                sys.exit("bench.py: the MFMA probe rejected its arguments or failed to launch")
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
    ap.add_argument("--settle-steps", type=int, default=200,
                    help="after the timed region asked for, keep stepping until this many steps have run in all, then "
                         "time K steps again and report them as `settled` (0: skip)")
    ap.add_argument("--rotate", type=int, default=2,
                    help="copies of every activation-sized tensor per direction, used in turn (cold buffers); 1: one copy (warm)")
    ap.add_argument("--config", default="c3_mlp7b")
    ap.add_argument("--cpu-rows", type=int, default=4096)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--unbatched", action="store_true",
                    help="one launch per tensor for the fake-quant operators instead of one per layer")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="instead of the workload: time the library's register-only MFMA loop under sustained load "
                         "(80 back-to-back launches per operand pattern) and print what the matrix units sustain")
    ap.add_argument("--tile-timestamps", action="store_true",
                    help="instead of the timings: run the workload on the instrumented build of the library (libsasq_ts.so: "
                         "cycle and wall-clock stamps at five points of every tile of the batched GEMM), settle for W + K steps, "
                         "stamp one step and print where a tile's cycles go")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE",
                    help="force a kernel variant through sasq_set_tuning for the whole run (for profiles that compare variants): "
                         "path=twopass|fused, tile=256|128x256|128, mfma=32x32x32|16x16x64; path and tile act on single calls, "
                         "so combine them with --unbatched")
    ap.add_argument("--rowmajor", action="store_true", help="keep the weights in the row-major interchange format")
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

    if a.tile_timestamps:
        ts_lib = os.path.join(ROOT, "paper_2512_14481_amd", "libsasq_ts.so")
        if not os.path.exists(ts_lib):
            sys.exit(f"bench.py: {ts_lib} is missing: build it with `python -m paper_2512_14481_amd.build`")
        B.LIB_PATH = ts_lib                            # before the binding loads anything: same entry points, stamped GEMM

    knobs = {"path": (B.SASQ_TUNE_LINEAR_PATH, {"twopass": 1, "fused": 2}),
             "tile": (B.SASQ_TUNE_LINEAR_TILE, {"256": 1, "128x256": 2, "128": 3}),
             "mfma": (B.SASQ_TUNE_LINEAR_MFMA, {"32x32x32": 1, "16x16x64": 2})}
    for t in a.tune:
        name, _, val = t.partition("=")
        if name not in knobs or val not in knobs[name][1]:
            sys.exit(f"bench.py: unknown --tune {t}")
        B.sasq_set_tuning(knobs[name][0], knobs[name][1][val])
    global ROWMAJOR
    ROWMAJOR = a.rowmajor or any(t.startswith("path=") for t in a.tune)   # both activation paths exist for row-major weights only

    cfg = wl.CONFIGS[a.config]
    rot = max(1, a.rotate)
    ws_small = B.new_workspace(max(B.sasq_absmax_scale_workspace(1, 1), B.sasq_fakequant_bwd_workspace(1, 1)))
    acts_f, acts_b = {}, {}
    for act in cfg.acts:
        x0 = dev16(wl.activation(cfg, act.name), cfg.dtype)
        acts_f[act.name] = [x0] + [x0.clone() for _ in range(rot - 1)]
        acts_b[act.name] = [x0.clone() for _ in range(rot)] if rot > 1 else [x0]
    projs = [Projection(cfg, p, acts_f[p.x], acts_b[p.x], ws_small, rot) for p in cfg.projs]
    layer = Layer(projs, rot)
    run_step = (lambda ev=None: step_unbatched(layer, ws_small, ev)) if a.unbatched else (lambda ev=None: step(layer, ev))
    torch.cuda.synchronize()

    if a.tile_timestamps:
        tile_timestamps(cfg, layer, run_step, a.warmup + a.steps)
        return

    if a.calib:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                                 # 1 GiB read + 1 GiB written by a plain copy kernel
        torch.cuda.synchronize()
        del src, dst

    total_ops = sum(p.ops for p in projs)

    def timed(steps):
        """Time `steps` steps (host clock around the loop, events around the calls inside)."""
        layer.s_all.copy_(layer.s0_all)               # every timed run starts from the same scales
        torch.cuda.synchronize()
        ev = {"fq": [], "fq_each": [], "lin": [], "lin_batch": []}
        t0 = time.perf_counter()
        for _ in range(steps):
            run_step(ev)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        r = {"ev": ev, "ms_per_step": dt / steps * 1e3}
        if ev["lin_batch"]:
            lin_all = sorted(e0.elapsed_time(e1) for e0, e1 in ev["lin_batch"])
            r["lin_ops_per_call"] = total_ops
        else:
            lin_all = sorted(e0.elapsed_time(e1) for e0, e1, _ in ev["lin"])
            r["lin_ops_per_call"] = total_ops / len(projs)     # average over the projections' calls
        r["lin_all"] = lin_all
        r["lin_avg_ms"] = sum(lin_all) / len(lin_all)
        r["lin_tops"] = r["lin_ops_per_call"] / (r["lin_avg_ms"] * 1e-3) / 1e12
        if a.unbatched:
            fq_all = sorted(e0.elapsed_time(e1) for e0, e1, _ in ev["fq_each"])
            r["fq_ms_per_step"] = sum(fq_all) / steps
        else:
            fq_all = sorted(e0.elapsed_time(e1) for e0, e1 in ev["fq"])
            r["fq_ms_per_step"] = sum(fq_all) / len(fq_all)
        r["fq_all"] = fq_all
        r["fq_gbps"] = layer.fq_bytes / (r["fq_ms_per_step"] * 1e-3) / 1e9
        r["fq_gbps_moved"] = (layer.fq_bytes if a.unbatched else layer.fq_bytes_moved) / (r["fq_ms_per_step"] * 1e-3) / 1e9
        return r

    # 1. exactly what was asked for: W untimed warm-up steps, then K timed steps
    for _ in range(a.warmup):
        run_step()
    asked = timed(a.steps)
    # 2. the same measurement once the part has settled under the load.  The GEMM's time keeps moving for
    #    about 80 steps of continuous load (power management first over-throttles, then relaxes); a serving or
    #    training job sits in that state.  Steps run so far count towards the settling.
    done = a.warmup + a.steps
    for _ in range(max(0, a.settle_steps - done)):
        run_step()
    settled = timed(a.steps) if a.settle_steps > 0 else None

    # per-projection figures: the unbatched pass, outside the timed regions
    ev = asked["ev"]
    if not a.unbatched:
        layer.s_all.copy_(layer.s0_all)
        ev = {"fq": [], "fq_each": [], "lin": [], "lin_batch": []}
        for _ in range(4 * rot + 1):
            step_unbatched(layer, ws_small, ev)
        torch.cuda.synchronize()
    lin_ms = [(e0.elapsed_time(e1), p) for e0, e1, p in ev["lin"]]
    fq_ms = [(e0.elapsed_time(e1), p) for e0, e1, p in ev["fq_each"]]
    med = lambda v: v[len(v) // 2] if v else None
    per_proj = {}
    for pp in projs:
        tl = [t for t, p in lin_ms if p.name == pp.name]
        tf = [t for t, p in fq_ms if p.name == pp.name]
        tl_med, tf_med = med(sorted(tl)), med(sorted(tf))      # medians: a first call on fresh buffers can be far out
        per_proj[pp.name] = {"linear_us": round(1e3 * tl_med, 2),
                             "linear_tops": round(pp.ops / (tl_med * 1e-3) / 1e12, 1),
                             "fakequant_fwd_bwd_us": round(1e3 * tf_med, 2),
                             "fakequant_gbps": round(pp.fq_bytes / (tf_med * 1e-3) / 1e9, 1),
                             "fakequant_frac": round(pp.fq_bytes / (tf_med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
    ms_per_step = asked["ms_per_step"]

    # the single-tensor operators on their own: nothing but the forward and backward launches of one tensor, over
    # enough distinct copies (about 1.5 GB) that every launch reads cold memory; one entry per tensor size of the config
    single = {}
    for pp in projs:
        n = pp.M * pp.K
        if str(n) in single:
            continue
        sets = max(2, int(1.5e9 // (n * 8)))
        xs = [pp.xf[0].clone() for _ in range(sets)]
        dys = [pp.dy[0].clone() for _ in range(sets)]
        ys = [torch.empty_like(pp.xf[0]) for _ in range(sets)]
        dxs = [torch.empty_like(pp.xf[0]) for _ in range(sets)]
        def pair(i):
            B.sasq_fakequant_fwd(xs[i % sets], pp.s, ys[i % sets], None, 8)
            B.sasq_fakequant_bwd(xs[(i + sets // 2) % sets], dys[i % sets], pp.s, dxs[i % sets], pp.ds, ws_small, 8)
        for i in range(sets):
            pair(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 6 * sets
        e0.record()
        for i in range(reps):
            pair(i)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        single[str(n)] = {"shape": [pp.M, pp.K], "fwd_bwd_us": round(us, 2), "gbps": round(10 * n / us / 1e3, 1),
                          "frac": round(10 * n / us / 1e3 / HBM_PEAK_GBPS, 4), "copies": sets}
        del xs, dys, ys, dxs

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
                B.sasq_fakequant_fwd_pc(p.x, sv, p.xhat[0], None, 8)
                B.sasq_fakequant_bwd_pc(p.x, p.dy[0], sv, p.dx[0], dsv, wsp, 8)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                B.sasq_fakequant_fwd_pc(p.x, sv, p.xhat[0], None, 8)
                B.sasq_fakequant_bwd_pc(p.x, p.dy[0], sv, p.dx[0], dsv, wsp, 8)
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
        fwd_items = [(p.x, svs[i], p.xhat[0]) for i, p in enumerate(projs)]
        bwd_items = [(p.x, p.dy[0], svs[i], p.dx[0], dsvs[i]) for i, p in enumerate(projs)]
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

    # static linear with one activation factor per group of 32 / 128 / 512 input channels (the grouped form
    # the paper gives for per-channel activation factors), measured after the timed region
    grouped = None
    if cfg.name == "c3_mlp7b":
        grouped = {}
        for group in (32, 128, 512):
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
        # the strict per-channel case (group = 1) has no MFMA form: a scalar kernel, timed once on the gate projection
        p = projs[0]
        if p.wf in (B.SASQ_W_INT8, B.SASQ_W_INT4_PACKED):
            wq1, wf1 = p.wq, p.wf
        else:                                              # the scalar kernel takes the row-major interchange format
            wf1 = B.SASQ_W_INT8 if cfg.w_fmt == wl.W_INT8 else B.SASQ_W_INT4_PACKED
            w = torch.from_numpy(wl.weight_fp32(cfg, p.name)).cuda()
            wq1 = torch.empty((p.N, p.K if wf1 == B.SASQ_W_INT8 else p.K // 2),
                              dtype=torch.int8 if wf1 == B.SASQ_W_INT8 else torch.uint8, device="cuda")
            B.sasq_quantize_weight(w, wq1, torch.empty_like(p.s_w), wf1)
            del w
        sg1 = p.s.expand(p.K).contiguous()
        B.sasq_static_linear_grouped(p.x, sg1, wq1, p.s_w, None, p.y, 1, wf1, p.ws_lin)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.sasq_static_linear_grouped(p.x, sg1, wq1, p.s_w, None, p.y, 1, wf1, p.ws_lin)
        e1.record()
        torch.cuda.synchronize()
        ms1 = e0.elapsed_time(e1)
        grouped["group_1"] = {"achieved": round(p.ops / (ms1 * 1e-3) / 1e12, 2), "unit": "TOP/s", "us_per_call": round(1e3 * ms1, 1),
                              "calls": 1, "note": "scalar kernel (one thread per output), gate projection, one timed call"}
        del wq1, sg1
        grouped["note"] = ("sasq_static_linear_grouped on the projections whose K the group divides "
                           "(gate, up, down for 32 and 128; gate, up for 512); warm repeat of 5.  group_32 "
                           "multiplies every 64-channel K tile twice (half of the channels zeroed each time): its "
                           "TOP/s counts the useful operations only")

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

    def roofline_of(r):
        lin_all = r["lin_all"]
        return {"achieved": round(r["lin_tops"], 1), "frac": round(r["lin_tops"] / INT8_MFMA_PEAK_TOPS, 4),
                "avg_launch_us": round(r["lin_avg_ms"] * 1e3, 2), "median_launch_us": round(med(lin_all) * 1e3, 2),
                "min_launch_us": round(lin_all[0] * 1e3, 2)}

    def fakequant_of(r):
        return {"achieved": round(r["fq_gbps"], 1), "frac": round(r["fq_gbps"] / HBM_PEAK_GBPS, 4),
                "achieved_bytes_moved": round(r["fq_gbps_moved"], 1), "frac_bytes_moved": round(r["fq_gbps_moved"] / HBM_PEAK_GBPS, 4),
                "us_per_step": round(r["fq_ms_per_step"] * 1e3, 2), "median_us": round(med(r["fq_all"]) * 1e3, 2),
                "min_us": round(r["fq_all"][0] * 1e3, 2)}

    batched = bool(asked["ev"]["lin_batch"])
    calls = 1 if batched else len(projs)
    roof = {"bound": "mfma",
            "kernel": ("sasq_static_linear_batch: all projections of the layer, one activation-quantize launch + one "
                       "int8 MFMA GEMM launch with fused dequantize" if batched else
                       "sasq_static_linear (activation quantize + int8 MFMA GEMM + dequant)"),
            "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s"}
    roof.update(roofline_of(asked))
    roof.update({"note": "timed right after the warm-up asked for; for about 100 steps after an idle period the part's power management "
                         "runs this kernel 10-25 % slower than in steady state: `settled` holds the steady-state figure of the same run",
                 "sustained_mfma_only": INT8_MFMA_SUSTAINED_TOPS,
                 "frac_of_sustained": round(asked["lin_tops"] / INT8_MFMA_SUSTAINED_TOPS, 4),
                 "traffic": (C3_LINEAR_BATCH_TRAFFIC_BYTES if batched else C3_LINEAR_TRAFFIC_BYTES) if cfg.name == "c3_mlp7b" else None,
                 "traffic_unit": "bytes per call", "traffic_source": TRAFFIC_SOURCE if cfg.name == "c3_mlp7b" else None,
                 "algorithmic_bytes": int(sum(p.lin_bytes for p in projs) / calls),
                 "algorithmic_bytes_formula": "sum over projections of e*M*K + w*N*K + e*M*N + 4*N (e = 2, w = 1 or 0.5)",
                 "staging_bytes": int(sum(p.lin_staging_bytes for p in projs) / calls),
                 "staging_note": "int8 activation codes written by the library's pre-pass and read by its GEMM (not algorithmic)"})
    fq = {"bound": "hbm", "peak": HBM_PEAK_GBPS, "unit": "GB/s", "bytes_per_element": 10}
    fq.update(fakequant_of(asked))
    fq["bytes_counted"] = int(layer.fq_bytes)
    fq["bytes_moved"] = int(layer.fq_bytes if a.unbatched else layer.fq_bytes_moved)
    fq["single_tensor_alone"] = single
    fq["single_tensor_alone_note"] = ("sasq_fakequant_fwd + sasq_fakequant_bwd of ONE tensor per launch pair, back to back over `copies` "
                                      "distinct sets of buffers (cold), nothing else running; per_projection times the same pair inside "
                                      "the unbatched step, between GEMMs")
    fq["protocol"] = (f"cold: {rot} copies of x, dy, x', dx per direction used in turn; whatever a launch reads was last touched "
                      "more than 1 GB of traffic earlier" if rot > 1 else "warm: one copy of every tensor")
    fq["note"] = ("achieved/frac count 10 B/element per operator (fwd 2+2, bwd 2+2+2); operators in front of projections that "
                  "share an activation read it once in the forward launch: *_bytes_moved count what is really moved; " +
                  ("events around each tensor's pair of launches" if a.unbatched else
                   "one batched launch each way for all projection inputs of the layer, events around the two launches; "
                   "per_projection holds the one-launch-per-tensor figures measured after the timed region"))
    out = {
        "metric": "static-scale W8A8 linear TOPS (% int8 MFMA peak); fake-quant fwd+bwd GB/s",
        "value": round(total_ops / (ms_per_step * 1e-3) / 1e12, 2),
        "unit": "TOPS",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: LLaMA-2-7B MLP, M=4096 tokens, gate/up 4096->11008, down 11008->4096, "
                               "fp16 activations, int8 per-channel weights, per-tensor static scale; "
                               "step = fake-quant fwd + STE bwd + ds + SGD + static W8A8 linear per projection"
                   if cfg.name == "c3_mlp7b" else cfg.name,
                   "buffers": fq["protocol"]},
        "roofline": roof,
        "fakequant": fq,
        "settled": None if settled is None else {
            "note": f"the same {a.steps} timed steps repeated after {max(done, a.settle_steps)} steps of continuous load",
            "value": round(total_ops / (settled["ms_per_step"] * 1e-3) / 1e12, 2), "ms_per_step": round(settled["ms_per_step"], 4),
            "roofline": roofline_of(settled), "fakequant": fakequant_of(settled)},
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
