"""Build the SASQ HIP library (libsasq.so) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsasq.so")
BENCH_CSRC = os.path.join(PKG, "bench_csrc")
BENCH_LIB = os.path.join(PKG, "libsasq_bench.so")    # benchmark tooling (register-only MFMA probe), not part of the C ABI
TS_LIB = os.path.join(PKG, "libsasq_ts.so")          # benchmark tooling: the library with per-tile timestamps in the batched GEMM
TS_SOURCE = "static_linear_k64.hip"                  # the one source the instrumented build compiles differently

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # the numerical contract pins every fp32 rounding
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(ROOT, "include", "sasq.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = True, incremental: bool = False) -> str:
    """Compile every source to an object file (in parallel: the GEMM file alone takes two minutes),
    then link.  Objects live in a temporary directory; only libsasq.so stays in the tree.
    incremental=True (a developer's shortcut, `python -m paper_2512_14481_amd.build -i`) keeps the
    objects in _build/ at the repository root and recompiles only sources newer than their object
    (every source after a header change)."""
    import concurrent.futures
    import contextlib
    import tempfile

    compile_flags = [f for f in FLAGS if f != "-shared"]
    headers = glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(ROOT, "include", "sasq.h")]
    if incremental:
        keep = os.path.join(ROOT, "_build")
        os.makedirs(keep, exist_ok=True)
        tmp_ctx = contextlib.nullcontext(keep)
    else:
        tmp_ctx = tempfile.TemporaryDirectory(prefix="sasq_build_")
    with tmp_ctx as tmp:
        def compile_one(src: str) -> str:
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            if incremental and os.path.exists(obj) and all(os.path.getmtime(d) <= os.path.getmtime(obj) for d in [src] + headers):
                return obj
            cmd = [HIPCC] + compile_flags + ["-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj

        def compile_ts(src: str) -> str:
            obj = os.path.join(tmp, os.path.basename(src) + ".ts.o")
            if incremental and os.path.exists(obj) and all(os.path.getmtime(d) <= os.path.getmtime(obj) for d in [src] + headers):
                return obj
            cmd = [HIPCC] + compile_flags + ["-DSASQ_GEMM_TIMESTAMPS", "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj

        srcs = sources()
        workers = max(1, min(len(srcs) + 1, int(os.environ.get("MAX_JOBS", "0")) or os.cpu_count() or 1))
        with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
            ts_future = pool.submit(compile_ts, os.path.join(CSRC, TS_SOURCE))
            objs = list(pool.map(compile_one, srcs))
            ts_obj = ts_future.result()
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
        # the same library with the instrumented GEMM object in place of the plain one
        ts_objs = [ts_obj if os.path.basename(o) == TS_SOURCE + ".o" else o for o in objs]
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", TS_LIB] + ts_objs
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    # the benchmark's own tooling: one small library beside the product
    bench_srcs = sorted(glob.glob(os.path.join(BENCH_CSRC, "*.hip")))
    if bench_srcs and not (incremental and os.path.exists(BENCH_LIB) and
                           all(os.path.getmtime(f) <= os.path.getmtime(BENCH_LIB) for f in bench_srcs)):
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
               "-o", BENCH_LIB] + bench_srcs
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(incremental="-i" in sys.argv[1:])
    sys.exit(0)
