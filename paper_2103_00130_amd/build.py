"""Build libabftgemm.so (hand-written HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libabftgemm.so")
SOURCES = ["api.hip", "pack.hip", "gemm_tile.hip", "gemm_tile_a256.hip", "gemm_tile_a256w24.hip", "gemm_tile_a256w42.hip",
           "gemm_tile_a128.hip", "gemm_tile_a64.hip", "gemm_tile_a64r8.hip", "gemm_tile_a64r4.hip", "gemm_tile_a64s.hip", "gemm_tile_a64k2.hip", "gemm_tile_g128.hip", "gemm_tile_g64.hip", "gemm_smallm.hip",
           "rowops.hip", "locate.hip", "eb.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
    # packed-FP32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off",
]


def build_library(force: bool = True, verbose: bool = False, clock_trace: bool = False) -> str:
    """clock_trace: build libabftgemm_clocktrace.so instead, the same sources with ABFT_CLOCK_TRACE defined (tiled
    kernels record cycle and wall counters per workgroup; load it through ABFT_LIBRARY, see bench.py --clock-trace)."""
    if clock_trace:
        return _build(force, verbose, os.path.join(HERE, "_build_clocktrace"), os.path.join(HERE, "libabftgemm_clocktrace.so"),
                      ["-DABFT_CLOCK_TRACE"])
    return _build(force, verbose, os.path.join(HERE, "_build"), LIB, [])


def _build(force, verbose, build_dir, lib, extra) -> str:
    os.makedirs(build_dir, exist_ok=True)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", h) for h in ("abft_gemm.h", "abft_eb.h")]
    newest = max(os.path.getmtime(d) for d in deps)
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < newest:
            cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            print(f"---- {src} failed ----\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(f"---- {src} ----\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    print(build_library(force="--force" in sys.argv, verbose=True, clock_trace="--clock-trace" in sys.argv))
