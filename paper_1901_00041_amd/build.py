"""Builds libst_conv.so and libst_bench_probe.so (HIP, gfx950 only) in-tree with hipcc.

Run: python -m paper_1901_00041_amd.build [--incremental]
Every call compiles every source (objects in parallel); --incremental skips objects newer than their sources
and headers (a convenience while developing)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJDIR = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libst_conv.so")
SOURCES = ["st_kernels.hip", "st_chain.hip", "st_plan.cpp", "st_chain.cpp"]
# the benchmark's achievable-roof probe: its own small library, not part of the convolution library's ABI
PROBE_LIB = os.path.join(PKG, "libst_bench_probe.so")
PROBE_SOURCES = ["st_bench_probe.hip"]
# packed fp32 instructions are switched off for all device code (they are not needed here)
CFLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-pthread", "-x", "hip",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-command-line-argument"]
NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def _headers_mtime() -> float:
    hs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return max(os.path.getmtime(h) for h in hs)


def _objects(sources, verbose, extra, incremental):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    hm = _headers_mtime()
    jobs, objs = [], []
    for s in sources:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJDIR, s + ".o")
        objs.append(obj)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), hm):
            continue
        jobs.append([hipcc] + CFLAGS + list(extra) + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=max(1, len(jobs))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    return objs


def _link(objs, lib, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread"] + objs + ["-o", lib], verbose)
    return lib


def build(verbose: bool = False, extra=(), incremental: bool = False) -> str:
    objs = _objects(SOURCES + PROBE_SOURCES, verbose, extra, incremental)
    _link(objs[len(SOURCES):], PROBE_LIB, verbose)
    return _link(objs[:len(SOURCES)], LIB, verbose)


if __name__ == "__main__":
    args = sys.argv[1:]
    inc = "--incremental" in args
    print(build(verbose=True, extra=[a for a in args if a != "--incremental"], incremental=inc))
