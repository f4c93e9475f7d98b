"""Builds libpb.so (HIP kernels + host tree compiler + C ABI) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
# (PB_LIBRARY: load another build of the library, e.g. one compiled with different tuning constants for a sweep)
LIB = os.environ.get("PB_LIBRARY") or os.path.join(PKG, "libpb.so")
PROBE_LIB = os.path.join(PKG, "libpb_probe.so")  # measurement probes of bench.py, not part of the product library
SOURCES = ["pb_compile.cpp", "pb_kernels.hip", "pb_frames.hip", "pb_wide.hip", "pb_api.hip"]
HEADERS = ["pb_tree.hpp", "pb_kernels.hpp", "pb_wave.hpp", os.path.join(ROOT, "include", "pb.h")]
OBJDIR = os.path.join(PKG, "_build")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    # packed-fp32 instructions stay off: some of their forms have given wrong results on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the leading scalar and pointer arguments of a kernel are in registers when its waves start (the single-step
    # kernels are a few dependent memory accesses long; the fetch of the argument block was one of them)
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def compile_command(src: str, obj: str, extra=()) -> list:
    return ["hipcc", "-c"] + FLAGS + list(extra) + ["-o", obj, os.path.join(CSRC, src)]


def link_command(objs, out: str = LIB) -> list:
    return ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + list(objs)


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False, extra=(), out: str = LIB) -> str:
    """Compiles the library (one hipcc process per source, side by side); with force=False only when it is missing."""
    if not force and os.path.exists(out):
        return out
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJDIR, exist_ok=True)
    tag = "" if out == LIB else "." + os.path.basename(out)
    objs = [os.path.join(OBJDIR, s + tag + ".o") for s in SOURCES]

    def one(pair):
        cmd = compile_command(pair[0], pair[1], extra)
        if verbose:
            print(" ".join(cmd), file=sys.stderr)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
        list(pool.map(one, zip(SOURCES, objs)))
    cmd = link_command(objs, out)
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return out


def build_probe(force: bool = True, verbose: bool = False) -> str:
    """Compiles the bench-only probe library."""
    if not force and os.path.exists(PROBE_LIB):
        return PROBE_LIB
    cmd = ["hipcc", "-shared"] + FLAGS + ["-o", PROBE_LIB, os.path.join(CSRC, "pb_probe.hip")]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return PROBE_LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    build_probe(force=True, verbose=True)
    print(LIB)
