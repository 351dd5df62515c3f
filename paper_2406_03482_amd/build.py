"""Compile the HIP sources of the QJL library into libqjl.so for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqjl.so")
BENCH_LIB = os.path.join(HERE, "libqjl_ceilings.so")      # calibration kernels of bench.py, not part of the library
BENCH_SOURCES = ["bench_ceilings.hip"]
SOURCES = ["qjl_api.hip", "qjl_sketch.hip", "qjl_project.hip", "qjl_quantize.hip",
           "qjl_scores.hip", "qjl_decode.hip", "qjl_outlier.hip", "qjl_values.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the QJL library needs ROCm to build")
    return exe


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compile every source and link libqjl.so next to this file; returns its path."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    for src in SOURCES + BENCH_SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(lines))
        if verbose and lines:
            print("\n".join(lines))
        objs.append(obj)
    for lib, group in ((LIB, objs[:len(SOURCES)]), (BENCH_LIB, objs[len(SOURCES):])):
        cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *group, "-o", lib]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stdout)
        if verbose:
            print(f"built {lib}")
    return LIB


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
