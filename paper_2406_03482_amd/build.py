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


def build_host_sanitizer_driver(verbose: bool = False) -> str:
    """The library's sources compiled with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST code only
    (the device code is compiled as usual and never runs), linked with tests/host/abi_sanitize.cpp into an
    executable that exercises what the host decides by itself: argument validation and the decode planner.
    Returns the executable's path; rebuilt only when a source is newer."""
    objdir = os.path.join(HERE, "_build", "host_sanitize")
    os.makedirs(objdir, exist_ok=True)
    exe = os.path.join(objdir, "abi_sanitize")
    driver = os.path.join(ROOT, "tests", "host", "abi_sanitize.cpp")
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [driver, os.path.join(ROOT, "include", "qjl.h")]
    if os.path.exists(exe) and all(os.path.getmtime(exe) >= os.path.getmtime(d) for d in deps):
        return exe
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g"] + san
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc (host sanitizers) failed on {src}:\n" + out)
        objs.append(obj)
    cmd = [hipcc(), "--offload-arch=gfx950", "-O1", "-g", *san, "-I", os.path.join(ROOT, "include"), "-x", "hip", driver,
           "-x", "none", *objs, "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link of the sanitizer driver failed:\n" + r.stdout)
    if verbose:
        print(f"built {exe}")
    return exe


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
