"""Build libcofree.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2308_03209_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcofree.so")
GATHER_CEILING = os.path.join(HERE, "gather_ceiling")   # stand-alone micro-benchmark (csrc/gather_ceiling.hip)
SOURCES = ["partition.cpp", "dropedge.hip", "spmm.hip", "gemm.hip", "gemm_bf16.hip", "loss_step.hip", "layers.cpp", "profile.cpp"]
HEADERS = [os.path.join(CSRC, "common.h"), os.path.join(HERE, "..", "include", "cofree.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    if not os.path.exists(GATHER_CEILING) or os.path.getmtime(os.path.join(CSRC, "gather_ceiling.hip")) > os.path.getmtime(GATHER_CEILING):
        return True
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = True) -> str:
    """Compile every translation unit and link the shared library.  Returns its path."""
    if not force and not stale():
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()
    procs = []
    objs = []
    for s in SOURCES:
        obj = os.path.join(objdir, s + ".o")
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, s), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if out and verbose:
            print(out)
        if p.returncode != 0:
            failed = True
            print(f"[build] {s} failed", file=sys.stderr)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB + ".tmp", "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(LIB + ".tmp", LIB)
    # the bare-gather micro-benchmark the aggregation kernels are held against (a program of its own)
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unknown-warning-option", os.path.join(CSRC, "gather_ceiling.hip"), "-o",
           GATHER_CEILING + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if out and verbose:
        print(out)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed on gather_ceiling.hip")
    os.replace(GATHER_CEILING + ".tmp", GATHER_CEILING)
    return LIB


if __name__ == "__main__":
    build(force=True)
    print("built", LIB)
