"""Build libspin.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2503_15921_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspin.so")
PROBE_LIB = os.path.join(HERE, "libspin_probe.so")   # streaming-read probe of bench.py --calib-stream; not part of the product
SOURCES = ["spin_host.cpp", "spin_ctx.hip", "spin_attn.hip", "spin_accept.hip"]

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions from scalar float code
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        cmd = [hipcc, *HIP_FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "is not a recognized feature for this target" not in l]
        if p.returncode != 0:
            failed = True
        if lines and (verbose or p.returncode != 0):
            print("\n".join(lines), flush=True)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    cmd = [hipcc, *HIP_FLAGS, "-shared", "-x", "hip", os.path.join(CSRC, "stream_probe.hip"), "-o", PROBE_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in out.stdout.splitlines() if "is not a recognized feature for this target" not in l]
    if lines and (verbose or out.returncode != 0):
        print("\n".join(lines), flush=True)
    if out.returncode != 0:
        raise RuntimeError("hipcc failed")
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
