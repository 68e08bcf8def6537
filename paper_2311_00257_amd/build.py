"""Builds the HIP shared libraries in-tree for gfx950 with hipcc.

``python -m paper_2311_00257_amd.build`` compiles
  csrc/amsp_kernels.hip + csrc/amsp_planner.cpp -> libamsp.so   (the C-ABI library of include/amsp.h)
  csrc/synth_fill.hip   -> libamsp_synth.so  (device fill kernels of the input generator)
  csrc/traffic_probe.hip -> libamsp_probe.so (traffic-only kernels timed by bench.py beside the product)
hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")

LIB_AMSP = os.path.join(PKG, "libamsp.so")
LIB_SYNTH = os.path.join(PKG, "libamsp_synth.so")
LIB_PROBE = os.path.join(PKG, "libamsp_probe.so")
LIB_SYNTH_HOST = os.path.join(PKG, "libamsp_synth_host.so")

# packed fp32 instructions are switched off on purpose (they have misbehaved on the test machines)
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument", "-I", INCLUDE]

TARGETS = (((os.path.join(CSRC, "amsp_kernels.hip"), os.path.join(CSRC, "amsp_planner.cpp")), LIB_AMSP),
           ((os.path.join(CSRC, "synth_fill.hip"),), LIB_SYNTH),
           ((os.path.join(CSRC, "traffic_probe.hip"),), LIB_PROBE))


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build_all(extra_flags=(), verbose: bool = True) -> None:
    for srcs, out in TARGETS:
        tmp = out + ".tmp%d" % os.getpid()
        cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-o", tmp, *srcs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, out)
    build_host_synth(force=True)


def build_host_synth(force: bool = False) -> str:
    """gcc-compiles the host-side input generator (plain C, no GPU code)."""
    src = os.path.join(CSRC, "synth_host.c")
    if force or not os.path.exists(LIB_SYNTH_HOST) or os.path.getmtime(LIB_SYNTH_HOST) < os.path.getmtime(src):
        tmp = LIB_SYNTH_HOST + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-o", tmp, src, "-lm"])
        os.replace(tmp, LIB_SYNTH_HOST)
    return LIB_SYNTH_HOST


def built() -> bool:
    return all(os.path.exists(out) for _, out in TARGETS)


if __name__ == "__main__":
    build_all(tuple(sys.argv[1:]))
