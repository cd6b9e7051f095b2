"""Builds libdsq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdsq.so")
SOURCES = ["dsq_tile_quant4.hip", "dsq_tile_quant2.hip", "dsq_tile_quant8.hip", "dsq_tile_sign.hip", "dsq_tile_misc.hip", "dsq_host.cpp", "dsq_api.hip",
           "dsq_topk_kernels.hip", "dsq_l2norm_kernels.hip", "dsq_workload_kernels.hip"]

# -ffp-contract=off: every fused multiply-add in the kernels is written out as fmaf, nothing else may fuse
#  (bit-level agreement of codes and scales depends on it).  The packed-fp32 feature is switched off because
#  some packed forms have been seen to give wrong results on this hardware.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def build(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs, procs = [], []
    for src in SOURCES:                                       # the translation units compile side by side
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
               os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd)))
        objs.append(obj)
    for cmd, proc in procs:
        if proc.wait() != 0:
            raise subprocess.CalledProcessError(proc.returncode, cmd)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def ensure_built(verbose: bool = False) -> str:
    """Builds the library only if no built one is there (tests, the smoke check and the benchmark call this)."""
    return LIB if os.path.exists(LIB) else build(verbose=verbose)


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
