"""Builds libdsq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdsq.so")
SOURCES = ["dsq_tile_quant4.hip", "dsq_tile_quant2.hip", "dsq_tile_quant8.hip", "dsq_tile_sign.hip", "dsq_tile_misc.hip", "dsq_host.cpp", "dsq_api.hip",
           "dsq_topk_kernels.hip", "dsq_l2norm_kernels.hip", "dsq_workload_kernels.hip",
           "dsq_compare_quant4.hip", "dsq_compare_quant2.hip", "dsq_compare_quant8.hip", "dsq_compare_sign.hip"]

# -ffp-contract=off: every fused multiply-add in the kernels is written out as fmaf, nothing else may fuse
#  (bit-level agreement of codes and scales depends on it).  The packed-fp32 feature is switched off because
#  some packed forms have been seen to give wrong results on this hardware.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


ID_FILE = LIB + ".id"


def source_id(extra_flags=()) -> str:
    """Hash of everything the library is built from: sources, headers, flags."""
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h", ".cpp")))
    for path in files + [os.path.join(ROOT, "include", "dsq.h")]:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join([*FLAGS, *extra_flags]).encode())
    return h.hexdigest()[:16]


def build(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    build_id = source_id(extra_flags)
    objs, procs = [], []
    for src in SOURCES:                                       # the translation units compile side by side
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *FLAGS, *extra_flags, f'-DDSQ_BUILD_ID="{build_id}"', "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
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
    with open(ID_FILE, "w") as f:
        f.write(build_id + "\n")
    return LIB


def built_id() -> str:
    """The source hash the library on disk was built from ("" if there is none, or it predates the hash)."""
    if not (os.path.exists(LIB) and os.path.exists(ID_FILE)):
        return ""
    with open(ID_FILE) as f:
        return f.read().strip()


def ensure_built(verbose: bool = False) -> str:
    """Builds the library unless the one on disk was built from exactly the present sources and flags (tests, the
    smoke check and the benchmark call this before loading it: a stale binary must not answer for the sources)."""
    return LIB if built_id() == source_id() else build(verbose=verbose)


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
