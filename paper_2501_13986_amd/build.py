"""Builds libcgtp.so (the C-ABI library) in-tree with hipcc for gfx950.

Usage: python -m paper_2501_13986_amd.build   (also called by __graft_entry__.build()).
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcgtp.so")
SOURCES = ["api.cpp", "cg_real.cpp", "emit_uvu.cpp", "emit_uvw.cpp", "emit_uvw_ps.cpp", "jit.cpp", "csr.hip"]
# packed fp32 instructions are disabled for every HIP translation unit of this project
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, "-c", "-O2", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-result", "-D__HIP_PLATFORM_AMD__",
               os.path.join(CSRC, src), "-o", obj]
        if src.endswith(".hip"):
            cmd += DEVICE_FLAGS
        else:
            cmd += ["-x", "c++", "-I/opt/rocm/include"]
            # -x must precede the input: rebuild the command in the right order
            cmd = [hipcc, "-c", "-O2", "-fPIC", "-std=c++17", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                   "-x", "c++", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        objs.append(obj)
    cmd = [hipcc, "-shared", "-o", LIB] + objs + ["-L/opt/rocm/lib", "-lhiprtc", "-lamd_comgr", "-lamdhip64", "-ldl",
                                                  "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
