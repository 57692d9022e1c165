"""Builds libtbe.so (HIP, gfx950 only) next to this file with hipcc.  Run as a module:
    python -m paper_2104_05158_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtbe.so")
SOURCES = [os.path.join(CSRC, "tbe_api.hip"), os.path.join(CSRC, "tbe_inputs_api.hip")]
HEADERS = [os.path.join(CSRC, "tbe_kernels.hip.h"), os.path.join(CSRC, "tbe_inputs_kernels.hip.h"),
           os.path.join(ROOT, "include", "tbe.h"), os.path.join(ROOT, "include", "tbe_inputs.h")]

# packed fp32 ALU ops are switched off for all device code of this library
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-parameter"]


def build_library(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra_flags, "-DTBE_BUILDING=1", f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}",
           "-o", LIB, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
