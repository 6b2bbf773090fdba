"""Builds libgnnagg.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libgnnagg.so")
OBJ_DIR = os.path.join(PKG, "_build")

SOURCES = ["aggregate.hip", "blocked.hip", "ap.hip", "gemm.hip", "layer.hip", "plan.hip", "graph.hip", "util.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-I", INCLUDE, "-I", CSRC,
    # packed-fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build_library(verbose: bool = True) -> str:
    """Compile every .hip source and link libgnnagg.so (always recompiles)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(_compile, SOURCES))
    tmp = LIB + ".tmp"
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}", file=sys.stderr)
    build_profiling_driver(verbose)
    return LIB


def build_profiling_driver(verbose: bool = True) -> bool:
    """The stand-alone driver for rocprofv3 counter runs (links against the library).  A tool beside
    the product: its failure is reported, not raised."""
    try:
        subprocess.check_call([_hipcc(), "-O2", "-std=c++17", "-I", INCLUDE, os.path.join(CSRC, "agg_profile.cpp"),
                               "-o", os.path.join(PKG, "agg_profile"), "-L", PKG, "-lgnnagg", "-Wl,-rpath,$ORIGIN"])
        return True
    except (subprocess.CalledProcessError, OSError) as err:
        if verbose:
            print(f"warning: the profiling driver agg_profile was not built ({err})", file=sys.stderr)
        return False


if __name__ == "__main__":
    build_library()
