"""Compile the HIP sources under csrc/ for gfx950 (hipcc cross-compiles without a GPU):
csrc/libwcc.so, the library, and csrc/libwcc_probe.so, the plain streaming kernels that bench.py
times beside it (a measurement aid, not part of the library)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(CSRC, "libwcc.so")
PROBE_LIB = os.path.join(CSRC, "libwcc_probe.so")
SOURCES = ["haar_fwd.hip", "haar_keep.hip", "haar_inv.hip", "select.hip", "gather.hip", "pointwise.hip",
           "depthwise.hip", "haar_chain.hip", "wcc_api.hip"]
PROBE_SOURCES = ["stream_probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, "_build", src.replace(".hip", ".o"))
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(verbose: bool = False) -> str:
    """Always recompiles every source; returns the path of the shared library."""
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES + PROBE_SOURCES))
    for lib, part in ((LIB, objs[:len(SOURCES)]), (PROBE_LIB, objs[len(SOURCES):])):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *part]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
