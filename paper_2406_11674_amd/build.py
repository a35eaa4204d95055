"""Builds libendor.so (the C-ABI library of include/endor.h) for gfx950 with hipcc.

The library is built in-tree, next to this file; tests, smoke() and bench.py
load what is there and never build by themselves."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libendor.so")
SOURCES = [os.path.join(HERE, "csrc", "endor_kernels.hip"),
           os.path.join(HERE, "csrc", "endor_gemm.hip"),
           os.path.join(HERE, "csrc", "endor_pipeline.hip"),
           os.path.join(HERE, "csrc", "endor_host.cpp")]
# the streaming yardstick kernels bench.py times beside the library (not part of the product path)
PROBE_LIB = os.path.join(HERE, "libendor_probe.so")
PROBE_SOURCES = [os.path.join(HERE, "csrc", "stream_probe.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
    # packed-fp32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def _compile(lib: str, sources, verbose: bool, extra_flags=()) -> str:
    tmp = lib + ".tmp%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", tmp, *sources]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, lib)
    return lib


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """libendor.so, and beside it libendor_probe.so (bench.py's streaming yardstick)."""
    _compile(PROBE_LIB, PROBE_SOURCES, verbose)
    return _compile(LIB, SOURCES, verbose, extra_flags)


if __name__ == "__main__":
    print(build_library(verbose=True, extra_flags=sys.argv[1:]))
