"""Builds libktanh.so (the C-ABI library with the gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libktanh.so")
SOURCES = ["ktanh_stream.hip", "ktanh_lstm.hip", "ktanh_backward.hip", "ktanh_lut.cpp", "ktanh_fit.cpp"]
# measurement yardsticks (include/ktanh_probe.h): a library of their own, loaded only by the benchmark
PROBE_LIB_PATH = os.path.join(_HERE, "libktanh_probe.so")
PROBE_SOURCES = ["ktanh_probe.hip", "ktanh_lut.cpp", "ktanh_fit.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-std=c++17", "-O3", "-fPIC", "-shared",
    "-ffp-contract=off",                       # every fused multiply-add in the kernels is explicit
    "-fno-gpu-flush-denormals-to-zero",        # Float32 subnormals are kept
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the leading scalar arguments of every kernel arrive preloaded in scalar registers, so a
    # wavefront can issue its first load without a round trip to the argument buffer
    "-mllvm", "-amdgpu-kernarg-preload-count=12",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def _compile(sources, target, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in sources], "-o", target]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return target


def build_library(verbose: bool = False) -> str:
    """Compile every source of the library for gfx950; returns the path of the .so."""
    return _compile(SOURCES, LIB_PATH, verbose)


def build_probe_library(verbose: bool = False) -> str:
    """Compile the measurement yardsticks (libktanh_probe.so) for gfx950."""
    return _compile(PROBE_SOURCES, PROBE_LIB_PATH, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe_library(verbose=True))
