"""Build libanszp.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libanszp.so")
SOURCES = [os.path.join(CSRC, "anszp_host.cpp"), os.path.join(CSRC, "anszp_device.hip"),
           os.path.join(CSRC, "anszp_conv.hip"), os.path.join(CSRC, "anszp_encode.hip")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include")]


TEST_HELPER_SRC = os.path.join(ROOT, "tests", "gpu_helpers", "lds_fill.hip")
TEST_HELPER_LIB = os.path.join(ROOT, "tests", "gpu_helpers", "liblds_fill.so")


def build_test_helpers(verbose: bool = False) -> str:
    """The GPU tests' own helper kernels (tests/gpu_helpers), built in-tree like the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", TEST_HELPER_LIB, TEST_HELPER_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return TEST_HELPER_LIB


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_test_helpers(verbose=True))
