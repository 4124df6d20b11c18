"""Compile the HIP kernels and the C ABI into ``libmxfp8.so`` next to this file (gfx950 only)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libmxfp8.so")
SOURCES = ["api.hip", "quantize.hip", "dequantize.hip", "gemm.hip", "diagnostics.hip", "mxfp4.hip", "mxfp6.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed-FP32 code generation is switched off on purpose (the compiler would otherwise form
# v_pk_*_f32 from ordinary float code).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = False) -> str:
    """Always recompiles; returns the path of the shared library."""
    cmd = [HIPCC] + FLAGS + ["-o", LIB_PATH] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless, filtered
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB_PATH


EXAMPLE_SRC = os.path.join(_HERE, "examples", "linear_layer_step.cpp")
EXAMPLE_BIN = os.path.join(_HERE, "examples", "linear_layer_step")


def build_example() -> str:
    """The stand-alone C++ program that drives one linear-layer step through the C ABI (needs the library built)."""
    cmd = [HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", EXAMPLE_SRC, "-I", os.path.join(os.path.dirname(_HERE), "include"),
           "-L", _HERE, "-lmxfp8", "-Wl,-rpath,$ORIGIN/..", "-o", EXAMPLE_BIN]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stderr)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_example())
