#!/bin/bash
# Builds the CPU execution model of the library: the kernel sources, unchanged, as host C++.
#   tests/host_model/build.sh [output]            the test driver, with AddressSanitizer and alignment checks
#   tests/host_model/build.sh --shared [output]   the C ABI as a shared library (optimised, no sanitizer),
#                                                 loadable in place of libmxfp8.so
set -e
here="$(cd "$(dirname "$0")" && pwd)"
csrc="$here/../../paper_2506_08027_amd/csrc"
CXX="${HOST_CLANG:-/opt/rocm/llvm/bin/clang++}"
common=(-std=c++17 -x c++ -I "$here/shim" -Wall -Wno-unknown-pragmas -Wno-unused-function -Wno-psabi)
kernels=("$csrc/api.hip" "$csrc/quantize.hip" "$csrc/dequantize.hip" "$csrc/gemm.hip" "$csrc/diagnostics.hip" "$csrc/mxfp4.hip" "$csrc/mxfp6.hip")
if [ "$1" = "--shared" ]; then
    out="${2:-$here/_build/libmxfp8_hostmodel.so}"
    mkdir -p "$(dirname "$out")"
    "$CXX" "${common[@]}" -O2 -fPIC -shared -o "$out" "${kernels[@]}"
else
    out="${1:-$here/_build/hostmodel}"
    mkdir -p "$(dirname "$out")"
    "$CXX" "${common[@]}" -O0 -gline-tables-only -fsanitize=address,alignment -fno-sanitize-recover=all -fno-omit-frame-pointer \
        -o "$out" "$here/driver.cpp" "${kernels[@]}"
fi
