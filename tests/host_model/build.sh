#!/bin/bash
# Builds the CPU execution model of the library: the kernel sources, unchanged, as host C++ with
# AddressSanitizer and alignment checks. Usage: tests/host_model/build.sh [output path]
set -e
here="$(cd "$(dirname "$0")" && pwd)"
out="${1:-$here/_build/hostmodel}"
csrc="$here/../../paper_2506_08027_amd/csrc"
mkdir -p "$(dirname "$out")"
CXX="${HOST_CLANG:-/opt/rocm/llvm/bin/clang++}"
"$CXX" -std=c++17 -O1 -g -fsanitize=address,alignment -fno-sanitize-recover=all -fno-omit-frame-pointer \
    -x c++ -I "$here/shim" -Wall -Wno-unknown-pragmas -Wno-unused-function -Wno-psabi \
    -o "$out" "$here/driver.cpp" "$csrc/api.hip" "$csrc/quantize.hip" "$csrc/dequantize.hip" "$csrc/gemm.hip"
