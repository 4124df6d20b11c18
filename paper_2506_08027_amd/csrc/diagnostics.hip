// Measurement aid: the rate at which this GPU sustains the scaled FP8 matrix instruction when nothing but
// the instruction runs (operands in registers, no memory traffic). The benchmark reports the GEMM against
// the chip's published peak and, beside it, against this measured rate, which includes whatever clock the
// power management settles on under a matrix-only load.
#include "mxfp8_device.h"

namespace mxfp8 {

// Every wavefront issues `iterations` x 64 independent MFMAs on register operands (16 accumulator tiles
// in rotation, so no instruction waits for its predecessor) and finally stores one float per work-item.
// The operands are four A and four B fragments of pseudo-random finite E4M3 codes (different in every
// lane, |value| < 2), used in rotation: the power drawn by the matrix pipes depends on how many operand
// bits change from one instruction to the next, and constant operands would flatter the result.
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iterations, float *__restrict__ sink)
{
    v8i a[4], b[4];
    uint32_t x = 0x9E3779B9u * (threadIdx.x + 1u) + 0x85EBCA6Bu * (blockIdx.x + 1u);
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x = x * 1664525u + 1013904223u;
            a[f][j] = (int)((x ^ (x >> 15)) & 0xBFBFBFBFu);   // exponent field below 8: no NaN code, |value| < 2
            x = x * 1664525u + 1013904223u;
            b[f][j] = (int)((x ^ (x >> 15)) & 0xBFBFBFBFu);
        }
    v4f acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t)
        acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int t = 0; t < 64; ++t)   // scale bytes 100: products around 2^-54, sums stay finite
            acc[t & 15] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[t & 3], b[(t >> 2) & 3], acc[t & 15], 0, 0, 0,
                                                                           100, 0, 100);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 16; ++t)
        s += acc[t][0] + acc[t][1] + acc[t][2] + acc[t][3];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

hipError_t launch_mfma_rate(int workgroups, int iterations, float *sink, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)workgroups), dim3(256), 0, stream, iterations, sink);
    return hipGetLastError();
}

}  // namespace mxfp8
