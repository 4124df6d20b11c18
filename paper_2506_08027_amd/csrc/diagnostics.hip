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
template <int FMT>  // cbsz = blgp: 0 = E4M3 operands, 4 = E2M1 operands (the first four dwords of each fragment)
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
            acc[t & 15] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[t & 3], b[(t >> 2) & 3], acc[t & 15], FMT, FMT, 0,
                                                                           100, 0, 100);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 16; ++t)
        s += acc[t][0] + acc[t][1] + acc[t][2] + acc[t][3];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Second measurement aid: a plain copy, the simplest stream the memory system can be given, written the way
// the quantizer moves its data (128-bit streaming loads and stores, several in flight per work-item). The
// benchmark times it next to the quantizer on the same tensors: what it reaches is what HBM gives this chip's
// compute units for one read and one write stream, and the quantizer is reported against it as well as against
// the published bandwidth. `mode` picks how the 16-byte units are spread over the grid:
//   0  grid-stride, 4 units in flight per work-item;   1  grid-stride, 8 in flight;
//   2  each workgroup copies one contiguous slab, 4 in flight per work-item.
//   3 / 4  as 0, but the destination is written in runs of 128 / 256 bytes that lie far apart (consecutive
//          runs go to 64 interleaved regions), the way a transposed tile leaves a kernel: the same bytes end up
//          permuted in dst. For comparing write patterns; bytes must be a multiple of 64 runs.
template <int UNROLL, bool SLAB, int RUN_UNITS>
__global__ __launch_bounds__(256) void copy_rate_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t units)
{
    int64_t i, end, step;
    if constexpr (SLAB) {
        const int64_t per = (units + gridDim.x - 1) / gridDim.x;
        i = per * blockIdx.x + threadIdx.x;
        end = min(per * (blockIdx.x + 1), units);
        step = 256;
    } else {
        i = (int64_t)blockIdx.x * 256 + threadIdx.x;
        end = units;
        step = (int64_t)gridDim.x * 256;
    }
    auto where = [&](int64_t u) __attribute__((always_inline)) {
        if constexpr (RUN_UNITS == 0) {
            return u;
        } else {
            const int64_t run = u / RUN_UNITS, nruns = units / RUN_UNITS;  // nruns % 64 == 0 (checked by the caller)
            return ((run % 64) * (nruns / 64) + run / 64) * RUN_UNITS + u % RUN_UNITS;
        }
    };
    for (; i + (UNROLL - 1) * step < end; i += UNROLL * step) {
        uint4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            v[u] = stream_load(src + i + u * step);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            stream_store(dst + where(i + u * step), v[u]);
    }
    for (; i < end; i += step)
        stream_store(dst + where(i), stream_load(src + i));
}

hipError_t launch_copy_rate(const void *src, void *dst, int64_t bytes, int workgroups, int mode, hipStream_t stream)
{
    const uint4 *s = static_cast<const uint4 *>(src);
    uint4 *d = static_cast<uint4 *>(dst);
    const int64_t units = bytes / 16;
    const dim3 grid((unsigned)workgroups), block(256);
    if (mode == 0)
        hipLaunchKernelGGL((copy_rate_kernel<4, false, 0>), grid, block, 0, stream, s, d, units);
    else if (mode == 1)
        hipLaunchKernelGGL((copy_rate_kernel<8, false, 0>), grid, block, 0, stream, s, d, units);
    else if (mode == 2)
        hipLaunchKernelGGL((copy_rate_kernel<4, true, 0>), grid, block, 0, stream, s, d, units);
    else if (mode == 3)
        hipLaunchKernelGGL((copy_rate_kernel<4, false, 8>), grid, block, 0, stream, s, d, units);
    else
        hipLaunchKernelGGL((copy_rate_kernel<4, false, 16>), grid, block, 0, stream, s, d, units);
    return hipGetLastError();
}

// Third aid: hands the scaled matrix instruction registers straight from memory, one wavefront per experiment,
// so that a test can pin which operand register of which lane holds which (row, k) and which lane's scale
// byte applies to which k, for the element formats the product kernels use. Lane l of experiment x takes its
// eight A dwords from a[(64 x + l) * 8 ..], likewise B, its scale registers from sa / sb[64 x + l], starts
// from a zero accumulator and stores its four result registers to out[(64 x + l) * 4 ..].
template <int FMT>
__global__ __launch_bounds__(64) void mfma_layout_kernel(const v4i *__restrict__ a, const v4i *__restrict__ b,
                                                         const int *__restrict__ sa, const int *__restrict__ sb,
                                                         v4f *__restrict__ out)
{
    const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    const v4i a0 = a[2 * i], a1 = a[2 * i + 1], b0 = b[2 * i], b1 = b[2 * i + 1];
    const v8i av = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
    const v8i bv = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
    out[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, zero, FMT, FMT, 0, sa[i], 0, sb[i]);
}

hipError_t launch_mfma_layout(const void *a, const void *b, const int *sa, const int *sb, int experiments, bool fp4, float *out,
                              hipStream_t stream)
{
    const v4i *pa = static_cast<const v4i *>(a), *pb = static_cast<const v4i *>(b);
    if (fp4)
        hipLaunchKernelGGL(mfma_layout_kernel<4>, dim3((unsigned)experiments), dim3(64), 0, stream, pa, pb, sa, sb,
                           reinterpret_cast<v4f *>(out));
    else
        hipLaunchKernelGGL(mfma_layout_kernel<0>, dim3((unsigned)experiments), dim3(64), 0, stream, pa, pb, sa, sb,
                           reinterpret_cast<v4f *>(out));
    return hipGetLastError();
}

hipError_t launch_mfma_rate(int workgroups, int iterations, bool fp4, float *sink, hipStream_t stream)
{
    if (fp4)
        hipLaunchKernelGGL(mfma_rate_kernel<4>, dim3((unsigned)workgroups), dim3(256), 0, stream, iterations, sink);
    else
        hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3((unsigned)workgroups), dim3(256), 0, stream, iterations, sink);
    return hipGetLastError();
}

}  // namespace mxfp8
