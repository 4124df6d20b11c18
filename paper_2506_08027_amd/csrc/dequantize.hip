// MXFP8 decode for gfx950: value = E4M3(q) * 2^(s - 127) (Section 2), FP32 or BF16 output.
//
// Pure streaming: every thread produces 16 output bytes (4 FP32 or 8 BF16 values) from 4 or 8
// element bytes and the scale byte of their block. The E4M3 code is widened with the hardware
// converter and scaled with an exact ldexp, so the FP32 result is exact (or +-Inf when
// 448 * 2^127-class products overflow); BF16 output is one round-to-nearest-even of that value.
#include "mxfp8_device.h"

namespace mxfp8 {

typedef float v2f __attribute__((ext_vector_type(2)));

template <bool E5M2> __device__ __forceinline__ void decode4(uint32_t q, int e, float out[4])
{
    const v2f lo = E5M2 ? __builtin_amdgcn_cvt_pk_f32_bf8((int)q, false) : __builtin_amdgcn_cvt_pk_f32_fp8((int)q, false);
    const v2f hi = E5M2 ? __builtin_amdgcn_cvt_pk_f32_bf8((int)q, true) : __builtin_amdgcn_cvt_pk_f32_fp8((int)q, true);
    out[0] = ldexpf(lo[0], e);
    out[1] = ldexpf(lo[1], e);
    out[2] = ldexpf(hi[0], e);
    out[3] = ldexpf(hi[1], e);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    v2bf r = {(__bf16)a, (__bf16)b};  // v_cvt_pk_bf16_f32: round to nearest even
    return __builtin_bit_cast(uint32_t, r);
}

template <bool BF16, bool TILED, bool E5M2>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t *__restrict__ q,
                                                         const uint8_t *__restrict__ s, int64_t rows,
                                                         int64_t cols, uint8_t *__restrict__ dst,
                                                         int64_t ld_bytes)
{
    constexpr int EPT = BF16 ? 8 : 4;  // elements per thread
    const int64_t per_row = cols / EPT;
    const int64_t total = rows * per_row;
    const int64_t nb = cols / kBlock;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = t / per_row;
        const int64_t c = (t - r * per_row) * EPT;
        uint32_t sb;
        if constexpr (TILED) {  // byte of (row r, block b): ((r/64 * ceil(nb/4) + b/4) * 64 + r%64) * 4 + b%4
            const int64_t b = c / kBlock;
            sb = s[(((r >> 6) * ((nb + 3) / 4) + (b >> 2)) * 64 + (r & 63)) * 4 + (b & 3)];
        } else {
            sb = s[r * nb + c / kBlock];
        }
        const int e = (int)sb - 127;
        const float nanv = __uint_as_float(0x7FC00000u);
        if constexpr (BF16) {
            const uint2 qq = *reinterpret_cast<const uint2 *>(q + r * cols + c);
            float v[8];
            decode4<E5M2>(qq.x, e, v);
            decode4<E5M2>(qq.y, e, v + 4);
            if (sb == 0xFF)
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    v[i] = nanv;
            uint4 o = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]),
                                 pack_bf16(v[6], v[7]));
            *reinterpret_cast<uint4 *>(dst + r * ld_bytes + c * 2) = o;
        } else {
            const uint32_t qq = *reinterpret_cast<const uint32_t *>(q + r * cols + c);
            float v[4];
            decode4<E5M2>(qq, e, v);
            if (sb == 0xFF)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    v[i] = nanv;
            *reinterpret_cast<float4 *>(dst + r * ld_bytes + c * 4) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

template <bool TILED, bool E5M2>
static hipError_t launch_dequantize_t(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                                      bool bf16, int64_t ld, hipStream_t stream)
{
    const int64_t total = rows * (cols / (bf16 ? 8 : 4));
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64)
        blocks = 256 * 64;  // grid-stride beyond 64 workgroups per compute unit
    if (bf16)
        hipLaunchKernelGGL((dequantize_kernel<true, TILED, E5M2>), dim3((unsigned)blocks), dim3(256), 0, stream, q, s,
                           rows, cols, static_cast<uint8_t *>(dst), ld * 2);
    else
        hipLaunchKernelGGL((dequantize_kernel<false, TILED, E5M2>), dim3((unsigned)blocks), dim3(256), 0, stream, q, s,
                           rows, cols, static_cast<uint8_t *>(dst), ld * 4);
    return hipGetLastError();
}

hipError_t launch_dequantize(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                             bool bf16, bool tiled_scales, bool e5m2, int64_t ld, hipStream_t stream)
{
    if (e5m2)
        return tiled_scales ? launch_dequantize_t<true, true>(q, s, rows, cols, dst, bf16, ld, stream)
                            : launch_dequantize_t<false, true>(q, s, rows, cols, dst, bf16, ld, stream);
    return tiled_scales ? launch_dequantize_t<true, false>(q, s, rows, cols, dst, bf16, ld, stream)
                        : launch_dequantize_t<false, false>(q, s, rows, cols, dst, bf16, ld, stream);
}

}  // namespace mxfp8
