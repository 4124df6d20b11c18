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

// Launch shape, measured on an MI355X over sources that rotate through more than 1 GB: two resident workgroups per
// compute unit that stride over the items with four loads in flight each took 21.0 us for [8192 x 4096] -> BF16 and
// 112 us for [8192 x 14336] -> FP32, one short-lived work-item per item 22.5 and 120.7 us; more resident
// workgroups (4 .. 16 per unit) or a single one were slower, eight loads in flight changed nothing.
constexpr int kDeqUnroll = 4;
constexpr int kDeqGroupsPerCU = 2;

template <bool BF16, bool TILED, bool E5M2>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t *__restrict__ q,
                                                         const uint8_t *__restrict__ s, int64_t rows,
                                                         int64_t cols, uint8_t *__restrict__ dst,
                                                         int64_t ld_bytes)
{
    constexpr int EPT = BF16 ? 8 : 4;  // elements per item: 16 output bytes
    const int64_t per_row = cols / EPT;
    const int64_t total = rows * per_row;
    const int64_t nb = cols / kBlock;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    struct Item {
        uint2 q;  // FP32 output uses .x only
        uint32_t sb;
        int64_t out;  // byte offset of the item's 16 output bytes
    };
    auto fetch = [&](int64_t t) __attribute__((always_inline)) {
        Item it;
        const int64_t r = t / per_row;
        const int64_t c = (t - r * per_row) * EPT;
        if constexpr (TILED) {  // byte of (row r, block b): ((r/64 * ceil(nb/4) + b/4) * 64 + r%64) * 4 + b%4
            const int64_t b = c / kBlock;
            it.sb = s[(((r >> 6) * ((nb + 3) / 4) + (b >> 2)) * 64 + (r & 63)) * 4 + (b & 3)];
        } else {
            it.sb = s[r * nb + c / kBlock];
        }
        if constexpr (BF16) {
            const v2u v = __builtin_nontemporal_load(reinterpret_cast<const v2u *>(q + r * cols + c));
            it.q = make_uint2(v[0], v[1]);
        } else {
            it.q = make_uint2(__builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(q + r * cols + c)), 0u);
        }
        it.out = r * ld_bytes + c * (BF16 ? 2 : 4);
        return it;
    };
    auto emit = [&](const Item &it) __attribute__((always_inline)) {
        const int e = (int)it.sb - 127;
        const float nanv = __uint_as_float(0x7FC00000u);
        float v[EPT];
        decode4<E5M2>(it.q.x, e, v);
        if constexpr (BF16)
            decode4<E5M2>(it.q.y, e, v + 4);
        if (it.sb == 0xFF)
#pragma unroll
            for (int i = 0; i < EPT; ++i)
                v[i] = nanv;
        uint4 o;
        if constexpr (BF16)
            o = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
        else
            o = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
        stream_store(reinterpret_cast<uint4 *>(dst + it.out), o);
    };
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; t + (kDeqUnroll - 1) * step < total; t += kDeqUnroll * step) {
        Item it[kDeqUnroll];
#pragma unroll
        for (int u = 0; u < kDeqUnroll; ++u)
            it[u] = fetch(t + u * step);
#pragma unroll
        for (int u = 0; u < kDeqUnroll; ++u)
            emit(it[u]);
    }
    for (; t < total; t += step)
        emit(fetch(t));
}

template <bool TILED, bool E5M2>
static hipError_t launch_dequantize_t(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                                      bool bf16, int64_t ld, hipStream_t stream)
{
    const int64_t total = rows * (cols / (bf16 ? 8 : 4));
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess)
        return e;
    int64_t blocks = (total + 256 * kDeqUnroll - 1) / (256 * kDeqUnroll);
    if (cus > 0 && blocks > (int64_t)kDeqGroupsPerCU * cus)
        blocks = (int64_t)kDeqGroupsPerCU * cus;
    if (blocks < 1)
        blocks = 1;
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
