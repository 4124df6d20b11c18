// MXFP4 for gfx950: FP32/BF16 -> E2M1 elements (two per byte) + UE8M0 block scales, and back. Table 1 lists
// MXFP4 as the narrower member of the MX family; the conversion is the paper's (Section 3.3, Algorithm 1,
// Appendix A.1 and A.2) with the E2M1 constants: the scale is the smallest 2^n with amax <= 6 * 2^n, elements
// are RNE(V_i / X) to one of 0, 0.5, 1, 1.5, 2, 3, 4, 6, ties to the even code, saturating. E2M1 has no NaN
// and no Inf code: a NaN lives in the scale byte (0xFF) only.
//
// A workgroup stages its 128 x 128 tile in LDS as FP32 (row pitch 132 words: rows stay 16-byte aligned for 128-bit
// reads along a row, and walking down a column, neighbouring work-items on neighbouring columns, is conflict-free)
// and every work-item then converts whole 32-element blocks: along rows for the row copy, down columns for the
// transposed column copy, 16 packed bytes per block in one 128-bit store. Elements go through the hardware
// converter (v_cvt_scalef32_pk_fp4_f32: divides by the scale, rounds to nearest even, saturates, keeps the sign);
// blocks with an infinity take a software encoder, blocks with a NaN are not converted at all.
#include "mxfp8_device.h"

namespace mxfp8 {

constexpr int kFp4Tile = 128;
constexpr int kFp4Pitch = kFp4Tile + 4;
constexpr int kFp4Threads = 256;
constexpr int kFp4LdsBytes = kFp4Tile * kFp4Pitch * 4;

// n + 127 for the smallest n with amax <= 6 * 2^n = 1.5 * 2^(n + 2), from the magnitude bits of an FP32 amax:
// amax = (1 + f) * 2^e needs n = e - 2 when f <= 0.5 and e - 1 otherwise, i.e. the exponent field after adding
// 0x3FFFFF to the bits, less 2; clamped below at 0 (every subnormal and zero); Inf -> 254, NaN -> 0xFF.
__device__ __forceinline__ uint32_t fp4_scale_byte(uint32_t abs_bits)
{
    if (abs_bits > 0x7F800000u)
        return 0xFFu;
    if (abs_bits == 0x7F800000u)
        return 254u;
    const int b = (int)((abs_bits + 0x3FFFFFu) >> 23) - 2;
    return (uint32_t)max(b, 0);
}

// E2M1 code of v / 2^n: the seven thresholds are the midpoints of neighbouring magnitudes; a midpoint goes to
// the neighbour with the even code (0, 1, 2, 4 are even codes 0, 2, 4, 6), hence the mix of > and >=.
__device__ __forceinline__ uint32_t fp4_code(float v, int n)
{
    const float t = fabsf(ldexpf(v, -n));  // exact: a power-of-two scaling (Inf stays Inf and saturates)
    const uint32_t mag = (uint32_t)(t > 0.25f) + (uint32_t)(t >= 0.75f) + (uint32_t)(t > 1.25f) + (uint32_t)(t >= 1.75f) +
                         (uint32_t)(t > 2.5f) + (uint32_t)(t >= 3.5f) + (uint32_t)(t > 5.0f);
    return mag | ((__float_as_uint(v) >> 28) & 8u);
}

// 32 values -> 16 packed bytes and the block's scale byte (element 2k in the low nibble of byte k)
__device__ __forceinline__ uint4 fp4_block(const float (&v)[kBlock], uint32_t &scale)
{
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < kBlock; ++i)
        amax = umax(amax, __float_as_uint(v[i]) & 0x7FFFFFFFu);
    const uint32_t sb = fp4_scale_byte(amax);
    scale = sb;
    uint32_t w[4] = {0, 0, 0, 0};
    if (amax < 0x7F800000u) {
        const float x = scale_operand(sb);
#pragma unroll
        for (int i = 0; i < kBlock; i += 8) {
            uint32_t q = 0;
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, v[i], v[i + 1], x, 0);
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, v[i + 2], v[i + 3], x, 1);
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, v[i + 4], v[i + 5], x, 2);
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, v[i + 6], v[i + 7], x, 3);
            w[i / 8] = q;
        }
    } else if (sb != 0xFFu) {  // a block with an infinity: +-Inf -> +-6, finite values / 2^127
#pragma unroll
        for (int i = 0; i < kBlock; ++i)
            w[i / 8] |= fp4_code(v[i], 127) << (4 * (i % 8));
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// position of scale byte (r, b) of an operand with nb blocks per row
template <bool TILED> __device__ __forceinline__ int64_t fp4_scale_index(int64_t r, int64_t b, int64_t nb)
{
    return TILED ? (((r >> 6) * ((nb + 3) / 4) + (b >> 2)) * 64 + (r & 63)) * 4 + (b & 3) : r * nb + b;
}

// The grid is resident (a few workgroups per compute unit) and every workgroup walks over tiles blockIdx.x,
// blockIdx.x + gridDim.x, ...: the 128-bit loads of its next tile are issued into registers before the current
// tile is converted, so that the memory system always has reads in flight while blocks are being encoded.
template <bool BF16, bool ROW, bool COL, bool TILED>
__global__ __launch_bounds__(kFp4Threads) void quantize_fp4_kernel(const uint8_t *__restrict__ src, int64_t rows, int64_t cols,
                                                                   int64_t ld_bytes, uint8_t *__restrict__ q_row,
                                                                   uint8_t *__restrict__ s_row, uint8_t *__restrict__ q_colT,
                                                                   uint8_t *__restrict__ s_colT, uint32_t tiles_x, uint32_t ntiles)
{
    MXFP8_DYNAMIC_LDS(lds_raw);
    float *tile = reinterpret_cast<float *>(lds_raw);
    const int tid = threadIdx.x;
    constexpr int VEC = BF16 ? 8 : 4;                          // elements per 128-bit load
    constexpr int PER_ROW = kFp4Tile / VEC;                    // loads per tile row
    constexpr int LOADS = kFp4Tile * PER_ROW / kFp4Threads;    // loads per work-item and tile
    constexpr int BLOCKS = kFp4Tile / kBlock;                  // 4 blocks per tile row / column
    uint4 regs[LOADS];
    // rows % 32 == 0 and cols % 32 == 0: a 16-byte piece is wholly inside or outside; outside reads as zeros
    auto fetch = [&](uint32_t t) __attribute__((always_inline)) {
        const uint32_t ty = t / tiles_x, tx = t - ty * tiles_x;
        const int64_t row0 = (int64_t)ty * kFp4Tile, col0 = (int64_t)tx * kFp4Tile;
#pragma unroll
        for (int k = 0; k < LOADS; ++k) {
            const int idx = tid + k * kFp4Threads, r = idx / PER_ROW, c = (idx % PER_ROW) * VEC;
            regs[k] = make_uint4(0, 0, 0, 0);
            if (row0 + r < rows && col0 + c < cols)
                regs[k] = stream_load(reinterpret_cast<const uint4 *>(src + (row0 + r) * ld_bytes + (col0 + c) * (BF16 ? 2 : 4)));
        }
    };
    if (blockIdx.x < ntiles)
        fetch(blockIdx.x);
    for (uint32_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const uint32_t tile_y = t / tiles_x, tile_x = t - tile_y * tiles_x;
        const int64_t row0 = (int64_t)tile_y * kFp4Tile, col0 = (int64_t)tile_x * kFp4Tile;
        // ---- registers -> LDS, widened to FP32
#pragma unroll
        for (int k = 0; k < LOADS; ++k) {
            const int idx = tid + k * kFp4Threads, r = idx / PER_ROW, c = (idx % PER_ROW) * VEC;
            const uint4 v = regs[k];
            float *d = tile + r * kFp4Pitch + c;
            if constexpr (BF16) {
                *reinterpret_cast<float4 *>(d) = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u),
                                                             __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xFFFF0000u));
                *reinterpret_cast<float4 *>(d + 4) = make_float4(__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xFFFF0000u),
                                                                 __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xFFFF0000u));
            } else {
                *reinterpret_cast<float4 *>(d) = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
            }
        }
        __syncthreads();
        if (t + gridDim.x < ntiles)
            fetch(t + gridDim.x);  // in flight while this tile is converted
        if constexpr (ROW) {
            const int64_t nb = cols / kBlock;
            for (int item = tid; item < kFp4Tile * BLOCKS; item += kFp4Threads) {
                const int r = item / BLOCKS, b = item % BLOCKS;
                if (row0 + r < rows && col0 + b * kBlock < cols) {
                    uint32_t sb;
                    float v[kBlock];
#pragma unroll
                    for (int i = 0; i < kBlock; i += 4) {
                        const float4 f = *reinterpret_cast<const float4 *>(tile + r * kFp4Pitch + b * kBlock + i);
                        v[i] = f.x; v[i + 1] = f.y; v[i + 2] = f.z; v[i + 3] = f.w;
                    }
                    const uint4 q = fp4_block(v, sb);
                    *reinterpret_cast<uint4 *>(q_row + (row0 + r) * (cols / 2) + (col0 + b * kBlock) / 2) = q;
                    s_row[fp4_scale_index<TILED>(row0 + r, col0 / kBlock + b, nb)] = (uint8_t)sb;
                }
            }
        }
        if constexpr (COL) {
            const int64_t nbT = rows / kBlock;
            for (int item = tid; item < kFp4Tile * BLOCKS; item += kFp4Threads) {
                const int c = item % kFp4Tile, b = item / kFp4Tile;  // neighbouring work-items walk down neighbouring columns
                if (col0 + c < cols && row0 + b * kBlock < rows) {
                    uint32_t sb;
                    float v[kBlock];
#pragma unroll
                    for (int i = 0; i < kBlock; ++i)
                        v[i] = tile[(b * kBlock + i) * kFp4Pitch + c];
                    const uint4 q = fp4_block(v, sb);
                    *reinterpret_cast<uint4 *>(q_colT + (col0 + c) * (rows / 2) + (row0 + b * kBlock) / 2) = q;
                    s_colT[fp4_scale_index<TILED>(col0 + c, row0 / kBlock + b, nbT)] = (uint8_t)sb;
                }
            }
        }
        __syncthreads();  // the tile in LDS is overwritten by the next round
    }
}

template <bool BF16, bool TILED>
static hipError_t launch_quantize_fp4_t(const void *src, int64_t rows, int64_t cols, int64_t ld, int axis, uint8_t *q_row,
                                        uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, hipStream_t stream)
{
    const int64_t tiles_x = (cols + kFp4Tile - 1) / kFp4Tile, tiles_y = (rows + kFp4Tile - 1) / kFp4Tile;
    if (tiles_x * tiles_y > 0x7FFFFFFF)
        return hipErrorInvalidConfiguration;
    int dev = 0, cus = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err == hipSuccess)
        err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (err != hipSuccess)
        return err;
    const int64_t ntiles = tiles_x * tiles_y, resident = 2 * (int64_t)(cus > 0 ? cus : 1);  // two tiles of LDS fit a compute unit
    const dim3 grid((unsigned)(ntiles < resident ? ntiles : resident)), block(kFp4Threads);
    const uint8_t *s = static_cast<const uint8_t *>(src);
    const int64_t ldb = ld * (BF16 ? 2 : 4);
#define MXFP4_LAUNCH(R, C)                                                                                              \
    {                                                                                                                   \
        auto kern = quantize_fp4_kernel<BF16, R, C, TILED>;                                                             \
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                                  \
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kFp4LdsBytes);             \
        if (e != hipSuccess)                                                                                            \
            return e;                                                                                                   \
        hipLaunchKernelGGL(kern, grid, block, kFp4LdsBytes, stream, s, rows, cols, ldb, q_row, s_row, q_colT, s_colT,    \
                           (uint32_t)tiles_x, (uint32_t)ntiles);                                                                        \
    }
    if (axis == 1)
        MXFP4_LAUNCH(true, false)
    else if (axis == 2)
        MXFP4_LAUNCH(false, true)
    else
        MXFP4_LAUNCH(true, true)
#undef MXFP4_LAUNCH
    return hipGetLastError();
}

hipError_t launch_quantize_fp4(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis, uint8_t *q_row,
                               uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, bool tiled_scales, hipStream_t stream)
{
    if (bf16)
        return tiled_scales ? launch_quantize_fp4_t<true, true>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream)
                            : launch_quantize_fp4_t<true, false>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream);
    return tiled_scales ? launch_quantize_fp4_t<false, true>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream)
                        : launch_quantize_fp4_t<false, false>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream);
}

// ---- decode: value = E2M1(code) * 2^(s - 127) -----------------------------------------------------------------
__device__ __forceinline__ float fp4_value(uint32_t code)
{
    const uint32_t e = (code >> 1) & 3u, m = code & 1u;
    const float mag = e == 0 ? 0.5f * (float)m : ldexpf(1.0f + 0.5f * (float)m, (int)e - 1);
    return (code & 8u) ? -mag : mag;
}

// one work-item per dword of codes (8 elements): neighbouring work-items load neighbouring dwords and store
// neighbouring 16-byte (BF16) or 32-byte (FP32) pieces
template <bool BF16, bool TILED>
__global__ __launch_bounds__(256) void dequantize_fp4_kernel(const uint8_t *__restrict__ q, const uint8_t *__restrict__ s,
                                                             int64_t rows, int64_t cols, uint8_t *__restrict__ dst, int64_t ld_bytes)
{
    // the 16 values of the format in 16 LDS banks: a lookup per element, no bank conflicts between different codes
    __shared__ float value_of[16];
    if (threadIdx.x < 16)
        value_of[threadIdx.x] = fp4_value(threadIdx.x);
    __syncthreads();
    const int64_t per_row = cols / 8, nb = cols / kBlock, total = rows * per_row;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = t / per_row, j = t - r * per_row;
        const uint32_t sb = s[fp4_scale_index<TILED>(r, j / 4, nb)];
        const uint32_t w = *reinterpret_cast<const uint32_t *>(q + r * (cols / 2) + j * 4);
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            v[i] = sb == 0xFFu ? __uint_as_float(0x7FC00000u) : ldexpf(value_of[(w >> (4 * i)) & 0xFu], (int)sb - 127);
        uint8_t *out = dst + r * ld_bytes + j * 8 * (BF16 ? 2 : 4);
        if constexpr (BF16) {
            uint32_t p[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v2bf h = {(__bf16)v[2 * e], (__bf16)v[2 * e + 1]};
                p[e] = __builtin_bit_cast(uint32_t, h);
            }
            stream_store(reinterpret_cast<uint4 *>(out), make_uint4(p[0], p[1], p[2], p[3]));
        } else {
            stream_store(reinterpret_cast<uint4 *>(out), make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
            stream_store(reinterpret_cast<uint4 *>(out + 16), make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])));
        }
    }
}

hipError_t launch_dequantize_fp4(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst, bool bf16,
                                 bool tiled_scales, int64_t ld, hipStream_t stream)
{
    const int64_t total = rows * (cols / 8);
    const int64_t want = (total + 255) / 256;
    const dim3 grid((unsigned)(want < 16384 ? want : 16384)), block(256);
    uint8_t *d = static_cast<uint8_t *>(dst);
    const int64_t ldb = ld * (bf16 ? 2 : 4);
    if (bf16) {
        if (tiled_scales)
            hipLaunchKernelGGL((dequantize_fp4_kernel<true, true>), grid, block, 0, stream, q, s, rows, cols, d, ldb);
        else
            hipLaunchKernelGGL((dequantize_fp4_kernel<true, false>), grid, block, 0, stream, q, s, rows, cols, d, ldb);
    } else {
        if (tiled_scales)
            hipLaunchKernelGGL((dequantize_fp4_kernel<false, true>), grid, block, 0, stream, q, s, rows, cols, d, ldb);
        else
            hipLaunchKernelGGL((dequantize_fp4_kernel<false, false>), grid, block, 0, stream, q, s, rows, cols, d, ldb);
    }
    return hipGetLastError();
}

}  // namespace mxfp8
