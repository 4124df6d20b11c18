// MXFP6 for gfx950: FP32/BF16 -> E2M3 or E3M2 elements (32 six-bit codes packed into 24 bytes) + UE8M0 block
// scales, back to FP32/BF16, and the exact expansion of the codes to E4M3 bytes that lets the MXFP8 product
// kernels multiply MXFP6 operands. Table 1 lists MXFP6 between MXFP8 and MXFP4; the conversion is the paper's
// (Section 3.3, Algorithm 1, Appendix A.1 and A.2) with the 6-bit constants: the scale is the smallest 2^n with
// amax <= destmax * 2^n (destmax 7.5 for E2M3, 28 for E3M2), elements are RNE(V_i / X), ties to the even code,
// saturating. Neither format has a NaN or an Inf code: a NaN lives in the scale byte (0xFF) only.
//
// Why the product goes through E4M3: a block of 32 six-bit codes is 24 bytes, which does not tile into the
// 16-byte pieces that the product kernels move through LDS, while every E2M3 and every E3M2 value is also an
// E4M3 value (at most 3 mantissa bits, magnitudes between 2^-4 and 28). Expanding the codes (0.75 -> 1 byte per
// element, scales untouched) gives an MXFP8 operand whose product IS the MXFP6 product; what is given up is the
// higher rate of the 6-bit matrix instruction, what is kept is the smaller footprint of the stored tensor.
#include "mxfp8_device.h"

namespace mxfp8 {

template <int E_, int M_> struct Fp6 {
    static constexpr int E = E_, M = M_;
    static constexpr int BIAS = (1 << (E - 1)) - 1;
    static constexpr int EMAX = (1 << E) - 1 - BIAS;  // exponent of the top binade (2 / 4)
    static constexpr int EMIN = 1 - BIAS;             // exponent of the smallest normal (0 / -2)
    static constexpr uint32_t TOP_FRAC = ((1u << M) - 1u) << (23 - M);  // FP32 fraction bits of destmax's significand
    static constexpr int QMAX = (1 << (M + 1)) - 1;   // largest significand in units of the top binade's step
};
using E2M3 = Fp6<2, 3>;
using E3M2 = Fp6<3, 2>;

constexpr int kFp6Tile = 128;
constexpr int kFp6Pitch = kFp6Tile + 4;  // words: rows stay 16-byte aligned, column walks are conflict-free
constexpr int kFp6Threads = 256;
constexpr int kFp6LdsBytes = kFp6Tile * kFp6Pitch * 4;
constexpr int kFp6BlockBytes = 24;

// n + 127 for the smallest n with amax <= destmax * 2^n: amax = (1 + f) * 2^e needs n = e - EMAX when f does not
// exceed destmax's fraction and one more otherwise, i.e. the exponent field after adding (all-ones fraction -
// destmax's fraction) to the bits, less EMAX; clamped below at 0; Inf -> 254, NaN -> 0xFF.
template <class F> __device__ __forceinline__ uint32_t fp6_scale_byte(uint32_t abs_bits)
{
    if (abs_bits > 0x7F800000u)
        return 0xFFu;
    if (abs_bits == 0x7F800000u)
        return 254u;
    const int b = (int)((abs_bits + (0x7FFFFFu - F::TOP_FRAC)) >> 23) - F::EMAX;
    return (uint32_t)max(b, 0);
}

// code of v / 2^n: the binade of the quotient (held inside the format's range) fixes the step, the quotient is
// rounded to a whole number of steps (rintf: nearest, ties to even = ties to the even code) and clamped at the top;
// exponent field and mantissa then add up to ((e - EMIN) << M) + steps in every case: subnormal, normal, and a
// rounding that carries into the next binade.
template <class F> __device__ __forceinline__ uint32_t fp6_code(float v, int n)
{
    const float t = fabsf(ldexpf(v, -n));  // exact: a power-of-two scaling (Inf stays Inf and saturates)
    const int e = min(max((int)((__float_as_uint(t) >> 23) & 0xFFu) - 127, F::EMIN), F::EMAX);
    float q = rintf(ldexpf(t, F::M - e));
    if (e == F::EMAX)
        q = fminf(q, (float)F::QMAX);
    return (uint32_t)(((e - F::EMIN) << F::M) + (int)q) | ((__float_as_uint(v) >> 26) & 32u);
}

// 32 values -> six dwords (one little-endian 192-bit string, code i in bits 6i..6i+5) and the block's scale byte.
// Finite blocks go through the hardware converter (v_cvt_scalef32_2xpk16_{fp6,bf6}_f32: 2 x 16 values divided by
// the scale, rounded to nearest even, saturated, packed; element 2i of the result comes from the first source,
// 2i+1 from the second); blocks with an infinity take the software encoder, blocks with a NaN are not converted.
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v6u __attribute__((ext_vector_type(6)));
template <class F> __device__ __forceinline__ void fp6_block(const float (&v)[kBlock], uint32_t (&w)[6], uint32_t &scale)
{
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < kBlock; ++i)
        amax = umax(amax, __float_as_uint(v[i]) & 0x7FFFFFFFu);
    const uint32_t sb = fp6_scale_byte<F>(amax);
    scale = sb;
#pragma unroll
    for (int j = 0; j < 6; ++j)
        w[j] = 0;
    if (amax < 0x7F800000u) {
        v16f even, odd;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            even[i] = v[2 * i];
            odd[i] = v[2 * i + 1];
        }
        v6u r;
        if constexpr (F::E == 2)
            r = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(even, odd, scale_operand(sb));
        else
            r = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(even, odd, scale_operand(sb));
#pragma unroll
        for (int j = 0; j < 6; ++j)
            w[j] = r[j];
    } else if (sb != 0xFFu) {  // a block with an infinity: +-Inf -> +-destmax, finite values / 2^127
#pragma unroll
        for (int i = 0; i < kBlock; ++i) {
            const uint32_t c = fp6_code<F>(v[i], 127);
            const int pos = 6 * i;  // compile-time after unrolling
            w[pos / 32] |= c << (pos % 32);
            if (pos % 32 > 26)
                w[pos / 32 + 1] |= c >> (32 - pos % 32);
        }
    }
}

template <bool TILED> __device__ __forceinline__ int64_t fp6_scale_index(int64_t r, int64_t b, int64_t nb)
{
    return TILED ? (((r >> 6) * ((nb + 3) / 4) + (b >> 2)) * 64 + (r & 63)) * 4 + (b & 3) : r * nb + b;
}

__device__ __forceinline__ void fp6_store_block(uint8_t *p, const uint32_t (&w)[6])
{
    uint2 *d = reinterpret_cast<uint2 *>(p);  // 24-byte blocks start on 8-byte boundaries
    d[0] = make_uint2(w[0], w[1]);
    d[1] = make_uint2(w[2], w[3]);
    d[2] = make_uint2(w[4], w[5]);
}

// Resident grid over 128 x 128 tiles, the next tile's loads in registers while a tile is converted (the scheme of
// the MXFP4 quantizer); a block leaves as 24 bytes.
template <class F, bool BF16, bool ROW, bool COL, bool TILED>
__global__ __launch_bounds__(kFp6Threads) void quantize_fp6_kernel(const uint8_t *__restrict__ src, int64_t rows, int64_t cols,
                                                                   int64_t ld_bytes, uint8_t *__restrict__ q_row,
                                                                   uint8_t *__restrict__ s_row, uint8_t *__restrict__ q_colT,
                                                                   uint8_t *__restrict__ s_colT, uint32_t tiles_x, uint32_t ntiles)
{
    MXFP8_DYNAMIC_LDS(lds_raw);
    float *tile = reinterpret_cast<float *>(lds_raw);
    const int tid = threadIdx.x;
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int PER_ROW = kFp6Tile / VEC;
    constexpr int LOADS = kFp6Tile * PER_ROW / kFp6Threads;
    constexpr int BLOCKS = kFp6Tile / kBlock;
    uint4 regs[LOADS];
    // rows % 32 == 0 and cols % 32 == 0: a 16-byte piece is wholly inside or outside; outside reads as zeros
    auto fetch = [&](uint32_t t) __attribute__((always_inline)) {
        const uint32_t ty = t / tiles_x, tx = t - ty * tiles_x;
        const int64_t row0 = (int64_t)ty * kFp6Tile, col0 = (int64_t)tx * kFp6Tile;
#pragma unroll
        for (int k = 0; k < LOADS; ++k) {
            const int idx = tid + k * kFp6Threads, r = idx / PER_ROW, c = (idx % PER_ROW) * VEC;
            regs[k] = make_uint4(0, 0, 0, 0);
            if (row0 + r < rows && col0 + c < cols)
                regs[k] = stream_load(reinterpret_cast<const uint4 *>(src + (row0 + r) * ld_bytes + (col0 + c) * (BF16 ? 2 : 4)));
        }
    };
    if (blockIdx.x < ntiles)
        fetch(blockIdx.x);
    for (uint32_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const uint32_t tile_y = t / tiles_x, tile_x = t - tile_y * tiles_x;
        const int64_t row0 = (int64_t)tile_y * kFp6Tile, col0 = (int64_t)tile_x * kFp6Tile;
#pragma unroll
        for (int k = 0; k < LOADS; ++k) {
            const int idx = tid + k * kFp6Threads, r = idx / PER_ROW, c = (idx % PER_ROW) * VEC;
            const uint4 v = regs[k];
            float *d = tile + r * kFp6Pitch + c;
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
            for (int item = tid; item < kFp6Tile * BLOCKS; item += kFp6Threads) {
                const int r = item / BLOCKS, b = item % BLOCKS;
                if (row0 + r < rows && col0 + b * kBlock < cols) {
                    float v[kBlock];
#pragma unroll
                    for (int i = 0; i < kBlock; i += 4) {
                        const float4 f = *reinterpret_cast<const float4 *>(tile + r * kFp6Pitch + b * kBlock + i);
                        v[i] = f.x; v[i + 1] = f.y; v[i + 2] = f.z; v[i + 3] = f.w;
                    }
                    uint32_t w[6], sb;
                    fp6_block<F>(v, w, sb);
                    fp6_store_block(q_row + (row0 + r) * (cols / 4 * 3) + (col0 / kBlock + b) * kFp6BlockBytes, w);
                    s_row[fp6_scale_index<TILED>(row0 + r, col0 / kBlock + b, nb)] = (uint8_t)sb;
                }
            }
        }
        if constexpr (COL) {
            const int64_t nbT = rows / kBlock;
            for (int item = tid; item < kFp6Tile * BLOCKS; item += kFp6Threads) {
                const int c = item % kFp6Tile, b = item / kFp6Tile;  // neighbouring work-items walk down neighbouring columns
                if (col0 + c < cols && row0 + b * kBlock < rows) {
                    float v[kBlock];
#pragma unroll
                    for (int i = 0; i < kBlock; ++i)
                        v[i] = tile[(b * kBlock + i) * kFp6Pitch + c];
                    uint32_t w[6], sb;
                    fp6_block<F>(v, w, sb);
                    fp6_store_block(q_colT + (col0 + c) * (rows / 4 * 3) + (row0 / kBlock + b) * kFp6BlockBytes, w);
                    s_colT[fp6_scale_index<TILED>(col0 + c, row0 / kBlock + b, nbT)] = (uint8_t)sb;
                }
            }
        }
        __syncthreads();  // the tile in LDS is overwritten by the next round
    }
}

template <class F, bool BF16, bool TILED>
static hipError_t launch_quantize_fp6_t(const void *src, int64_t rows, int64_t cols, int64_t ld, int axis, uint8_t *q_row,
                                        uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, hipStream_t stream)
{
    const int64_t tiles_x = (cols + kFp6Tile - 1) / kFp6Tile, tiles_y = (rows + kFp6Tile - 1) / kFp6Tile;
    if (tiles_x * tiles_y > 0x7FFFFFFF)
        return hipErrorInvalidConfiguration;
    int dev = 0, cus = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err == hipSuccess)
        err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (err != hipSuccess)
        return err;
    const int64_t ntiles = tiles_x * tiles_y, resident = 2 * (int64_t)(cus > 0 ? cus : 1);  // two tiles of LDS fit a compute unit
    const dim3 grid((unsigned)(ntiles < resident ? ntiles : resident)), block(kFp6Threads);
    const uint8_t *s = static_cast<const uint8_t *>(src);
    const int64_t ldb = ld * (BF16 ? 2 : 4);
#define MXFP6_LAUNCH(R, C)                                                                                              \
    {                                                                                                                   \
        auto kern = quantize_fp6_kernel<F, BF16, R, C, TILED>;                                                          \
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                                  \
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kFp6LdsBytes);             \
        if (e != hipSuccess)                                                                                            \
            return e;                                                                                                   \
        hipLaunchKernelGGL(kern, grid, block, kFp6LdsBytes, stream, s, rows, cols, ldb, q_row, s_row, q_colT, s_colT,    \
                           (uint32_t)tiles_x, (uint32_t)ntiles);                                                        \
    }
    if (axis == 1)
        MXFP6_LAUNCH(true, false)
    else if (axis == 2)
        MXFP6_LAUNCH(false, true)
    else
        MXFP6_LAUNCH(true, true)
#undef MXFP6_LAUNCH
    return hipGetLastError();
}

template <class F>
static hipError_t launch_quantize_fp6_f(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis, uint8_t *q_row,
                                        uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, bool tiled, hipStream_t stream)
{
    if (bf16)
        return tiled ? launch_quantize_fp6_t<F, true, true>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream)
                     : launch_quantize_fp6_t<F, true, false>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream);
    return tiled ? launch_quantize_fp6_t<F, false, true>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream)
                 : launch_quantize_fp6_t<F, false, false>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream);
}

hipError_t launch_quantize_fp6(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis, bool e3m2, uint8_t *q_row,
                               uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, bool tiled_scales, hipStream_t stream)
{
    return e3m2 ? launch_quantize_fp6_f<E3M2>(src, bf16, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, tiled_scales, stream)
                : launch_quantize_fp6_f<E2M3>(src, bf16, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, tiled_scales, stream);
}

// ---- decode and expansion: one work-item per block (24 bytes in) -------------------------------------------------
// magnitude of a code as a float (exact): exponent field 0 is subnormal
template <class F> __device__ __forceinline__ float fp6_magnitude(uint32_t code)
{
    const int e = (int)((code >> F::M) & ((1u << F::E) - 1u)), m = (int)(code & ((1u << F::M) - 1u));
    return ldexpf((float)((e ? (1 << F::M) : 0) + m), (e ? e - 1 : 0) + F::EMIN - F::M);
}

__device__ __forceinline__ void fp6_load_block(const uint8_t *p, uint32_t (&w)[6])
{
    const uint2 *s = reinterpret_cast<const uint2 *>(p);
    const uint2 a = s[0], b = s[1], c = s[2];
    w[0] = a.x; w[1] = a.y; w[2] = b.x; w[3] = b.y; w[4] = c.x; w[5] = c.y;
}

__device__ __forceinline__ uint32_t fp6_code_at(const uint32_t (&w)[6], int i)  // i is a compile-time constant at every call
{
    const int pos = 6 * i;
    uint32_t c = w[pos / 32] >> (pos % 32);
    if (pos % 32 > 26)
        c |= w[pos / 32 + 1] << (32 - pos % 32);
    return c & 63u;
}

template <class F, bool BF16, bool TILED>
__global__ __launch_bounds__(256) void dequantize_fp6_kernel(const uint8_t *__restrict__ q, const uint8_t *__restrict__ s,
                                                             int64_t rows, int64_t cols, uint8_t *__restrict__ dst, int64_t ld_bytes)
{
    // The 64 values of the format, one per LDS bank: lanes that look up different codes never collide, lanes with
    // the same code share a broadcast. A lookup replaces about ten vector instructions per element.
    __shared__ float value_of[64];
    if (threadIdx.x < 64) {
        const float mag = fp6_magnitude<F>(threadIdx.x);
        value_of[threadIdx.x] = (threadIdx.x & 32u) ? -mag : mag;
    }
    __syncthreads();
    // An item = a quarter of a block: eight codes (48 bits at byte 6k of the block) -> 16 bytes of BF16 or 32 bytes of
    // FP32, so that neighbouring work-items read overlapping dwords of one line and store neighbouring pieces.
    const int64_t nb = cols / kBlock, total = rows * nb * 4;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t blk = t >> 2;
        const int k = (int)(t & 3);
        const int64_t r = blk / nb, b = blk - r * nb;
        const uint32_t sb = s[fp6_scale_index<TILED>(r, b, nb)];
        // two dwords from the dword boundary at or below byte 6k (bytes 0, 4, 12, 16 of the 24): all inside the block
        const uint32_t *src = reinterpret_cast<const uint32_t *>(q + blk * kFp6BlockBytes + ((6 * k) & ~3));
        const uint64_t both = ((uint64_t)src[1] << 32) | src[0];
        const uint64_t bits = both >> (16 * (k & 1));
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            v[i] = sb == 0xFFu ? __uint_as_float(0x7FC00000u)
                               : ldexpf(value_of[(uint32_t)(bits >> (6 * i)) & 63u], (int)sb - 127);
        uint8_t *out = dst + r * ld_bytes + (b * kBlock + 8 * k) * (BF16 ? 2 : 4);
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

// Expansion to E4M3 bytes, four codes at a time in the bytes of a dword. Every 6-bit magnitude is zero or a normal
// E4M3 number with at most 3 mantissa bits. A normal 6-bit number keeps its fields: exponent re-biased by 7 - BIAS,
// mantissa left-aligned in three bits, i.e. (magnitude << (3 - M)) + ((7 - BIAS) << 3). Zero and the 2^M - 1 subnormal
// magnitudes m * 2^(EMIN - M) come from an eight-byte table through one byte permute.
template <class F> constexpr uint32_t fp6_subnormal_as_e4m3(int m)  // E4M3 byte of m * 2^(EMIN - M), 0 <= m < 2^M
{
    if (m == 0)
        return 0u;
    int p = 0;
    while ((2 << p) <= m)
        ++p;  // m = 2^p * (1 + f)
    return (uint32_t)(((p + F::EMIN - F::M + 7) << 3) | (((m - (1 << p)) << (3 - p)) & 7));
}
template <class F> constexpr uint32_t fp6_subnormal_table(int first)  // entries first .. first + 3, one per byte
{
    uint32_t t = 0;
    for (int i = 0; i < 4; ++i)
        if (first + i < (1 << F::M))
            t |= fp6_subnormal_as_e4m3<F>(first + i) << (8 * i);
    return t;
}

__device__ __forceinline__ uint32_t fp6_spread4(uint32_t x)  // four codes in bits 0 .. 23 -> one per byte
{
    return (x & 0x3Fu) | ((x << 2) & 0x3F00u) | ((x << 4) & 0x3F0000u) | ((x << 6) & 0x3F000000u);
}

template <class F> __device__ __forceinline__ uint32_t fp6x4_as_e4m3(uint32_t codes)  // one code per byte in, one E4M3 byte each out
{
    const uint32_t mag = codes & 0x1F1F1F1Fu;
    uint32_t any = mag >> F::M;  // bit 0 of a byte <- the OR of its exponent bits (what spills in from the next byte lands above bit 0)
#pragma unroll
    for (int i = 1; i < F::E; ++i)
        any |= mag >> (F::M + i);
    const uint32_t one = any & 0x01010101u;
    const uint32_t normal = (one << 8) - one;  // 0xFF in the bytes that hold a normal number
    const uint32_t kept = (mag << (3 - F::M)) + 0x01010101u * (uint32_t)((7 - F::BIAS) << 3);
    const uint32_t looked_up = __builtin_amdgcn_perm(fp6_subnormal_table<F>(4), fp6_subnormal_table<F>(0), mag & 0x07070707u);
    return (normal & kept) | (~normal & looked_up) | ((codes & 0x20202020u) << 2);
}

template <class F>
__global__ __launch_bounds__(256) void expand_fp6_kernel(const uint8_t *__restrict__ q, int64_t blocks, uint8_t *__restrict__ q8)
{
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < blocks; t += (int64_t)gridDim.x * blockDim.x) {
        uint32_t w[6];
        fp6_load_block(q + t * kFp6BlockBytes, w);
        uint32_t o[8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {  // three dwords hold sixteen codes: 24 bits at offsets 0, 24, 48, 72
            const uint32_t a = w[3 * h], b = w[3 * h + 1], c = w[3 * h + 2];
            o[4 * h] = fp6x4_as_e4m3<F>(fp6_spread4(a));
            o[4 * h + 1] = fp6x4_as_e4m3<F>(fp6_spread4((a >> 24) | (b << 8)));
            o[4 * h + 2] = fp6x4_as_e4m3<F>(fp6_spread4((b >> 16) | (c << 16)));
            o[4 * h + 3] = fp6x4_as_e4m3<F>(fp6_spread4(c >> 8));
        }
        uint4 *d = reinterpret_cast<uint4 *>(q8 + t * kBlock);
        d[0] = make_uint4(o[0], o[1], o[2], o[3]);
        d[1] = make_uint4(o[4], o[5], o[6], o[7]);
    }
}

static dim3 fp6_block_grid(int64_t blocks)
{
    const int64_t want = (blocks + 255) / 256;
    return dim3((unsigned)(want < 65536 ? want : 65536));
}

hipError_t launch_dequantize_fp6(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, bool e3m2, void *dst, bool bf16,
                                 bool tiled, int64_t ld, hipStream_t stream)
{
    const dim3 grid = fp6_block_grid(rows * (cols / kBlock) * 4), block(256);  // four work-items per block
    uint8_t *d = static_cast<uint8_t *>(dst);
    const int64_t ldb = ld * (bf16 ? 2 : 4);
#define MXFP6_DEQ(F)                                                                                                     \
    {                                                                                                                    \
        if (bf16) {                                                                                                      \
            if (tiled)                                                                                                   \
                hipLaunchKernelGGL((dequantize_fp6_kernel<F, true, true>), grid, block, 0, stream, q, s, rows, cols, d, ldb);  \
            else                                                                                                         \
                hipLaunchKernelGGL((dequantize_fp6_kernel<F, true, false>), grid, block, 0, stream, q, s, rows, cols, d, ldb); \
        } else {                                                                                                         \
            if (tiled)                                                                                                   \
                hipLaunchKernelGGL((dequantize_fp6_kernel<F, false, true>), grid, block, 0, stream, q, s, rows, cols, d, ldb); \
            else                                                                                                         \
                hipLaunchKernelGGL((dequantize_fp6_kernel<F, false, false>), grid, block, 0, stream, q, s, rows, cols, d, ldb);\
        }                                                                                                                \
    }
    if (e3m2)
        MXFP6_DEQ(E3M2)
    else
        MXFP6_DEQ(E2M3)
#undef MXFP6_DEQ
    return hipGetLastError();
}

hipError_t launch_expand_fp6(const uint8_t *q, int64_t rows, int64_t cols, bool e3m2, uint8_t *q8, hipStream_t stream)
{
    const int64_t blocks = rows * (cols / kBlock);
    const dim3 grid = fp6_block_grid(blocks), block(256);
    if (e3m2)
        hipLaunchKernelGGL(expand_fp6_kernel<E3M2>, grid, block, 0, stream, q, blocks, q8);
    else
        hipLaunchKernelGGL(expand_fp6_kernel<E2M3>, grid, block, 0, stream, q, blocks, q8);
    return hipGetLastError();
}

}  // namespace mxfp8
