// MXFP8 quantizer for gfx950: FP32/BF16 -> E4M3 elements + UE8M0 block scales, along rows, along
// columns, or both from a single read of the source (Section 3.2; conversion of Section 3.3,
// Algorithm 1, Appendix A.1 and A.2).
//
// Work decomposition. One wavefront owns a tile of 32 rows x 16*VEC columns, VEC = elements per
// 128-bit load (8 for BF16, 4 for FP32). Lane l = 16*rs + cc holds, in registers, rows
// 8*rs .. 8*rs+7 of column chunk cc (VEC consecutive columns): eight 128-bit loads, each covering
// 256 contiguous bytes of four rows per instruction.
//   * Row direction: a 32-column block is spread over 32/VEC neighbouring lanes of one row of 16
//     lanes, so its amax is a DPP butterfly (no LDS); each lane then converts its own VEC values.
//   * Column direction: a 32-row block is 8 rows in each of the four lanes {cc, cc+16, cc+32,
//     cc+48}; the per-lane maxima are combined with two lane exchanges, then every lane converts
//     its 8 rows x VEC columns walking DOWN the column, so the packed bytes come out in the order
//     the transposed copy stores them (8 consecutive bytes per column, no transpose in memory).
// A workgroup stacks four wavefronts vertically (128 rows), so the four 32-byte pieces of a
// 128-byte line of the transposed copy are written by the same workgroup at the same time.
//
// amax is taken as an unsigned integer maximum of the magnitude bits: exact, independent of
// denormal modes, and it orders NaN > Inf > finite, which is all the special-value rule needs.
#include "mxfp8_device.h"

namespace mxfp8 {

constexpr int kQuantWaves = 4;
constexpr int kQuantThreads = 64 * kQuantWaves;
constexpr int kTileRows = 32;  // per wavefront

template <bool BF16> struct Vec;
template <> struct Vec<true> { static constexpr int n = 8; };
template <> struct Vec<false> { static constexpr int n = 4; };

// magnitude bits of one 128-bit vector, reduced to one value per lane
template <bool BF16> __device__ __forceinline__ uint32_t lane_amax(const uint4 &x)
{
    if constexpr (BF16) {
        uint32_t m = pk_max_u16(pk_max_u16(x.x & 0x7FFF7FFFu, x.y & 0x7FFF7FFFu),
                                pk_max_u16(x.z & 0x7FFF7FFFu, x.w & 0x7FFF7FFFu));
        return umax(m & 0xFFFFu, m >> 16);
    } else {
        return umax(umax(x.x & 0x7FFFFFFFu, x.y & 0x7FFFFFFFu), umax(x.z & 0x7FFFFFFFu, x.w & 0x7FFFFFFFu));
    }
}

template <bool BF16> __device__ __forceinline__ uint32_t scale_byte(uint32_t abs_bits)
{
    if constexpr (BF16)
        return scale_byte_from_bf16_bits(abs_bits);
    else
        return scale_byte_from_f32_bits(abs_bits);
}

// BF16 element `j` (0..7) of a 128-bit vector, as 16 bits
__device__ __forceinline__ uint32_t bf16_at(const uint4 &x, int j)
{
    const uint32_t w = (j >> 1) == 0 ? x.x : (j >> 1) == 1 ? x.y : (j >> 1) == 2 ? x.z : x.w;
    return (j & 1) ? w >> 16 : w & 0xFFFFu;
}
__device__ __forceinline__ uint32_t word_at(const uint4 &x, int j)
{
    return j == 0 ? x.x : j == 1 ? x.y : j == 2 ? x.z : x.w;
}

template <bool BF16, bool ROW, bool COL>
__global__ __launch_bounds__(kQuantThreads) void quantize_kernel(
    const uint8_t *__restrict__ src, int64_t rows, int64_t cols, int64_t ld_bytes,
    uint8_t *__restrict__ q_row, uint8_t *__restrict__ s_row, uint8_t *__restrict__ q_colT,
    uint8_t *__restrict__ s_colT, uint32_t tiles_x)
{
    constexpr int VEC = Vec<BF16>::n;
    constexpr int TILE_COLS = 16 * VEC;
    constexpr int ESIZE = BF16 ? 2 : 4;
    constexpr int LANES_PER_BLOCK = kBlock / VEC;  // 4 (BF16) or 8 (FP32)

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int cc = lane & 15;
    const int rs = lane >> 4;
    const uint32_t tile_y = blockIdx.x / tiles_x, tile_x = blockIdx.x - tile_y * tiles_x;
    const int64_t col0 = (int64_t)tile_x * TILE_COLS + cc * VEC;
    const int64_t row0 = ((int64_t)tile_y * kQuantWaves + wave) * kTileRows + rs * 8;
    // rows % 32 == 0 and cols % 32 == 0: a wavefront tile is wholly inside or outside in rows, and
    // whole 32-column blocks (groups of LANES_PER_BLOCK lanes) are inside or outside in columns.
    const bool active = col0 < cols && row0 < rows;

    uint4 x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        x[i] = make_uint4(0, 0, 0, 0);
        if (active)
            x[i] = *reinterpret_cast<const uint4 *>(src + (row0 + i) * ld_bytes + col0 * ESIZE);
    }

    if constexpr (ROW) {
        const int64_t nb = cols / kBlock;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t am = lane_amax<BF16>(x[i]);
            am = umax(am, dpp_xor1(am));
            am = umax(am, dpp_xor2(am));
            if constexpr (!BF16)
                am = umax(am, dpp_half_mirror(am));
            const uint32_t sb = scale_byte<BF16>(am);
            const float sc = scale_operand(sb);
            uint32_t q0 = 0, q1 = 0;
            if constexpr (BF16) {
                q0 = cvt2_bf16(q0, x[i].x, sc, false);
                q0 = cvt2_bf16(q0, x[i].y, sc, true);
                q1 = cvt2_bf16(q1, x[i].z, sc, false);
                q1 = cvt2_bf16(q1, x[i].w, sc, true);
            } else {
                q0 = cvt2_f32(q0, __uint_as_float(x[i].x), __uint_as_float(x[i].y), sc, false);
                q0 = cvt2_f32(q0, __uint_as_float(x[i].z), __uint_as_float(x[i].w), sc, true);
            }
            if (sb >= 254) {  // block holds Inf or NaN: rare, handled byte by byte
                if (sb == 0xFF) {
                    q0 = 0x7F7F7F7Fu;
                    q1 = 0x7F7F7F7Fu;
                } else if constexpr (BF16) {
                    uint32_t f0 = 0, f1 = 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        f0 |= inf_byte_bf16(bf16_at(x[i], j), (q0 >> (8 * j)) & 0xFFu) << (8 * j);
                        f1 |= inf_byte_bf16(bf16_at(x[i], 4 + j), (q1 >> (8 * j)) & 0xFFu) << (8 * j);
                    }
                    q0 = f0;
                    q1 = f1;
                } else {
                    uint32_t f0 = 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        f0 |= inf_byte_f32(word_at(x[i], j), (q0 >> (8 * j)) & 0xFFu) << (8 * j);
                    q0 = f0;
                }
            }
            if (active) {
                uint8_t *qp = q_row + (row0 + i) * cols + col0;
                if constexpr (BF16)
                    *reinterpret_cast<uint2 *>(qp) = make_uint2(q0, q1);
                else
                    *reinterpret_cast<uint32_t *>(qp) = q0;
                if ((cc % LANES_PER_BLOCK) == 0)
                    s_row[(row0 + i) * nb + col0 / kBlock] = (uint8_t)sb;
            }
        }
    }

    if constexpr (COL) {
        const int64_t nb = rows / kBlock;
        // per-lane maxima of the 8 rows, element-wise over the VEC columns
        uint32_t cm[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            uint32_t m = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t v = word_at(x[i], w);
                if constexpr (BF16)
                    m = pk_max_u16(m, v & 0x7FFF7FFFu);
                else
                    m = umax(m, v & 0x7FFFFFFFu);
            }
            // the other three lanes holding rows of the same 32-row block: lane ^ 16, lane ^ 32
            uint32_t o = (uint32_t)__shfl_xor((int)m, 16, 64);
            m = BF16 ? pk_max_u16(m, o) : umax(m, o);
            o = (uint32_t)__shfl_xor((int)m, 32, 64);
            m = BF16 ? pk_max_u16(m, o) : umax(m, o);
            cm[w] = m;
        }
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            uint32_t am;
            if constexpr (BF16)
                am = (j & 1) ? cm[j >> 1] >> 16 : cm[j >> 1] & 0xFFFFu;
            else
                am = cm[j];
            const uint32_t sb = scale_byte<BF16>(am);
            const float sc = scale_operand(sb);
            uint32_t q0 = 0, q1 = 0;  // rows 0..3 and 4..7 of this lane, one byte each
            if constexpr (BF16) {
                // pair (row i, row i+1) of column j: bytes [1:0] or [3:2] of each word
                const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
#define MXFP8_PAIR(i) __builtin_amdgcn_perm(word_at(x[(i) + 1], j >> 1), word_at(x[i], j >> 1), sel)
                q0 = cvt2_bf16(q0, MXFP8_PAIR(0), sc, false);
                q0 = cvt2_bf16(q0, MXFP8_PAIR(2), sc, true);
                q1 = cvt2_bf16(q1, MXFP8_PAIR(4), sc, false);
                q1 = cvt2_bf16(q1, MXFP8_PAIR(6), sc, true);
#undef MXFP8_PAIR
            } else {
#define MXFP8_F(i) __uint_as_float(word_at(x[i], j))
                q0 = cvt2_f32(q0, MXFP8_F(0), MXFP8_F(1), sc, false);
                q0 = cvt2_f32(q0, MXFP8_F(2), MXFP8_F(3), sc, true);
                q1 = cvt2_f32(q1, MXFP8_F(4), MXFP8_F(5), sc, false);
                q1 = cvt2_f32(q1, MXFP8_F(6), MXFP8_F(7), sc, true);
#undef MXFP8_F
            }
            if (sb >= 254) {
                if (sb == 0xFF) {
                    q0 = 0x7F7F7F7Fu;
                    q1 = 0x7F7F7F7Fu;
                } else {
                    uint32_t f0 = 0, f1 = 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if constexpr (BF16) {
                            f0 |= inf_byte_bf16(bf16_at(x[i], j), (q0 >> (8 * i)) & 0xFFu) << (8 * i);
                            f1 |= inf_byte_bf16(bf16_at(x[4 + i], j), (q1 >> (8 * i)) & 0xFFu) << (8 * i);
                        } else {
                            f0 |= inf_byte_f32(word_at(x[i], j), (q0 >> (8 * i)) & 0xFFu) << (8 * i);
                            f1 |= inf_byte_f32(word_at(x[4 + i], j), (q1 >> (8 * i)) & 0xFFu) << (8 * i);
                        }
                    }
                    q0 = f0;
                    q1 = f1;
                }
            }
            if (active) {
                *reinterpret_cast<uint2 *>(q_colT + (col0 + j) * rows + row0) = make_uint2(q0, q1);
                if (rs == 0)
                    s_colT[(col0 + j) * nb + row0 / kBlock] = (uint8_t)sb;
            }
        }
    }
}

template <bool BF16>
static hipError_t launch_quantize_t(const void *src, int64_t rows, int64_t cols, int64_t ld, int axis,
                                    uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                                    hipStream_t stream)
{
    constexpr int TILE_COLS = 16 * Vec<BF16>::n;
    const int64_t tiles_x = (cols + TILE_COLS - 1) / TILE_COLS;
    const int64_t tiles_y = (rows + kTileRows * kQuantWaves - 1) / (kTileRows * kQuantWaves);
    if (tiles_x * tiles_y > 0x7FFFFFFF)
        return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)(tiles_x * tiles_y));
    dim3 block(kQuantThreads);
    const uint8_t *s = static_cast<const uint8_t *>(src);
    const int64_t ldb = ld * (BF16 ? 2 : 4);
    if (axis == 1)
        hipLaunchKernelGGL((quantize_kernel<BF16, true, false>), grid, block, 0, stream, s, rows, cols, ldb,
                           q_row, s_row, q_colT, s_colT, (uint32_t)tiles_x);
    else if (axis == 2)
        hipLaunchKernelGGL((quantize_kernel<BF16, false, true>), grid, block, 0, stream, s, rows, cols, ldb,
                           q_row, s_row, q_colT, s_colT, (uint32_t)tiles_x);
    else
        hipLaunchKernelGGL((quantize_kernel<BF16, true, true>), grid, block, 0, stream, s, rows, cols, ldb,
                           q_row, s_row, q_colT, s_colT, (uint32_t)tiles_x);
    return hipGetLastError();
}

hipError_t launch_quantize(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis,
                           uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                           hipStream_t stream)
{
    return bf16 ? launch_quantize_t<true>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream)
                : launch_quantize_t<false>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream);
}

}  // namespace mxfp8
