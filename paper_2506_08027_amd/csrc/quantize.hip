// MXFP8 quantizer for gfx950: FP32/BF16 -> E4M3 elements + UE8M0 block scales, along rows, along
// columns, or both from a single read of the source (Section 3.2; conversion of Section 3.3,
// Algorithm 1, Appendix A.1 and A.2).
//
// Work decomposition. A workgroup of four wavefronts owns a tile of 128 rows x 128 columns; each
// wavefront owns 32 rows of it (one column block) and holds them in registers:
//   BF16: lane l = 16*rs + cc holds rows 8*rs..8*rs+7   of columns 8*cc..8*cc+7 (8 x 128-bit loads)
//   FP32: lane l = 32*rs + cc holds rows 16*rs..16*rs+15 of columns 4*cc..4*cc+3 (16 x 128-bit loads)
// so every load instruction reads whole 256/512-byte row segments.
//   * Row direction: a 32-column block is spread over 4 (BF16) or 8 (FP32) neighbouring lanes of a
//     DPP row, so its amax is a DPP butterfly; each lane converts its own values and stores them
//     directly: the 16 or 32 lanes of a row segment write one full 128-byte line.
//   * Column direction: a 32-row block is split over the 4 (BF16) or 2 (FP32) lanes that share cc;
//     the per-lane maxima are combined with lane exchanges, then every lane converts its rows
//     walking DOWN each column, so the packed bytes come out in the order the transposed copy
//     stores them. The 8- or 16-byte pieces are staged in LDS as [column][128 row bytes] and
//     written out by the whole workgroup as full 128-byte lines of q_colT (a direct store would
//     scatter 32-byte pieces, which the memory system handles at roughly half the rate).
//   * Scale bytes take the same road: they are collected in LDS and leave as one dword per row
//     (4 column blocks) and one dword per column (4 row blocks) instead of single bytes.
//
// amax is taken as an unsigned integer maximum of the magnitude bits: exact, independent of
// denormal modes, and it orders NaN > Inf > finite, which is all the special-value rule needs.
#include "mxfp8_device.h"

namespace mxfp8 {

constexpr int kQuantWaves = 4;
constexpr int kQuantThreads = 64 * kQuantWaves;
constexpr int kTile = 128;  // rows and columns per workgroup

template <bool BF16> struct QTraits;
template <> struct QTraits<true> {
    static constexpr int VEC = 8;    // elements per 128-bit load
    static constexpr int ROWS = 8;   // rows per lane
    static constexpr int CC = 16;    // lanes along the columns
};
template <> struct QTraits<false> {
    static constexpr int VEC = 4;
    static constexpr int ROWS = 16;
    static constexpr int CC = 32;
};

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

template <bool BF16, int MODE> __device__ __forceinline__ uint32_t scale_byte(uint32_t abs_bits)
{
    if constexpr (MODE == 0)
        return BF16 ? scale_byte_from_bf16_bits(abs_bits) : scale_byte_from_f32_bits(abs_bits);
    else
        return BF16 ? scale_byte_mode_bf16_bits<MODE>(abs_bits) : scale_byte_mode_f32_bits<MODE>(abs_bits);
}
// the pair conversions in the element format of MODE
template <int MODE> __device__ __forceinline__ uint32_t cvt_pair_bf16(uint32_t old, uint32_t pair, float sc, bool hi)
{
    if constexpr (MODE & kModeE5M2)
        return cvt2_e5m2_bf16(old, pair, sc, hi);
    else
        return cvt2_bf16(old, pair, sc, hi);
}
template <int MODE> __device__ __forceinline__ uint32_t cvt_pair_f32(uint32_t old, float a, float b, float sc, bool hi)
{
    if constexpr (MODE & kModeE5M2)
        return cvt2_e5m2_f32(old, a, b, sc, hi);
    else
        return cvt2_f32(old, a, b, sc, hi);
}

__device__ __forceinline__ uint32_t word_at(const uint4 &x, int j)
{
    return j == 0 ? x.x : j == 1 ? x.y : j == 2 ? x.z : x.w;
}
// element j of a 128-bit vector as raw bits (16 bits for BF16, 32 for FP32)
template <bool BF16> __device__ __forceinline__ uint32_t elem_at(const uint4 &x, int j)
{
    if constexpr (BF16) {
        const uint32_t w = word_at(x, j >> 1);
        return (j & 1) ? w >> 16 : w & 0xFFFFu;
    } else {
        return word_at(x, j);
    }
}
// What becomes of element byte q whose input has the raw bits `bits`, in a block that holds no NaN: the
// recipe (MODE 0) only has infinities to clamp; the ablation arms clamp whatever rounds beyond the maximum.
template <bool BF16, int MODE> __device__ __forceinline__ uint32_t inf_byte(uint32_t bits, uint32_t q)
{
    if constexpr (MODE == 0) {
        return BF16 ? inf_byte_bf16(bits, q) : inf_byte_f32(bits, q);
    } else {
        const bool negative = BF16 ? (bits & 0x8000u) != 0 : (bits & 0x80000000u) != 0;
        const bool inf = BF16 ? (bits & 0x7FFFu) == 0x7F80u : (bits & 0x7FFFFFFFu) == 0x7F800000u;
        return saturate_byte<MODE>(q, negative, inf);
    }
}

// Four element bytes of column j taken from rows r0..r0+3 of the lane's registers.
template <bool BF16, int MODE, int NROWS>
__device__ __forceinline__ uint32_t convert_down4(const uint4 (&x)[NROWS], int r0, int j, float sc)
{
    uint32_t q = 0;
    if constexpr (BF16) {
        // pair (row r, row r+1) of column j: bytes [1:0] or [3:2] of each word
        const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
        q = cvt_pair_bf16<MODE>(q, __builtin_amdgcn_perm(word_at(x[r0 + 1], j >> 1), word_at(x[r0], j >> 1), sel), sc, false);
        q = cvt_pair_bf16<MODE>(q, __builtin_amdgcn_perm(word_at(x[r0 + 3], j >> 1), word_at(x[r0 + 2], j >> 1), sel), sc, true);
    } else {
        q = cvt_pair_f32<MODE>(q, __uint_as_float(word_at(x[r0], j)), __uint_as_float(word_at(x[r0 + 1], j)), sc, false);
        q = cvt_pair_f32<MODE>(q, __uint_as_float(word_at(x[r0 + 2], j)), __uint_as_float(word_at(x[r0 + 3], j)), sc, true);
    }
    return q;
}

// Four E4M3 codes and the scale byte of their block as four FP32 values (exact: a code has 4 significant bits
// and FP32 holds every Q * 2^n down to its subnormals); a 0xFF scale gives NaN.
__device__ __forceinline__ uint4 decode_mx4(uint32_t q, uint32_t sb)
{
    typedef float v2f __attribute__((ext_vector_type(2)));
    const v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)q, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)q, true);
    const int e = (int)sb - 127;
    if (sb == 0xFF)
        return make_uint4(0x7FC00000u, 0x7FC00000u, 0x7FC00000u, 0x7FC00000u);
    return make_uint4(__float_as_uint(ldexpf(lo[0], e)), __float_as_uint(ldexpf(lo[1], e)), __float_as_uint(ldexpf(hi[0], e)),
                      __float_as_uint(ldexpf(hi[1], e)));
}

// MXSRC (BF16 = false): the source is itself an MXFP8 row copy, src = its element bytes [rows x cols] (dense),
// src_s = its scale bytes in the same layout as the outputs. Every value is decoded exactly on load and then
// treated like an FP32 source: this derives the column copy of a tensor from its row copy (single-copy
// storage, Section 5) at the price of a second rounding.
template <bool BF16, bool ROW, bool COL, bool TILED, int MODE, bool MXSRC = false>
__global__ __launch_bounds__(kQuantThreads) void quantize_kernel(
    const uint8_t *__restrict__ src, int64_t rows, int64_t cols, int64_t ld_bytes,
    uint8_t *__restrict__ q_row, uint8_t *__restrict__ s_row, uint8_t *__restrict__ q_colT,
    uint8_t *__restrict__ s_colT, uint32_t tiles_x, uint32_t ntiles, const uint8_t *__restrict__ src_s)
{
    static_assert(!MXSRC || !BF16, "an MXFP8 source goes through the FP32 register layout");
    using T = QTraits<BF16>;
    constexpr int VEC = T::VEC, ROWS = T::ROWS, CC = T::CC;
    constexpr int ESIZE = BF16 ? 2 : 4;
    constexpr int LANES_PER_BLOCK = kBlock / VEC;  // lanes sharing a row block: 4 (BF16) or 8 (FP32)
    [[maybe_unused]] constexpr int PIECE = ROWS;                    // bytes a lane contributes to one column of q_colT

    // column copy staged as [128 columns][128 row bytes]; row / column scale bytes as [128][4]
    __shared__ __attribute__((aligned(16))) uint8_t lds_q[COL ? kTile * kTile : 16];
    __shared__ __attribute__((aligned(16))) uint8_t lds_rs[ROW ? kTile * 4 : 16];
    __shared__ __attribute__((aligned(16))) uint8_t lds_cs[COL ? kTile * 4 : 16];
    // MXFP8 source: the tile's element bytes (full 128-byte rows, loaded 16 bytes per work-item) and one dword
    // of scale bytes per row; the lanes pick their 4 codes per row from here
    __shared__ __attribute__((aligned(16))) uint8_t lds_src[MXSRC ? kTile * kTile : 16];
    __shared__ uint32_t lds_src_s[MXSRC ? kTile : 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int cc = lane % CC;
    const int rs = lane / CC;
    const int lrow0 = wave * 32 + rs * ROWS;  // first row of this lane inside the tile
    const int lcol0 = cc * VEC;               // first column of this lane inside the tile
    const int64_t nb_row = cols / kBlock, nb_col = rows / kBlock;

    // a workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x, ... (one tile each when the grid has one per tile)
    for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        // Order of the tiles over the workgroup ids: along the rows of the source, except that a wide tensor (more
        // columns than rows) whose column copy is wanted is walked down its columns, so that the workgroups running
        // side by side append to the same rows of the transposed copy. Measured on an MI355X over six shapes, both
        // source types: 6 % (both copies) to 17 % (column copy only) less time where the rule switches, 5 .. 30 %
        // more wherever it does not.
        const bool walk_down = COL && cols > rows;
        const uint32_t tiles_y = ntiles / tiles_x;
        const uint32_t tile_y = walk_down ? tile % tiles_y : tile / tiles_x, tile_x = walk_down ? tile / tiles_y : tile % tiles_x;
        const int64_t wg_col0 = (int64_t)tile_x * kTile, wg_row0 = (int64_t)tile_y * kTile;
        const int64_t col0 = wg_col0 + lcol0, row0 = wg_row0 + lrow0;
        // rows % 32 == 0 and cols % 32 == 0: a wavefront's 32 rows are wholly inside or outside a
        // ragged tile, and whole 32-column blocks (groups of LANES_PER_BLOCK lanes) are too.
        const bool active = col0 < cols && row0 < rows;

        if constexpr (MXSRC) {
#pragma unroll
            for (int k = 0; k < kTile * kTile / 16 / kQuantThreads; ++k) {
                const int idx = k * kQuantThreads + tid, r = idx / (kTile / 16), c = (idx % (kTile / 16)) * 16;
                if (wg_row0 + r < rows && wg_col0 + c < cols)   // cols % 32 == 0: a 16-byte piece is wholly inside or outside
                    *reinterpret_cast<uint4 *>(lds_src + r * kTile + c) =
                        stream_load(reinterpret_cast<const uint4 *>(src + (wg_row0 + r) * cols + wg_col0 + c));
            }
            if (tid < kTile && wg_row0 + tid < rows) {
                const int64_t r = wg_row0 + tid, b0 = wg_col0 / kBlock;  // b0 % 4 == 0
                uint32_t w = 0;
                if constexpr (TILED) {
                    w = *reinterpret_cast<const uint32_t *>(src_s + (((r >> 6) * ((nb_row + 3) / 4) + (b0 >> 2)) * 64 + (r & 63)) * 4);
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (b0 + b < nb_row)
                            w |= (uint32_t)src_s[r * nb_row + b0 + b] << (8 * b);
                }
                lds_src_s[tid] = w;
            }
            __syncthreads();
        }
        uint4 x[ROWS];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            x[i] = make_uint4(0, 0, 0, 0);
            if constexpr (MXSRC) {
                if (active)
                    x[i] = decode_mx4(*reinterpret_cast<const uint32_t *>(lds_src + (lrow0 + i) * kTile + lcol0),
                                      (lds_src_s[lrow0 + i] >> (8 * (lcol0 / kBlock))) & 0xFFu);
            } else if (active) {
                x[i] = stream_load(reinterpret_cast<const uint4 *>(src + (row0 + i) * ld_bytes + col0 * ESIZE));
            }
        }

        if constexpr (ROW) {
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                uint32_t am = lane_amax<BF16>(x[i]);
                am = umax(am, dpp_xor1(am));
                am = umax(am, dpp_xor2(am));
                if constexpr (!BF16)
                    am = umax(am, dpp_half_mirror(am));
                const uint32_t sb = scale_byte<BF16, MODE>(am);
                const float sc = scale_operand(sb);
                uint32_t q0 = 0, q1 = 0;
                if constexpr (BF16) {
                    q0 = cvt_pair_bf16<MODE>(q0, x[i].x, sc, false);
                    q0 = cvt_pair_bf16<MODE>(q0, x[i].y, sc, true);
                    q1 = cvt_pair_bf16<MODE>(q1, x[i].z, sc, false);
                    q1 = cvt_pair_bf16<MODE>(q1, x[i].w, sc, true);
                } else {
                    q0 = cvt_pair_f32<MODE>(q0, __uint_as_float(x[i].x), __uint_as_float(x[i].y), sc, false);
                    q0 = cvt_pair_f32<MODE>(q0, __uint_as_float(x[i].z), __uint_as_float(x[i].w), sc, true);
                }
                if (MODE != 0 || sb >= 254) {  // recipe: only blocks with Inf or NaN (rare); ablation arms: every block
                    if (sb == 0xFF) {
                        q0 = 0x7F7F7F7Fu;
                        q1 = 0x7F7F7F7Fu;
                    } else {
                        uint32_t f0 = 0, f1 = 0;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            f0 |= inf_byte<BF16, MODE>(elem_at<BF16>(x[i], j), (q0 >> (8 * j)) & 0xFFu) << (8 * j);
                            if constexpr (BF16)
                                f1 |= inf_byte<BF16, MODE>(elem_at<BF16>(x[i], 4 + j), (q1 >> (8 * j)) & 0xFFu) << (8 * j);
                        }
                        q0 = f0;
                        q1 = f1;
                    }
                }
                if (active) {
                    uint8_t *qp = q_row + (row0 + i) * cols + col0;
                    if constexpr (BF16)
                        stream_store(reinterpret_cast<uint2 *>(qp), make_uint2(q0, q1));
                    else
                        stream_store(reinterpret_cast<uint32_t *>(qp), q0);
                }
                if ((cc % LANES_PER_BLOCK) == 0)
                    lds_rs[(lrow0 + i) * 4 + cc / LANES_PER_BLOCK] = (uint8_t)sb;
            }
        }

        if constexpr (COL) {
            // per-lane maxima of the lane's rows, element-wise over the VEC columns
            uint32_t cm[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t m = 0;
#pragma unroll
                for (int i = 0; i < ROWS; ++i) {
                    const uint32_t v = word_at(x[i], w);
                    if constexpr (BF16)
                        m = pk_max_u16(m, v & 0x7FFF7FFFu);
                    else
                        m = umax(m, v & 0x7FFFFFFFu);
                }
                // the other lanes holding rows of the same 32-row block share cc: lane ^ 32 (and ^ 16)
                uint32_t o = (uint32_t)__shfl_xor((int)m, 32, 64);
                m = BF16 ? pk_max_u16(m, o) : umax(m, o);
                if constexpr (BF16) {
                    o = (uint32_t)__shfl_xor((int)m, 16, 64);
                    m = pk_max_u16(m, o);
                }
                cm[w] = m;
            }
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                uint32_t am;
                if constexpr (BF16)
                    am = (j & 1) ? cm[j >> 1] >> 16 : cm[j >> 1] & 0xFFFFu;
                else
                    am = cm[j];
                const uint32_t sb = scale_byte<BF16, MODE>(am);
                const float sc = scale_operand(sb);
                uint32_t q[ROWS / 4];  // one byte per row of this lane, in row order
#pragma unroll
                for (int r = 0; r < ROWS / 4; ++r)
                    q[r] = convert_down4<BF16, MODE, ROWS>(x, 4 * r, j, sc);
                if (MODE != 0 || sb >= 254) {
#pragma unroll
                    for (int r = 0; r < ROWS / 4; ++r) {
                        if (sb == 0xFF) {
                            q[r] = 0x7F7F7F7Fu;
                        } else {
                            uint32_t f = 0;
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                f |= inf_byte<BF16, MODE>(elem_at<BF16>(x[4 * r + i], j), (q[r] >> (8 * i)) & 0xFFu) << (8 * i);
                            q[r] = f;
                        }
                    }
                }
                // stage: column (lcol0 + j), row bytes lrow0 .. lrow0 + PIECE - 1. The 16-byte slot index
                // inside the 128-byte column line is XORed with the column chunk so that the lanes of one
                // store instruction (same j, consecutive cc) fall into different LDS banks.
                const int col = lcol0 + j;
                const int slot16 = (lrow0 >> 4) ^ (cc & 7);
                uint8_t *dst = lds_q + col * kTile + slot16 * 16 + (lrow0 & 15);
                if constexpr (BF16)
                    *reinterpret_cast<uint2 *>(dst) = make_uint2(q[0], q[1]);
                else
                    *reinterpret_cast<uint4 *>(dst) = make_uint4(q[0], q[1], q[2], q[3]);
                if (rs == 0)
                    lds_cs[col * 4 + wave] = (uint8_t)sb;
            }
        }

        __syncthreads();

        // ---- write-out of the staged pieces: full 128-byte lines, one dword of scales per row/column
        if constexpr (ROW) {
            if (tid < kTile) {
                const int64_t r = wg_row0 + tid;
                if (r < rows) {
                    const uint32_t w = *reinterpret_cast<const uint32_t *>(lds_rs + tid * 4);
                    if constexpr (TILED) {
                        // tiled scales: the dwords of 64 consecutive rows and one group of 4 blocks are
                        // contiguous, so the 64 lanes write 256 consecutive bytes (blocks past `cols`
                        // carry filler that nobody reads)
                        const int64_t kt_row = (nb_row + 3) / 4;
                        *reinterpret_cast<uint32_t *>(s_row + (((r >> 6) * kt_row + tile_x) * 64 + (r & 63)) * 4) = w;
                    } else {
                        uint8_t *sp = s_row + r * nb_row + wg_col0 / kBlock;
                        if (wg_col0 + kTile <= cols && (nb_row & 3) == 0 && (reinterpret_cast<uintptr_t>(s_row) & 3) == 0) {
                            *reinterpret_cast<uint32_t *>(sp) = w;
                        } else {
#pragma unroll
                            for (int b = 0; b < 4; ++b)
                                if (wg_col0 + b * kBlock < cols)
                                    sp[b] = (uint8_t)(w >> (8 * b));
                        }
                    }
                }
            }
        }
        if constexpr (COL) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int chunk = p * kQuantThreads + tid;  // 16-byte chunk of the staged tile
                const int col = chunk >> 3, part = chunk & 7;
                const int64_t c = wg_col0 + col, r = wg_row0 + part * 16;
                if (c < cols && r < rows) {
                    const int slot16 = part ^ ((col / VEC) & 7);
                    const uint4 v = *reinterpret_cast<const uint4 *>(lds_q + col * kTile + slot16 * 16);
                    stream_store(reinterpret_cast<uint4 *>(q_colT + c * rows + r), v);
                }
            }
            if (tid >= kTile) {  // the upper half of the workgroup, so that it overlaps the row scales
                const int col = tid - kTile;
                const int64_t c = wg_col0 + col;
                if (c < cols) {
                    const uint32_t w = *reinterpret_cast<const uint32_t *>(lds_cs + col * 4);
                    if constexpr (TILED) {
                        const int64_t kt_col = (nb_col + 3) / 4;
                        *reinterpret_cast<uint32_t *>(s_colT + (((c >> 6) * kt_col + tile_y) * 64 + (c & 63)) * 4) = w;
                    } else {
                        uint8_t *sp = s_colT + c * nb_col + wg_row0 / kBlock;
                        if (wg_row0 + kTile <= rows && (nb_col & 3) == 0 && (reinterpret_cast<uintptr_t>(s_colT) & 3) == 0) {
                            *reinterpret_cast<uint32_t *>(sp) = w;
                        } else {
#pragma unroll
                            for (int b = 0; b < 4; ++b)
                                if (wg_row0 + b * kBlock < rows)
                                    sp[b] = (uint8_t)(w >> (8 * b));
                        }
                    }
                }
            }
        }
        __syncthreads();  // the next tile reuses the staging arrays
    }
}

template <bool BF16, bool TILED, int MODE>
static hipError_t launch_quantize_t(const void *src, int64_t rows, int64_t cols, int64_t ld, int axis,
                                    uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                                    hipStream_t stream)
{
    const int64_t tiles_x = (cols + kTile - 1) / kTile;
    const int64_t tiles_y = (rows + kTile - 1) / kTile;
    if (tiles_x * tiles_y > 0x7FFFFFFF)
        return hipErrorInvalidConfiguration;
    // One workgroup per tile, except where a resident grid that walks over the tiles measured faster on an
    // MI355X: the both-axes pass over BF16 sources with 4 workgroups per compute unit (+6 % on [8192 x 4096];
    // FP32 sources and other grid sizes gained nothing).
    int64_t groups = tiles_x * tiles_y;
    if (BF16 && axis == 3) {
        int dev = 0, cus = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess)
            e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess)
            return e;
        if (cus > 0 && groups > 4 * (int64_t)cus)
            groups = 4 * (int64_t)cus;
    }
    dim3 grid((unsigned)groups);
    dim3 block(kQuantThreads);
    const uint8_t *s = static_cast<const uint8_t *>(src);
    const int64_t ldb = ld * (BF16 ? 2 : 4);
    if (axis == 1)
        hipLaunchKernelGGL((quantize_kernel<BF16, true, false, TILED, MODE>), grid, block, 0, stream, s, rows, cols, ldb,
                           q_row, s_row, q_colT, s_colT, (uint32_t)tiles_x, (uint32_t)(tiles_x * tiles_y), static_cast<const uint8_t *>(nullptr));
    else if (axis == 2)
        hipLaunchKernelGGL((quantize_kernel<BF16, false, true, TILED, MODE>), grid, block, 0, stream, s, rows, cols, ldb,
                           q_row, s_row, q_colT, s_colT, (uint32_t)tiles_x, (uint32_t)(tiles_x * tiles_y), static_cast<const uint8_t *>(nullptr));
    else
        hipLaunchKernelGGL((quantize_kernel<BF16, true, true, TILED, MODE>), grid, block, 0, stream, s, rows, cols, ldb,
                           q_row, s_row, q_colT, s_colT, (uint32_t)tiles_x, (uint32_t)(tiles_x * tiles_y), static_cast<const uint8_t *>(nullptr));
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_quantize_mode(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis,
                                       uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                                       bool tiled_scales, hipStream_t stream)
{
    if (tiled_scales)
        return bf16 ? launch_quantize_t<true, true, MODE>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream)
                    : launch_quantize_t<false, true, MODE>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream);
    return bf16 ? launch_quantize_t<true, false, MODE>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream)
                : launch_quantize_t<false, false, MODE>(src, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, stream);
}

// mode: bit 0 = E5M2 elements, bit 1 = OCP v1 scale rule (0 = the recipe)
// Column copy of a tensor derived from its MXFP8 row copy (see quantize_kernel, MXSRC).
hipError_t launch_requantize_colwise(const uint8_t *q_row, const uint8_t *s_row, int64_t rows, int64_t cols, uint8_t *q_colT,
                                     uint8_t *s_colT, bool tiled_scales, hipStream_t stream)
{
    const int64_t tiles_x = (cols + kTile - 1) / kTile, tiles_y = (rows + kTile - 1) / kTile;
    if (tiles_x * tiles_y > 0x7FFFFFFF)
        return hipErrorInvalidConfiguration;
    const dim3 grid((unsigned)(tiles_x * tiles_y)), block(kQuantThreads);
    uint8_t *none = nullptr;
    if (tiled_scales)
        hipLaunchKernelGGL((quantize_kernel<false, false, true, true, 0, true>), grid, block, 0, stream, q_row, rows, cols, cols, none,
                           none, q_colT, s_colT, (uint32_t)tiles_x, (uint32_t)(tiles_x * tiles_y), s_row);
    else
        hipLaunchKernelGGL((quantize_kernel<false, false, true, false, 0, true>), grid, block, 0, stream, q_row, rows, cols, cols, none,
                           none, q_colT, s_colT, (uint32_t)tiles_x, (uint32_t)(tiles_x * tiles_y), s_row);
    return hipGetLastError();
}

hipError_t launch_quantize(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis,
                           uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, bool tiled_scales,
                           int mode, hipStream_t stream)
{
    switch (mode) {
    case 1: return launch_quantize_mode<1>(src, bf16, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, tiled_scales, stream);
    case 2: return launch_quantize_mode<2>(src, bf16, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, tiled_scales, stream);
    case 3: return launch_quantize_mode<3>(src, bf16, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, tiled_scales, stream);
    default: return launch_quantize_mode<0>(src, bf16, rows, cols, ld, axis, q_row, s_row, q_colT, s_colT, tiled_scales, stream);
    }
}

}  // namespace mxfp8
