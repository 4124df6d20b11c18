/*
 * mxfp8.h -- C ABI of the MXFP8 linear-layer path for AMD MI355X (gfx950 / CDNA4).
 *
 * The library implements, as hand-written HIP kernels, the three operations a linear layer
 * needs when it is trained with the MXFP8 recipe:
 *
 *   quantize    a FP32/BF16 tensor -> blocks of K = 32 E4M3 elements Q_i sharing one UE8M0
 *               power-of-two scale X (Section 2; conversion rule of Section 3.3, Algorithm 1 and
 *               Appendix A.1/A.2: X = amax/448 rounded UP to a power of two, Q_i = RNE(V_i / X),
 *               saturating), along rows, along columns, or both from one read of the source
 *               (Section 3.2: every tensor is kept in two copies, one per reduction axis);
 *   gemm        the block-scaled matrix product with FP32 accumulation for the forward pass,
 *               the activation-gradient pass and the weight-gradient pass (Section 2,
 *               Section 3.2 / Figure 2, Appendix A.3), on the scaled MX MFMA instructions;
 *   dequantize  the decode Q_i * X (Section 2).
 *
 * Around these three, each declared below with the passage it serves: the same calls with the scale bytes in a
 * tiled layout and a bound on the workgroups (_ex); the product that also emits the MXFP8 copies of its output;
 * E5M2 elements and the OCP v1 scale rule of the paper's ablations (_mode_ex, for quantize, dequantize and the
 * product); the BF16 product of the simulated path; grouped products for mixture-of-experts layers; the column
 * copy derived from a kept row copy; the MXFP4 and MXFP6 members of Table 1; and measurement aids.
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers (HIP global memory of the current device). The
 *     caller owns every buffer; the library allocates nothing, keeps no state between calls and
 *     never synchronises: work is enqueued on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and the call returns immediately.
 *   - All tensors are row-major. "ld" arguments are leading dimensions in ELEMENTS.
 *   - A block is 32 consecutive elements along the quantization axis, so that axis must be a
 *     multiple of 32 (the paper defines no partial block); the quantizer works on tiles made of
 *     whole blocks in both directions and asks for both dimensions to be multiples of 32,
 *     whichever axis is selected. A dimension of 0 is accepted and does nothing.
 *   - Scale bytes hold n + 127 for X = 2^n, n in [-127, 127]; 0xFF marks a NaN block.
 *     Element bytes are OCP E4M3 (bias 7, max 448, 0x7F/0xFF = NaN, no infinity).
 *   - Errors are reported by return code only, detected on the host before any launch; when a
 *     call fails no output byte has been written. MXFP8_ERR_HIP means the launch itself was
 *     rejected by the runtime (the HIP error stays readable through hipGetLastError()).
 *   - The code objects are built for gfx950 only: on any other device the launch is rejected and
 *     the call returns MXFP8_ERR_HIP.
 */
#ifndef MXFP8_H
#define MXFP8_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MXFP8_OK = 0,
    MXFP8_ERR_NULL = 1,  /* a required pointer is NULL */
    MXFP8_ERR_SHAPE = 2, /* negative dimension, axis not a multiple of 32, ld too small */
    MXFP8_ERR_ALIGN = 3, /* pointer or leading dimension not aligned as documented */
    MXFP8_ERR_DTYPE = 4, /* unknown mxfp8_dtype */
    MXFP8_ERR_MODE = 5,  /* unknown axis / pass / scale layout / element / scale rule, negative workgroup bound */
    MXFP8_ERR_HIP = 6    /* kernel launch rejected by the HIP runtime, or not a gfx950 device */
} mxfp8_status;

typedef enum { MXFP8_F32 = 0, MXFP8_BF16 = 1 } mxfp8_dtype;
typedef enum { MXFP8_ROWWISE = 1, MXFP8_COLWISE = 2, MXFP8_BOTH = 3 } mxfp8_axis;
typedef enum { MXFP8_FPROP = 0, MXFP8_DGRAD = 1, MXFP8_WGRAD = 2 } mxfp8_pass;

/*
 * How the scale bytes of a quantized [rows x cols] operand (nb = cols/32 blocks per row) are stored.
 * The paper fixes the values, not their place in memory; both layouts hold the same bytes.
 *   MXFP8_SCALES_ROWMAJOR  s[r * nb + b]: dense [rows x nb]. What the plain entry points use.
 *   MXFP8_SCALES_TILED     s[((r/64 * ceil(nb/4) + b/4) * 64 + r%64) * 4 + b%4]: the four scale bytes
 *                          that one 128-wide K step of the GEMM needs for a row form a dword, and the
 *                          dwords of 64 consecutive rows are contiguous (256 bytes), so both the
 *                          quantizer's scale stores and the GEMM's scale loads move whole cache lines
 *                          instead of 4 bytes per line. The buffer holds ceil(rows/64) * ceil(nb/4)
 *                          * 256 bytes (mxfp8_scale_bytes); bytes that belong to rows >= rows or
 *                          blocks >= nb are unspecified filler. Must be 16-byte aligned.
 */
typedef enum { MXFP8_SCALES_ROWMAJOR = 0, MXFP8_SCALES_TILED = 1 } mxfp8_scale_layout;

/*
 * The two choices of the conversion that the paper studies as ablations. The recipe, and every entry point
 * without these arguments, is MXFP8_E4M3 with MXFP8_SCALE_ROUND_UP.
 *   mxfp8_element     MXFP8_E4M3: 1-4-3, bias 7, max 448 (Table 1). MXFP8_E5M2: 1-5-2, bias 15, max 57344,
 *                     IEEE-style Inf/NaN codes (Table 1; Section 3.2.2 compares the two per tensor role).
 *   mxfp8_scale_rule  MXFP8_SCALE_ROUND_UP: X = amax / max rounded UP to a power of two (Algorithm 1,
 *                     Appendix A.1): no element of a finite block exceeds the FP8 maximum.
 *                     MXFP8_SCALE_OCP_V1: X = 2^(floor(log2(amax)) - emax), i.e. rounded DOWN (the OCP v1.0
 *                     suggestion that Section 3.3 replaces): elements of a block whose amax has a
 *                     significand above 1.75 exceed the maximum and saturate to +-max.
 */
typedef enum { MXFP8_E4M3 = 0, MXFP8_E5M2 = 1 } mxfp8_element;
typedef enum { MXFP8_SCALE_ROUND_UP = 0, MXFP8_SCALE_OCP_V1 = 1 } mxfp8_scale_rule;

/* Size in bytes of the scale buffer of a [rows x cols] operand in `layout` (host arithmetic only);
 * -1 for negative sizes, sizes beyond 2^31 - 1, cols not a multiple of 32 or an unknown layout. */
int64_t mxfp8_scale_bytes(int64_t rows, int64_t cols, mxfp8_scale_layout layout);

/*
 * Convert src [rows x cols] (FP32 or BF16, leading dimension ld_src >= cols) to MXFP8-E4M3.
 * Section 3.3 / Algorithm 1 / Appendix A.1 (scale), Appendix A.2 (elements), Section 3.2 (axes).
 *
 *   MXFP8_ROWWISE  blocks are 32 consecutive columns of a row:
 *                    q_row [rows x cols] bytes, s_row [rows x cols/32] bytes.
 *   MXFP8_COLWISE  blocks are 32 consecutive rows of a column; the copy is stored TRANSPOSED so
 *                  that each block is again contiguous:
 *                    q_colT [cols x rows] bytes, s_colT [cols x rows/32] bytes.
 *   MXFP8_BOTH     both copies, each computed from the source itself, in one pass over src.
 *
 * Requirements: rows % 32 == 0 and cols % 32 == 0; src 16-byte aligned and ld_src a multiple
 * of 16 bytes; q_row and q_colT 16-byte aligned. Outputs not selected by `axis` are ignored and
 * may be NULL. Outputs are dense (leading dimension = their column count) and must not overlap src.
 *
 * Special values (the paper asks for "special care" without fixing it): a block containing a NaN
 * gets scale 0xFF and all elements 0x7F; a block containing +-Inf and no NaN gets scale 254
 * (Algorithm 1's clamp), its infinities saturate to +-448 and its finite values are divided by
 * 2^127; the sign of every input, zero included, is kept.
 */
mxfp8_status mxfp8_quantize(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                            int64_t ld_src, mxfp8_axis axis, uint8_t *q_row, uint8_t *s_row,
                            uint8_t *q_colT, uint8_t *s_colT, void *hip_stream);

/* mxfp8_quantize with the scale bytes of both copies stored in `scale_layout` (s_row describes the
 * [rows x cols] operand, s_colT the transposed [cols x rows] one). Same values, same requirements;
 * tiled scale buffers must be 16-byte aligned and sized by mxfp8_scale_bytes. */
mxfp8_status mxfp8_quantize_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                               int64_t ld_src, mxfp8_axis axis, uint8_t *q_row, uint8_t *s_row,
                               uint8_t *q_colT, uint8_t *s_colT, mxfp8_scale_layout scale_layout,
                               void *hip_stream);

/* mxfp8_quantize_ex with the element format and the scale rule chosen by the caller (Table 1; Section 3.2.2;
 * Section 3.3 with Figure 4's comparison arm). Same layouts, requirements and special-value rules; values that
 * round beyond the largest finite code saturate to it with the sign of the input (Appendix A.2), infinities
 * included; a block with a NaN gets scale 0xFF and all elements 0x7F in either format. Unknown element or
 * rule: MXFP8_ERR_MODE. */
mxfp8_status mxfp8_quantize_mode_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                                    int64_t ld_src, mxfp8_axis axis, mxfp8_element element, mxfp8_scale_rule rule,
                                    uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                                    mxfp8_scale_layout scale_layout, void *hip_stream);

/*
 * C [M x N] = A [M x K] * B [N x K]^T with per-block scales (Section 2, Appendix A.3):
 *   C[m, n] = sum over blocks b of 2^(a_s[m,b] + b_s[n,b] - 254) * sum_{i<32} A[m,32b+i] * B[n,32b+i]
 * accumulated in FP32 by the scaled MFMA instructions. Both operands are K-contiguous MXFP8:
 * a_q [M x K], a_s [M x K/32], b_q [N x K], b_s [N x K/32] (dense).
 *
 * `pass` names which of the three products of a linear layer this is (Section 3.2, Figure 2),
 * i.e. which quantized copies the caller passes; the arithmetic is the same for all three:
 *   MXFP8_FPROP  Y  [T x O] : A = X_row  [T x H], B = W_row  [O x H]   (reduction over H)
 *   MXFP8_DGRAD  dX [T x H] : A = dY_row [T x O], B = W_colT [H x O]   (reduction over O)
 *   MXFP8_WGRAD  dW [O x H] : A = dY_colT[O x T], B = X_colT [H x T]   (reduction over T)
 *
 * c is FP32 or BF16 (rounded to nearest even from the FP32 accumulator), leading dimension
 * ldc >= N. Requirements: K % 128 == 0 (one scaled MFMA consumes four blocks); a_q, b_q, a_s, b_s
 * 16-byte aligned; c aligned to its element size. When c is 16-byte aligned and
 * ldc * sizeof(element) is a multiple of 16 the result is written with 128-bit stores, otherwise
 * element by element (slower, same values). M and N are arbitrary up to 2^30 with at most 2^31 - 1
 * tiles of 128 x 128 in C, K up to 2^24 (larger shapes return MXFP8_ERR_SHAPE); M, N or K equal to
 * 0 is accepted (K == 0 stores zeros).
 * A scale byte 0xFF or an element NaN makes every output it touches NaN; products that overflow
 * FP32 give +-Inf or NaN as the hardware accumulator does.
 */
mxfp8_status mxfp8_gemm(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s,
                        const uint8_t *b_q, const uint8_t *b_s, int64_t M, int64_t N, int64_t K,
                        void *c, mxfp8_dtype c_dtype, int64_t ldc, void *hip_stream);

/* mxfp8_gemm with a_s and b_s both stored in `scale_layout` (Section 2, Appendix A.3: same sum), on at
 * most `max_workgroups` compute units. Problems made of full output tiles (M and N multiples of 256, or of
 * 128 when ceil(M/256)*ceil(N/256) < 128; K >= 256; c 16-byte aligned with ldc*sizeof(element) a multiple
 * of 16) run as one resident workgroup per compute unit that walks over its share of the tiles;
 * max_workgroups > 0 caps the number of those workgroups, e.g. to leave compute units to a kernel that
 * runs beside the product, max_workgroups == 0 takes every compute unit of the current device, a negative
 * value returns MXFP8_ERR_MODE. Other shapes take one workgroup per tile and ignore the bound. The result
 * does not depend on it. */
mxfp8_status mxfp8_gemm_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s,
                           const uint8_t *b_q, const uint8_t *b_s, int64_t M, int64_t N, int64_t K,
                           void *c, mxfp8_dtype c_dtype, int64_t ldc, mxfp8_scale_layout scale_layout,
                           int32_t max_workgroups, void *hip_stream);

/* mxfp8_gemm_ex with the element format of each operand chosen by the caller (Table 1; Section 3.2.2 compares E4M3
 * and E5M2 for weights, activations and gradients): a_q holds a_element codes, b_q b_element codes, as
 * mxfp8_quantize_mode_ex writes them; the same sum with the other decode table. E5M2 has Inf and NaN codes (the
 * quantizer never writes them): they propagate as in IEEE arithmetic. Unknown element: MXFP8_ERR_MODE. */
mxfp8_status mxfp8_gemm_mode_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, mxfp8_element a_element,
                                const uint8_t *b_q, const uint8_t *b_s, mxfp8_element b_element, int64_t M,
                                int64_t N, int64_t K, void *c, mxfp8_dtype c_dtype, int64_t ldc,
                                mxfp8_scale_layout scale_layout, int32_t max_workgroups, void *hip_stream);

/*
 * Single-copy storage (Section 5 names the two stored copies per tensor as the overhead to remove): keep
 * only the row copy of a tensor and derive the column copy from it when the backward pass needs it. Every
 * element of q_row [rows x cols] / s_row is decoded exactly (Q_i * X) and the decoded tensor is quantized along
 * its columns exactly as mxfp8_quantize_ex(MXFP8_COLWISE) would quantize an FP32 source holding those values:
 *   q_colT [cols x rows], s_colT = scales of the transposed copy (mxfp8_scale_bytes(cols, rows, layout)).
 * The result differs from the column copy of the ORIGINAL tensor by one more rounding (values that the row
 * copy represents exactly come out identical). s_row and s_colT are in `scale_layout`. Requirements: rows % 32
 * == 0, cols % 32 == 0, q_row and q_colT 16-byte aligned, nothing overlaps. A 0xFF scale or NaN code in the row
 * copy makes the column blocks it touches NaN blocks.
 */
mxfp8_status mxfp8_requantize_colwise_ex(const uint8_t *q_row, const uint8_t *s_row, int64_t rows, int64_t cols,
                                         uint8_t *q_colT, uint8_t *s_colT, mxfp8_scale_layout scale_layout,
                                         void *hip_stream);

/*
 * Grouped products for mixture-of-experts layers (Appendix A.4: the recipe applies unchanged to the expert
 * GEMMs). Tokens are sorted by expert: tokens [group_ends[e-1], group_ends[e]) (from 0 for e = 0) belong to
 * expert e. group_ends is a DEVICE array of `groups` int32 (token counts come from the router on the GPU;
 * nothing is copied back): non-decreasing, the last at most the number of tokens. The library cannot check
 * its contents: ends are clamped to [previous end, number of tokens] on the device so that no access leaves
 * a buffer, but ends that break the alignment rules below give undefined values. An expert may be empty.
 *
 * MXFP8_FPROP (A = X_row, B_e = W_e_row) and MXFP8_DGRAD (A = dY_row, B_e = W_e_colT): tokens are the M rows of A,
 *   a_q [M x K], a_s            one operand, as in mxfp8_gemm_ex
 *   b_q [groups x N x K]        expert e's operand starts N*K bytes after expert e-1's
 *   b_s                         expert e's scales start mxfp8_scale_bytes(N, K, scale_layout) bytes after e-1's
 *   c   [M x N], ldc            C[m, :] = A[m, :] . B_e^T for the expert e that owns row m; rows at or beyond
 *                               group_ends[groups-1] are not written.
 *   With MXFP8_SCALES_TILED every end must be a multiple of 64 (the scale layout's row group). Requirements:
 *   N % 128 == 0, K % 128 == 0, K >= 256; c 16-byte aligned, ldc * sizeof(element) a multiple of 16. One resident
 *   workgroup per compute unit (at most max_workgroups if positive) walks over the tiles; the result does
 *   not depend on that number.
 * MXFP8_WGRAD (A = dY_colT [M x K], B = X_colT [N x K]): tokens are the reduction axis K of both operands,
 *   every end must be a multiple of 128 (whole K steps; ends in between are cut down to one), and each expert
 *   gets its own product over its own tokens:
 *   c   [groups x M x N]        dW_e starts M*ldc elements after dW_(e-1); an expert without tokens gets zeros.
 *   Requirements: K % 128 == 0; c aligned to its element size (128-bit stores when c is 16-byte aligned and
 *   ldc * sizeof(element) and M * ldc * sizeof(element) are multiples of 16). One workgroup per expert and tile;
 *   max_workgroups is ignored.
 * All passes: groups <= 4096; a_q, a_s, b_q, b_s 16-byte aligned, group_ends 4-byte aligned.
 */
mxfp8_status mxfp8_gemm_grouped_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s,
                                   const uint8_t *b_q, const uint8_t *b_s, const int32_t *group_ends,
                                   int32_t groups, int64_t M, int64_t N, int64_t K, void *c,
                                   mxfp8_dtype c_dtype, int64_t ldc, mxfp8_scale_layout scale_layout,
                                   int32_t max_workgroups, void *hip_stream);

/*
 * The GEMM of the simulated MX path (Section 3.1: the paper's own training runs convert every BF16 GEMM
 * input to MXFP8 and straight back to BF16 and then run an ordinary BF16 GEMM):
 *   C[m, n] = sum_k A[m, k] * B[n, k],  A [M x K] and B [N x K] dense BF16, both K-contiguous,
 * accumulated in FP32 by the BF16 matrix instructions (every product of two BF16 values is exact in FP32).
 * The round trip itself is mxfp8_quantize followed by mxfp8_dequantize to BF16 of the copy that the pass
 * uses (the operand table of mxfp8_gemm), so that "quantize -> dequantize -> mxfp8_gemm_bf16" and
 * "quantize -> mxfp8_gemm" compute the same sums and differ only in how the hardware adds them.
 * c is FP32 or BF16 (RNE), leading dimension ldc >= N. Requirements: K % 64 == 0 and K <= 2^23; a_bf16 and
 * b_bf16 16-byte aligned; c, ldc, max_workgroups, zero sizes and the NaN / overflow behaviour as in
 * mxfp8_gemm_ex.
 */
mxfp8_status mxfp8_gemm_bf16(const void *a_bf16, const void *b_bf16, int64_t M, int64_t N, int64_t K,
                             void *c, mxfp8_dtype c_dtype, int64_t ldc, int32_t max_workgroups,
                             void *hip_stream);

/*
 * mxfp8_gemm_ex with BF16 output AND, from the same pass, MXFP8 copies of that output, i.e. the next
 * layer's operands (Section 2: the FP32 result is re-quantized when it is needed in MX format;
 * Section 3.2 for the two axes; Section 3.3, Appendix A.1/A.2 for the conversion). c_bf16 [M x N] is the
 * accumulator rounded to BF16 (RNE); the copies selected by `axis` are exactly what
 * mxfp8_quantize_ex(c_bf16, BF16, M, N, ldc, axis, ...) would give:
 *   cq_row  [M x N], cs_row  = scales of C   as an [M x N] operand (mxfp8_scale_bytes(M, N, layout))
 *   cq_colT [N x M], cs_colT = scales of C^T as an [N x M] operand (mxfp8_scale_bytes(N, M, layout))
 * Outputs not selected by `axis` are ignored and may be NULL. Requirements beyond mxfp8_gemm_ex: M and N
 * multiples of the output tile (256 when ceil(M/256)*ceil(N/256) >= 128, else 128), K >= 256, c_bf16
 * 16-byte aligned with ldc*2 a multiple of 16, every selected output 16-byte aligned; anything else
 * returns MXFP8_ERR_SHAPE / MXFP8_ERR_ALIGN. max_workgroups as in mxfp8_gemm_ex.
 */
mxfp8_status mxfp8_gemm_quantize_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s,
                                    const uint8_t *b_q, const uint8_t *b_s, int64_t M, int64_t N, int64_t K,
                                    void *c_bf16, int64_t ldc, mxfp8_axis axis, uint8_t *cq_row,
                                    uint8_t *cs_row, uint8_t *cq_colT, uint8_t *cs_colT,
                                    mxfp8_scale_layout scale_layout, int32_t max_workgroups, void *hip_stream);

/*
 * Decode q [rows x cols], s [rows x cols/32] (dense, blocks along a row) to
 * dst[r, c] = E4M3(q[r, c]) * 2^(s[r, c/32] - 127) (Section 2), FP32 or BF16, leading dimension
 * ld_dst >= cols. The product is rounded once to the destination type (exact in FP32 unless it
 * overflows to +-Inf); scale 0xFF or element 0x7F/0xFF gives NaN.
 * Requirements: cols % 32 == 0; q and dst 16-byte aligned; ld_dst * sizeof(element) a multiple
 * of 16. A colwise copy is decoded by passing q_colT/s_colT with rows and cols swapped.
 */
mxfp8_status mxfp8_dequantize(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols,
                              void *dst, mxfp8_dtype dst_dtype, int64_t ld_dst, void *hip_stream);

/* mxfp8_dequantize with s stored in `scale_layout` (Section 2). */
mxfp8_status mxfp8_dequantize_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols,
                                 void *dst, mxfp8_dtype dst_dtype, int64_t ld_dst,
                                 mxfp8_scale_layout scale_layout, void *hip_stream);

/* mxfp8_dequantize_ex for element bytes in `element` format (Section 2 decode; Table 1): E5M2 codes 0x7C / 0xFC
 * decode to +-Inf, 0x7D..0x7F / 0xFD..0xFF to NaN. */
mxfp8_status mxfp8_dequantize_mode_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols,
                                      mxfp8_element element, void *dst, mxfp8_dtype dst_dtype, int64_t ld_dst,
                                      mxfp8_scale_layout scale_layout, void *hip_stream);

/*
 * MXFP4 (Table 1: E2M1 elements, largest magnitude 6, 32-element blocks with a UE8M0 scale), the narrower
 * format of the family that the conversion of Section 3.3 / Algorithm 1 / Appendix A.1 and A.2 covers with
 * other constants: X = 2^n for the smallest n with amax <= 6 * 2^n (clamped to [-127, 127]), Q_i = V_i / X
 * rounded to the nearest of 0, 0.5, 1, 1.5, 2, 3, 4, 6 (ties to the code with an even mantissa bit), saturating
 * at +-6, sign kept. Two elements per byte: element 2k of a block in the low nibble of byte k, element 2k + 1
 * in the high nibble (code = sign << 3 | exponent << 1 | mantissa).
 *   MXFP8_ROWWISE   q_row  [rows x cols/2] bytes, s_row  [rows x cols/32] bytes
 *   MXFP8_COLWISE   q_colT [cols x rows/2] bytes, s_colT [cols x rows/32] bytes  (stored transposed)
 *   MXFP8_BOTH      both, each from the source itself.
 * Scale bytes are in `scale_layout`, sized by mxfp8_scale_bytes as for MXFP8. Requirements as for
 * mxfp8_quantize_ex: rows % 32 == 0, cols % 32 == 0, src 16-byte aligned with ld_src a multiple of 16 bytes,
 * q_row and q_colT 16-byte aligned, nothing overlaps. E2M1 has neither NaN nor Inf: a block with a NaN gets
 * scale 0xFF and all codes 0 (the scale alone marks it), a block with +-Inf and no NaN gets scale 254, its
 * infinities become +-6 and its finite values are divided by 2^127 (they round to +-0).
 */
mxfp8_status mxfp8_fp4_quantize_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                                   int64_t ld_src, mxfp8_axis axis, uint8_t *q_row, uint8_t *s_row,
                                   uint8_t *q_colT, uint8_t *s_colT, mxfp8_scale_layout scale_layout,
                                   void *hip_stream);

/* dst[r, c] = E2M1(code(r, c)) * 2^(s[r, c/32] - 127) for an MXFP4 operand q [rows x cols/2], s (Section 2:
 * value = X * P_i). dst is FP32 or BF16 with leading dimension ld_dst >= cols; every decoded value is exact in
 * BF16 unless it lies below 2^-133 or above the format's range (then RNE / +-Inf as the conversion gives).
 * A 0xFF scale decodes to NaN. Requirements: cols % 32 == 0; q and dst 16-byte aligned, ld_dst a multiple of
 * 16 bytes. */
mxfp8_status mxfp8_fp4_dequantize_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                                     mxfp8_dtype dst_dtype, int64_t ld_dst, mxfp8_scale_layout scale_layout,
                                     void *hip_stream);

/*
 * mxfp8_gemm_ex for MXFP4 operands (Table 1; the sum of Section 2 and Appendix A.3 with E2M1 elements):
 *   C[m, n] = sum over blocks b of 2^(a_s[m,b] + b_s[n,b] - 254) * sum_{i<32} A[m,32b+i] * B[n,32b+i]
 * with a_q [M x K/2], b_q [N x K/2] packed as mxfp8_fp4_quantize_ex writes them, a_s [M x K/32], b_s [N x K/32] in
 * `scale_layout`, FP32 accumulation on the 4-bit form of the scaled matrix instruction. `pass` only names the
 * operands (same table as mxfp8_gemm). Requirements: K % 256 == 0 (one K step of the kernels is 128 operand
 * bytes); everything else (alignment, ldc, zero sizes, limits, max_workgroups, NaN through a 0xFF scale) as in
 * mxfp8_gemm_ex. E2M1 has no NaN or Inf code: only a scale byte can make an output NaN.
 */
mxfp8_status mxfp8_fp4_gemm_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q,
                               const uint8_t *b_s, int64_t M, int64_t N, int64_t K, void *c, mxfp8_dtype c_dtype,
                               int64_t ldc, mxfp8_scale_layout scale_layout, int32_t max_workgroups,
                               void *hip_stream);

/*
 * MXFP6 (Table 1: E2M3 elements, largest magnitude 7.5, or E3M2 elements, largest magnitude 28; 32-element blocks
 * with a UE8M0 scale): the conversion of Section 3.3 / Algorithm 1 / Appendix A.1 and A.2 with those constants.
 * X = 2^n for the smallest n with amax <= destmax * 2^n (clamped to [-127, 127]), Q_i = V_i / X rounded to the
 * nearest representable value (ties to the code with an even mantissa), saturating at +-destmax, sign kept.
 * E3M2's smallest subnormal is 2^-4 (bias 3, two mantissa bits: the value Table 1's binade count implies).
 * Storage: the 32 six-bit codes of a block (sign << 5 | exponent << M | mantissa) form one little-endian 192-bit
 * string, code i in bits 6i .. 6i+5 = 24 bytes per block:
 *   MXFP8_ROWWISE   q_row  [rows x cols*3/4] bytes, s_row  [rows x cols/32] bytes
 *   MXFP8_COLWISE   q_colT [cols x rows*3/4] bytes, s_colT [cols x rows/32] bytes  (stored transposed)
 * Scale bytes in `scale_layout`, sized by mxfp8_scale_bytes. Requirements as for mxfp8_quantize_ex. Neither
 * format has a NaN or an Inf code: a block with a NaN gets scale 0xFF and all codes 0, a block with +-Inf and no
 * NaN gets scale 254, its infinities become +-destmax and its finite values are divided by 2^127.
 */
typedef enum { MXFP8_E2M3 = 0, MXFP8_E3M2 = 1 } mxfp8_fp6_element;

mxfp8_status mxfp8_fp6_quantize_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                                   int64_t ld_src, mxfp8_axis axis, mxfp8_fp6_element element, uint8_t *q_row,
                                   uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                                   mxfp8_scale_layout scale_layout, void *hip_stream);

/* dst[r, c] = value(code(r, c)) * 2^(s[r, c/32] - 127) for an MXFP6 operand q [rows x cols*3/4], s (Section 2:
 * value = X * P_i); dst FP32 or BF16 (every decoded value has at most 4 significant bits), leading dimension
 * ld_dst >= cols. A 0xFF scale decodes to NaN. cols % 32 == 0; q and dst 16-byte aligned, ld_dst a multiple of
 * 16 bytes. */
mxfp8_status mxfp8_fp6_dequantize_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols,
                                     mxfp8_fp6_element element, void *dst, mxfp8_dtype dst_dtype, int64_t ld_dst,
                                     mxfp8_scale_layout scale_layout, void *hip_stream);

/*
 * The product of MXFP6 operands: every E2M3 and every E3M2 value is also an E4M3 value, so q [rows x cols*3/4]
 * is expanded, exactly, to E4M3 bytes q_e4m3 [rows x cols]; together with the operand's UNCHANGED scale bytes
 * that is an MXFP8 operand, and mxfp8_gemm_ex of two such operands computes the MXFP6 sum of Section 2 /
 * Appendix A.3 (the two operands may use different 6-bit formats, or one may be a genuine MXFP8 operand).
 * cols % 32 == 0; q and q_e4m3 16-byte aligned, not overlapping.
 */
mxfp8_status mxfp8_fp6_expand_ex(const uint8_t *q, int64_t rows, int64_t cols, mxfp8_fp6_element element,
                                 uint8_t *q_e4m3, void *hip_stream);

/*
 * Measurement aid for benchmarks (no operation of the paper): `workgroups` workgroups of 4 wavefronts each
 * issue iterations * 64 independent scaled FP8 matrix instructions (16x16x128, 65536 flop each) on register
 * operands, without memory traffic, and then store one float per work-item to sink[workgroups * 256]
 * (device memory, 4-byte aligned, contents meaningless). Timing the call gives the matrix rate this GPU
 * sustains at whatever clock its power management settles on: workgroups * 4 * iterations * 64 * 65536 flop.
 * workgroups in [0, 2^20], iterations in [0, 2^24], else MXFP8_ERR_SHAPE; workgroups == 0 does nothing.
 */
mxfp8_status mxfp8_mfma_rate_probe(int32_t workgroups, int32_t iterations, float *sink, void *hip_stream);

/* mxfp8_mfma_rate_probe with the element width of the operands: 8 (E4M3, what the call above does) or 4 (E2M1, the
 * instruction form of the MXFP4 product; same flop count per instruction); anything else MXFP8_ERR_MODE. */
mxfp8_status mxfp8_mfma_rate_probe_ex(int32_t workgroups, int32_t iterations, int32_t element_bits, float *sink,
                                      void *hip_stream);

/*
 * Second measurement aid (no operation of the paper): copies `bytes` bytes from src to dst (device memory, both
 * 16-byte aligned, not overlapping, bytes a multiple of 16) with 128-bit streaming loads and stores on
 * `workgroups` workgroups of 256 work-items. mode 0 / 1: grid-stride with 4 / 8 units in flight per work-item;
 * mode 2: one contiguous slab per workgroup; mode 3 / 4: as mode 0 but dst is written in runs of 128 / 256 bytes that
 * lie far apart (consecutive runs go to 64 interleaved regions: dst ends up a permutation of src; bytes must be
 * a multiple of 64 runs), the write pattern of a transposed tile. Timing it gives the rate the memory system sustains for one read
 * and one write stream issued the way the quantizer issues its own: 2 * bytes per call.
 * workgroups in [1, 2^20], else MXFP8_ERR_SHAPE; an unknown mode is MXFP8_ERR_MODE; bytes == 0 does nothing.
 */
mxfp8_status mxfp8_copy_rate_probe(const void *src, void *dst, int64_t bytes, int32_t workgroups, int32_t mode,
                                   void *hip_stream);

/*
 * Third measurement aid (no operation of the paper): runs ONE scaled 16x16x128 matrix instruction per experiment
 * on registers taken straight from memory, so that tests can pin the operand layout the product kernels rely on.
 * Experiment x, lane l (0..63): operand registers a_regs / b_regs[(64 x + l) * 8 .. + 7] (dwords; with 4-bit
 * elements only the first four are used), scale registers a_scale_regs / b_scale_regs[64 x + l] (byte 0 is
 * used), zero accumulator; the lane's four result registers go to out[(64 x + l) * 4 .. + 3].
 * element_bits 8: both operands E4M3; 4: both E2M1; anything else MXFP8_ERR_MODE. experiments in [0, 65536].
 * a_regs, b_regs and out 16-byte aligned, the scale arrays 4-byte aligned; all device memory.
 */
mxfp8_status mxfp8_mfma_layout_probe(const void *a_regs, const void *b_regs, const int32_t *a_scale_regs,
                                     const int32_t *b_scale_regs, int32_t experiments, int32_t element_bits,
                                     float *out, void *hip_stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char *mxfp8_status_string(mxfp8_status status);

#ifdef __cplusplus
}
#endif
#endif /* MXFP8_H */
