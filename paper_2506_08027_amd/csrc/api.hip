// C ABI of the MXFP8 library: argument validation on the host, then one kernel launch on the
// caller's stream. Nothing is allocated, nothing is synchronised, no state is kept.
#include "../../include/mxfp8.h"

#include <hip/hip_runtime.h>

namespace mxfp8 {
hipError_t launch_quantize(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis,
                           uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, bool tiled_scales,
                           int mode, hipStream_t stream);
hipError_t launch_dequantize(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                             bool bf16, bool tiled_scales, bool e5m2, int64_t ld, hipStream_t stream);
hipError_t launch_gemm(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s, int64_t M,
                       int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc, int max_workgroups,
                       hipStream_t stream);
hipError_t launch_gemm_fused(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                             int64_t M, int64_t N, int64_t K, void *c, int64_t ldc, int axis, uint8_t *cq,
                             uint8_t *cs, uint8_t *cqT, uint8_t *csT, bool tiled_scales, int max_workgroups,
                             hipStream_t stream);
hipError_t launch_quantize_fp4(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis, uint8_t *q_row,
                               uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, bool tiled_scales, hipStream_t stream);
hipError_t launch_dequantize_fp4(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst, bool bf16,
                                 bool tiled_scales, int64_t ld, hipStream_t stream);
hipError_t launch_mfma_layout(const void *a, const void *b, const int *sa, const int *sb, int experiments, bool fp4, float *out,
                              hipStream_t stream);
hipError_t launch_gemm_fp4(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s, int64_t M,
                           int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc, int max_workgroups,
                           hipStream_t stream);
hipError_t launch_quantize_fp6(const void *src, bool bf16, int64_t rows, int64_t cols, int64_t ld, int axis, bool e3m2, uint8_t *q_row,
                               uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT, bool tiled_scales, hipStream_t stream);
hipError_t launch_dequantize_fp6(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, bool e3m2, void *dst, bool bf16,
                                 bool tiled, int64_t ld, hipStream_t stream);
hipError_t launch_expand_fp6(const uint8_t *q, int64_t rows, int64_t cols, bool e3m2, uint8_t *q8, hipStream_t stream);
hipError_t launch_gemm_elements(const uint8_t *a_q, const uint8_t *a_s, bool a_e5m2, const uint8_t *b_q, const uint8_t *b_s,
                                bool b_e5m2, int64_t M, int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc,
                                int max_workgroups, hipStream_t stream);
hipError_t launch_requantize_colwise(const uint8_t *q_row, const uint8_t *s_row, int64_t rows, int64_t cols, uint8_t *q_colT,
                                     uint8_t *s_colT, bool tiled_scales, hipStream_t stream);
hipError_t launch_gemm_grouped(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                               const int32_t *group_ends, int groups, int64_t b_group_bytes, int64_t bs_group_bytes,
                               int64_t M, int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc,
                               int max_workgroups, hipStream_t stream);
hipError_t launch_gemm_kgrouped(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                                const int32_t *group_ends, int groups, int64_t M, int64_t N, int64_t K, void *c, bool c_bf16,
                                bool tiled_scales, int64_t ldc, hipStream_t stream);
hipError_t launch_gemm_bf16(const uint8_t *a, const uint8_t *b, int64_t M, int64_t N, int64_t K, void *c, bool c_bf16,
                            int64_t ldc, int max_workgroups, hipStream_t stream);
hipError_t launch_mfma_rate(int workgroups, int iterations, bool fp4, float *sink, hipStream_t stream);
hipError_t launch_copy_rate(const void *src, void *dst, int64_t bytes, int workgroups, int mode, hipStream_t stream);
}  // namespace mxfp8

namespace {
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool valid_dtype(int d) { return d == MXFP8_F32 || d == MXFP8_BF16; }
inline bool valid_layout(int l) { return l == MXFP8_SCALES_ROWMAJOR || l == MXFP8_SCALES_TILED; }
inline int64_t esize(int d) { return d == MXFP8_BF16 ? 2 : 4; }
constexpr int64_t kMaxDim = 0x7FFFFFFF;  // kernels index rows and columns with 32-bit tile math
// GEMM: tile origins (multiples of up to 256 past M or N) stay in 32 bits, a lane's byte offset inside
// a 256-row operand tile (255 * K + 127) stays in 32 bits unsigned, and the grid (one workgroup per
// 128x128 tile at the finest) fits the launch
constexpr int64_t kMaxGemmMN = int64_t(1) << 30, kMaxGemmK = int64_t(1) << 24;
constexpr int32_t kMaxGroups = 4096;  // every tile lookup of the grouped product scans the group ends
}  // namespace

extern "C" {

int64_t mxfp8_scale_bytes(int64_t rows, int64_t cols, mxfp8_scale_layout layout)
{
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || cols % 32 || !valid_layout(layout))
        return -1;
    const int64_t nb = cols / 32;
    return layout == MXFP8_SCALES_TILED ? ((rows + 63) / 64) * ((nb + 3) / 4) * 256 : rows * nb;
}

mxfp8_status mxfp8_quantize(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                            int64_t ld_src, mxfp8_axis axis, uint8_t *q_row, uint8_t *s_row,
                            uint8_t *q_colT, uint8_t *s_colT, void *hip_stream)
{
    return mxfp8_quantize_ex(src, src_dtype, rows, cols, ld_src, axis, q_row, s_row, q_colT, s_colT,
                             MXFP8_SCALES_ROWMAJOR, hip_stream);
}

mxfp8_status mxfp8_quantize_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                               int64_t ld_src, mxfp8_axis axis, uint8_t *q_row, uint8_t *s_row,
                               uint8_t *q_colT, uint8_t *s_colT, mxfp8_scale_layout scale_layout,
                               void *hip_stream)
{
    return mxfp8_quantize_mode_ex(src, src_dtype, rows, cols, ld_src, axis, MXFP8_E4M3, MXFP8_SCALE_ROUND_UP, q_row, s_row,
                                  q_colT, s_colT, scale_layout, hip_stream);
}

mxfp8_status mxfp8_quantize_mode_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                                    int64_t ld_src, mxfp8_axis axis, mxfp8_element element, mxfp8_scale_rule rule,
                                    uint8_t *q_row, uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                                    mxfp8_scale_layout scale_layout, void *hip_stream)
{
    if (!valid_dtype(src_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || (element != MXFP8_E4M3 && element != MXFP8_E5M2) ||
        (rule != MXFP8_SCALE_ROUND_UP && rule != MXFP8_SCALE_OCP_V1))
        return MXFP8_ERR_MODE;
    if (axis != MXFP8_ROWWISE && axis != MXFP8_COLWISE && axis != MXFP8_BOTH)
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || rows % 32 || cols % 32 || ld_src < cols)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    const bool want_row = axis & MXFP8_ROWWISE, want_col = axis & MXFP8_COLWISE;
    if (!src || (want_row && (!q_row || !s_row)) || (want_col && (!q_colT || !s_colT)))
        return MXFP8_ERR_NULL;
    if (!aligned16(src) || (ld_src * esize(src_dtype)) % 16 || (want_row && !aligned16(q_row)) ||
        (want_col && !aligned16(q_colT)))
        return MXFP8_ERR_ALIGN;
    const bool tiled = scale_layout == MXFP8_SCALES_TILED;  // tiled scales are written as dwords
    if (tiled && ((want_row && !aligned16(s_row)) || (want_col && !aligned16(s_colT))))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_quantize(src, src_dtype == MXFP8_BF16, rows, cols, ld_src, (int)axis,
                                                q_row, s_row, q_colT, s_colT, tiled,
                                                (element == MXFP8_E5M2 ? 1 : 0) | (rule == MXFP8_SCALE_OCP_V1 ? 2 : 0),
                                                static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_requantize_colwise_ex(const uint8_t *q_row, const uint8_t *s_row, int64_t rows, int64_t cols,
                                         uint8_t *q_colT, uint8_t *s_colT, mxfp8_scale_layout scale_layout, void *hip_stream)
{
    if (!valid_layout(scale_layout))
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || rows % 32 || cols % 32)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    if (!q_row || !s_row || !q_colT || !s_colT)
        return MXFP8_ERR_NULL;
    if (!aligned16(q_row) || !aligned16(q_colT))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_requantize_colwise(q_row, s_row, rows, cols, q_colT, s_colT,
                                                          scale_layout == MXFP8_SCALES_TILED, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_gemm(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q,
                        const uint8_t *b_s, int64_t M, int64_t N, int64_t K, void *c, mxfp8_dtype c_dtype,
                        int64_t ldc, void *hip_stream)
{
    return mxfp8_gemm_ex(pass, a_q, a_s, b_q, b_s, M, N, K, c, c_dtype, ldc, MXFP8_SCALES_ROWMAJOR, 0, hip_stream);
}

mxfp8_status mxfp8_gemm_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q,
                           const uint8_t *b_s, int64_t M, int64_t N, int64_t K, void *c, mxfp8_dtype c_dtype,
                           int64_t ldc, mxfp8_scale_layout scale_layout, int32_t max_workgroups, void *hip_stream)
{
    if (!valid_dtype(c_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || max_workgroups < 0)
        return MXFP8_ERR_MODE;
    if (pass != MXFP8_FPROP && pass != MXFP8_DGRAD && pass != MXFP8_WGRAD)
        return MXFP8_ERR_MODE;
    if (M < 0 || N < 0 || K < 0 || M > kMaxGemmMN || N > kMaxGemmMN || K > kMaxGemmK || K % 128 || ldc < N ||
        ((M + 127) / 128) * ((N + 127) / 128) > kMaxDim)
        return MXFP8_ERR_SHAPE;
    if (M == 0 || N == 0)
        return MXFP8_OK;
    if (!c || (K > 0 && (!a_q || !a_s || !b_q || !b_s)))
        return MXFP8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(c) % esize(c_dtype) ||
        (K > 0 && (!aligned16(a_q) || !aligned16(a_s) || !aligned16(b_q) || !aligned16(b_s))))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_gemm(a_q, a_s, b_q, b_s, M, N, K, c, c_dtype == MXFP8_BF16,
                                            scale_layout == MXFP8_SCALES_TILED, ldc, max_workgroups,
                                            static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_gemm_mode_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, mxfp8_element a_element,
                                const uint8_t *b_q, const uint8_t *b_s, mxfp8_element b_element, int64_t M, int64_t N,
                                int64_t K, void *c, mxfp8_dtype c_dtype, int64_t ldc, mxfp8_scale_layout scale_layout,
                                int32_t max_workgroups, void *hip_stream)
{
    if (!valid_dtype(c_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || max_workgroups < 0 || (a_element != MXFP8_E4M3 && a_element != MXFP8_E5M2) ||
        (b_element != MXFP8_E4M3 && b_element != MXFP8_E5M2))
        return MXFP8_ERR_MODE;
    if (pass != MXFP8_FPROP && pass != MXFP8_DGRAD && pass != MXFP8_WGRAD)
        return MXFP8_ERR_MODE;
    if (M < 0 || N < 0 || K < 0 || M > kMaxGemmMN || N > kMaxGemmMN || K > kMaxGemmK || K % 128 || ldc < N ||
        ((M + 127) / 128) * ((N + 127) / 128) > kMaxDim)
        return MXFP8_ERR_SHAPE;
    if (M == 0 || N == 0)
        return MXFP8_OK;
    if (!c || (K > 0 && (!a_q || !a_s || !b_q || !b_s)))
        return MXFP8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(c) % esize(c_dtype) ||
        (K > 0 && (!aligned16(a_q) || !aligned16(a_s) || !aligned16(b_q) || !aligned16(b_s))))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_gemm_elements(a_q, a_s, a_element == MXFP8_E5M2, b_q, b_s, b_element == MXFP8_E5M2, M, N, K, c,
                                                     c_dtype == MXFP8_BF16, scale_layout == MXFP8_SCALES_TILED, ldc,
                                                     max_workgroups, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_gemm_grouped_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q,
                                   const uint8_t *b_s, const int32_t *group_ends, int32_t groups, int64_t M, int64_t N,
                                   int64_t K, void *c, mxfp8_dtype c_dtype, int64_t ldc, mxfp8_scale_layout scale_layout,
                                   int32_t max_workgroups, void *hip_stream)
{
    if (!valid_dtype(c_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || max_workgroups < 0 || (pass != MXFP8_FPROP && pass != MXFP8_DGRAD && pass != MXFP8_WGRAD))
        return MXFP8_ERR_MODE;
    const bool wgrad = pass == MXFP8_WGRAD;  // experts split the reduction axis; otherwise the rows of A
    if (groups < 0 || groups > kMaxGroups || M < 0 || N < 0 || K < 0 || M > kMaxGemmMN || N > kMaxGemmMN || K > kMaxGemmK ||
        K % 128 || ldc < N)
        return MXFP8_ERR_SHAPE;
    if (wgrad ? ((M + 127) / 128) * ((N + 127) / 128) * groups > kMaxDim
              : (K < 256 || N % 128 || ((M + 127) / 128 + groups) * ((N + 127) / 128) > kMaxDim))
        return MXFP8_ERR_SHAPE;
    if (M == 0 || N == 0 || groups == 0)
        return MXFP8_OK;
    if (!c || !group_ends || (K > 0 && (!a_q || !a_s || !b_q || !b_s)))
        return MXFP8_ERR_NULL;
    if ((K > 0 && (!aligned16(a_q) || !aligned16(a_s) || !aligned16(b_q) || !aligned16(b_s))) ||
        reinterpret_cast<uintptr_t>(group_ends) % 4)
        return MXFP8_ERR_ALIGN;
    if (wgrad ? reinterpret_cast<uintptr_t>(c) % esize(c_dtype) != 0 : (!aligned16(c) || (ldc * esize(c_dtype)) % 16))
        return MXFP8_ERR_ALIGN;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool tiled = scale_layout == MXFP8_SCALES_TILED;
    const hipError_t e =
        wgrad ? mxfp8::launch_gemm_kgrouped(a_q, a_s, b_q, b_s, group_ends, groups, M, N, K, c, c_dtype == MXFP8_BF16, tiled, ldc, stream)
              : mxfp8::launch_gemm_grouped(a_q, a_s, b_q, b_s, group_ends, groups, N * K, mxfp8_scale_bytes(N, K, scale_layout), M,
                                           N, K, c, c_dtype == MXFP8_BF16, tiled, ldc, max_workgroups, stream);
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_gemm_bf16(const void *a_bf16, const void *b_bf16, int64_t M, int64_t N, int64_t K, void *c,
                             mxfp8_dtype c_dtype, int64_t ldc, int32_t max_workgroups, void *hip_stream)
{
    if (!valid_dtype(c_dtype))
        return MXFP8_ERR_DTYPE;
    if (max_workgroups < 0)
        return MXFP8_ERR_MODE;
    // rows are walked in 128-byte steps of 64 values; 2 * K bytes per row must fit the kernels' 32-bit offsets
    if (M < 0 || N < 0 || K < 0 || M > kMaxGemmMN || N > kMaxGemmMN || K > kMaxGemmK / 2 || K % 64 || ldc < N ||
        ((M + 127) / 128) * ((N + 127) / 128) > kMaxDim)
        return MXFP8_ERR_SHAPE;
    if (M == 0 || N == 0)
        return MXFP8_OK;
    if (!c || (K > 0 && (!a_bf16 || !b_bf16)))
        return MXFP8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(c) % esize(c_dtype) || (K > 0 && (!aligned16(a_bf16) || !aligned16(b_bf16))))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_gemm_bf16(static_cast<const uint8_t *>(a_bf16), static_cast<const uint8_t *>(b_bf16),
                                                 M, N, K, c, c_dtype == MXFP8_BF16, ldc, max_workgroups,
                                                 static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_gemm_quantize_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q,
                                    const uint8_t *b_s, int64_t M, int64_t N, int64_t K, void *c_bf16, int64_t ldc,
                                    mxfp8_axis axis, uint8_t *cq_row, uint8_t *cs_row, uint8_t *cq_colT,
                                    uint8_t *cs_colT, mxfp8_scale_layout scale_layout, int32_t max_workgroups,
                                    void *hip_stream)
{
    if (!valid_layout(scale_layout) || max_workgroups < 0)
        return MXFP8_ERR_MODE;
    if (axis != MXFP8_ROWWISE && axis != MXFP8_COLWISE && axis != MXFP8_BOTH)
        return MXFP8_ERR_MODE;
    const bool want_row = axis & MXFP8_ROWWISE, want_col = axis & MXFP8_COLWISE;
    if (pass != MXFP8_FPROP && pass != MXFP8_DGRAD && pass != MXFP8_WGRAD)
        return MXFP8_ERR_MODE;
    if (M < 0 || N < 0 || K < 0 || M > kMaxGemmMN || N > kMaxGemmMN || K > kMaxGemmK || K % 128 || K < 256 || ldc < N ||
        M % 128 || N % 128 || ((M + 127) / 128) * ((N + 127) / 128) > kMaxDim)
        return MXFP8_ERR_SHAPE;
    if (M == 0 || N == 0)
        return MXFP8_OK;
    if (!c_bf16 || !a_q || !a_s || !b_q || !b_s || (want_row && (!cq_row || !cs_row)) ||
        (want_col && (!cq_colT || !cs_colT)))
        return MXFP8_ERR_NULL;
    if (!aligned16(c_bf16) || (ldc * 2) % 16 || !aligned16(a_q) || !aligned16(a_s) || !aligned16(b_q) ||
        !aligned16(b_s) || (want_row && (!aligned16(cq_row) || !aligned16(cs_row))) ||
        (want_col && (!aligned16(cq_colT) || !aligned16(cs_colT))))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_gemm_fused(a_q, a_s, b_q, b_s, M, N, K, c_bf16, ldc, (int)axis, cq_row, cs_row,
                                                  cq_colT, cs_colT, scale_layout == MXFP8_SCALES_TILED, max_workgroups,
                                                  static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidConfiguration)  // the chosen tile does not divide M and N: nothing was launched
        return MXFP8_ERR_SHAPE;
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_dequantize(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                              mxfp8_dtype dst_dtype, int64_t ld_dst, void *hip_stream)
{
    return mxfp8_dequantize_ex(q, s, rows, cols, dst, dst_dtype, ld_dst, MXFP8_SCALES_ROWMAJOR, hip_stream);
}

mxfp8_status mxfp8_dequantize_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                                 mxfp8_dtype dst_dtype, int64_t ld_dst, mxfp8_scale_layout scale_layout,
                                 void *hip_stream)
{
    return mxfp8_dequantize_mode_ex(q, s, rows, cols, MXFP8_E4M3, dst, dst_dtype, ld_dst, scale_layout, hip_stream);
}

mxfp8_status mxfp8_dequantize_mode_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols,
                                      mxfp8_element element, void *dst, mxfp8_dtype dst_dtype, int64_t ld_dst,
                                      mxfp8_scale_layout scale_layout, void *hip_stream)
{
    if (!valid_dtype(dst_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || (element != MXFP8_E4M3 && element != MXFP8_E5M2))
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || cols % 32 || ld_dst < cols)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    if (!q || !s || !dst)
        return MXFP8_ERR_NULL;
    if (!aligned16(q) || !aligned16(dst) || (ld_dst * esize(dst_dtype)) % 16)
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_dequantize(q, s, rows, cols, dst, dst_dtype == MXFP8_BF16,
                                                  scale_layout == MXFP8_SCALES_TILED, element == MXFP8_E5M2, ld_dst,
                                                  static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_fp4_quantize_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                                   int64_t ld_src, mxfp8_axis axis, uint8_t *q_row, uint8_t *s_row,
                                   uint8_t *q_colT, uint8_t *s_colT, mxfp8_scale_layout scale_layout,
                                   void *hip_stream)
{
    if (!valid_dtype(src_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || (axis != MXFP8_ROWWISE && axis != MXFP8_COLWISE && axis != MXFP8_BOTH))
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || rows % 32 || cols % 32 || ld_src < cols)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    const bool want_row = axis & MXFP8_ROWWISE, want_col = axis & MXFP8_COLWISE;
    if (!src || (want_row && (!q_row || !s_row)) || (want_col && (!q_colT || !s_colT)))
        return MXFP8_ERR_NULL;
    if (!aligned16(src) || (ld_src * esize(src_dtype)) % 16 || (want_row && !aligned16(q_row)) ||
        (want_col && !aligned16(q_colT)))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_quantize_fp4(src, src_dtype == MXFP8_BF16, rows, cols, ld_src, (int)axis, q_row, s_row,
                                                    q_colT, s_colT, scale_layout == MXFP8_SCALES_TILED,
                                                    static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_fp4_dequantize_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, void *dst,
                                     mxfp8_dtype dst_dtype, int64_t ld_dst, mxfp8_scale_layout scale_layout,
                                     void *hip_stream)
{
    if (!valid_dtype(dst_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout))
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || cols % 32 || ld_dst < cols)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    if (!q || !s || !dst)
        return MXFP8_ERR_NULL;
    if (!aligned16(q) || !aligned16(dst) || (ld_dst * esize(dst_dtype)) % 16)
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_dequantize_fp4(q, s, rows, cols, dst, dst_dtype == MXFP8_BF16,
                                                      scale_layout == MXFP8_SCALES_TILED, ld_dst,
                                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_fp4_gemm_ex(mxfp8_pass pass, const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q,
                               const uint8_t *b_s, int64_t M, int64_t N, int64_t K, void *c, mxfp8_dtype c_dtype,
                               int64_t ldc, mxfp8_scale_layout scale_layout, int32_t max_workgroups, void *hip_stream)
{
    if (!valid_dtype(c_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || max_workgroups < 0)
        return MXFP8_ERR_MODE;
    if (pass != MXFP8_FPROP && pass != MXFP8_DGRAD && pass != MXFP8_WGRAD)
        return MXFP8_ERR_MODE;
    if (M < 0 || N < 0 || K < 0 || M > kMaxGemmMN || N > kMaxGemmMN || K > kMaxGemmK || K % 256 || ldc < N ||
        ((M + 127) / 128) * ((N + 127) / 128) > kMaxDim)
        return MXFP8_ERR_SHAPE;
    if (M == 0 || N == 0)
        return MXFP8_OK;
    if (!c || (K > 0 && (!a_q || !a_s || !b_q || !b_s)))
        return MXFP8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(c) % esize(c_dtype) ||
        (K > 0 && (!aligned16(a_q) || !aligned16(a_s) || !aligned16(b_q) || !aligned16(b_s))))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_gemm_fp4(a_q, a_s, b_q, b_s, M, N, K, c, c_dtype == MXFP8_BF16,
                                                scale_layout == MXFP8_SCALES_TILED, ldc, max_workgroups,
                                                static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_fp6_quantize_ex(const void *src, mxfp8_dtype src_dtype, int64_t rows, int64_t cols,
                                   int64_t ld_src, mxfp8_axis axis, mxfp8_fp6_element element, uint8_t *q_row,
                                   uint8_t *s_row, uint8_t *q_colT, uint8_t *s_colT,
                                   mxfp8_scale_layout scale_layout, void *hip_stream)
{
    if (!valid_dtype(src_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || (axis != MXFP8_ROWWISE && axis != MXFP8_COLWISE && axis != MXFP8_BOTH) ||
        (element != MXFP8_E2M3 && element != MXFP8_E3M2))
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || rows % 32 || cols % 32 || ld_src < cols)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    const bool want_row = axis & MXFP8_ROWWISE, want_col = axis & MXFP8_COLWISE;
    if (!src || (want_row && (!q_row || !s_row)) || (want_col && (!q_colT || !s_colT)))
        return MXFP8_ERR_NULL;
    if (!aligned16(src) || (ld_src * esize(src_dtype)) % 16 || (want_row && !aligned16(q_row)) ||
        (want_col && !aligned16(q_colT)))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_quantize_fp6(src, src_dtype == MXFP8_BF16, rows, cols, ld_src, (int)axis,
                                                    element == MXFP8_E3M2, q_row, s_row, q_colT, s_colT,
                                                    scale_layout == MXFP8_SCALES_TILED, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_fp6_dequantize_ex(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols,
                                     mxfp8_fp6_element element, void *dst, mxfp8_dtype dst_dtype, int64_t ld_dst,
                                     mxfp8_scale_layout scale_layout, void *hip_stream)
{
    if (!valid_dtype(dst_dtype))
        return MXFP8_ERR_DTYPE;
    if (!valid_layout(scale_layout) || (element != MXFP8_E2M3 && element != MXFP8_E3M2))
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || cols % 32 || ld_dst < cols)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    if (!q || !s || !dst)
        return MXFP8_ERR_NULL;
    if (!aligned16(q) || !aligned16(dst) || (ld_dst * esize(dst_dtype)) % 16)
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_dequantize_fp6(q, s, rows, cols, element == MXFP8_E3M2, dst, dst_dtype == MXFP8_BF16,
                                                      scale_layout == MXFP8_SCALES_TILED, ld_dst,
                                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_fp6_expand_ex(const uint8_t *q, int64_t rows, int64_t cols, mxfp8_fp6_element element,
                                 uint8_t *q_e4m3, void *hip_stream)
{
    if (element != MXFP8_E2M3 && element != MXFP8_E3M2)
        return MXFP8_ERR_MODE;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim || cols % 32)
        return MXFP8_ERR_SHAPE;
    if (rows == 0 || cols == 0)
        return MXFP8_OK;
    if (!q || !q_e4m3)
        return MXFP8_ERR_NULL;
    if (!aligned16(q) || !aligned16(q_e4m3))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_expand_fp6(q, rows, cols, element == MXFP8_E3M2, q_e4m3,
                                                  static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_mfma_rate_probe(int32_t workgroups, int32_t iterations, float *sink, void *hip_stream)
{
    return mxfp8_mfma_rate_probe_ex(workgroups, iterations, 8, sink, hip_stream);
}

mxfp8_status mxfp8_mfma_rate_probe_ex(int32_t workgroups, int32_t iterations, int32_t element_bits, float *sink,
                                      void *hip_stream)
{
    if (element_bits != 8 && element_bits != 4)
        return MXFP8_ERR_MODE;
    if (workgroups < 0 || iterations < 0 || workgroups > (1 << 20) || iterations > (1 << 24))
        return MXFP8_ERR_SHAPE;
    if (workgroups == 0)
        return MXFP8_OK;
    if (!sink)
        return MXFP8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(sink) % 4)
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_mfma_rate(workgroups, iterations, element_bits == 4, sink,
                                                 static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_mfma_layout_probe(const void *a_regs, const void *b_regs, const int32_t *a_scale_regs,
                                     const int32_t *b_scale_regs, int32_t experiments, int32_t element_bits, float *out,
                                     void *hip_stream)
{
    if (element_bits != 8 && element_bits != 4)
        return MXFP8_ERR_MODE;
    if (experiments < 0 || experiments > (1 << 16))
        return MXFP8_ERR_SHAPE;
    if (experiments == 0)
        return MXFP8_OK;
    if (!a_regs || !b_regs || !a_scale_regs || !b_scale_regs || !out)
        return MXFP8_ERR_NULL;
    if (!aligned16(a_regs) || !aligned16(b_regs) || !aligned16(out) ||
        reinterpret_cast<uintptr_t>(a_scale_regs) % 4 || reinterpret_cast<uintptr_t>(b_scale_regs) % 4)
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_mfma_layout(a_regs, b_regs, a_scale_regs, b_scale_regs, experiments, element_bits == 4,
                                                   out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

mxfp8_status mxfp8_copy_rate_probe(const void *src, void *dst, int64_t bytes, int32_t workgroups, int32_t mode, void *hip_stream)
{
    if (mode < 0 || mode > 4)
        return MXFP8_ERR_MODE;
    if (bytes < 0 || bytes % 16 || workgroups < 1 || workgroups > (1 << 20) || (mode == 3 && bytes % (64 * 128)) ||
        (mode == 4 && bytes % (64 * 256)))
        return MXFP8_ERR_SHAPE;
    if (bytes == 0)
        return MXFP8_OK;
    if (!src || !dst)
        return MXFP8_ERR_NULL;
    if (!aligned16(src) || !aligned16(dst))
        return MXFP8_ERR_ALIGN;
    const hipError_t e = mxfp8::launch_copy_rate(src, dst, bytes, workgroups, mode, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP8_OK : MXFP8_ERR_HIP;
}

const char *mxfp8_status_string(mxfp8_status status)
{
    switch (status) {
    case MXFP8_OK: return "ok";
    case MXFP8_ERR_NULL: return "required pointer is NULL";
    case MXFP8_ERR_SHAPE: return "bad shape: negative, not a multiple of the block size, or leading dimension too small";
    case MXFP8_ERR_ALIGN: return "pointer or leading dimension not 16-byte aligned";
    case MXFP8_ERR_DTYPE: return "unknown element type";
    case MXFP8_ERR_MODE: return "unknown axis, pass, scale layout, element format or scale rule, or a negative workgroup bound";
    case MXFP8_ERR_HIP: return "HIP launch failed (is this a gfx950 device?)";
    }
    return "unknown status";
}

}  // extern "C"
