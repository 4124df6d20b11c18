// Block-scaled MXFP8 GEMM for gfx950: C[M x N] = A[M x K] * B[N x K]^T, both operands K-contiguous
// E4M3 with one UE8M0 scale per 32 elements of K, FP32 accumulation (Section 2, Appendix A.3).
// The same kernel serves the forward, activation-gradient and weight-gradient products of a
// linear layer (Section 3.2, Figure 2): the column-wise quantized copies are stored transposed,
// which makes every one of them a K-contiguous "NT" product.
//
// Instruction. v_mfma_scale_f32_16x16x128_f8f6f4 multiplies a 16x128 by a 128x16 FP8 tile and
// applies, per operand, one scale byte per row and per 32-wide K block. Register layout (found by
// one-hot probing on the hardware): lane l = 16*g + r holds row r of its operand; its eight
// dwords hold K = 16g..16g+15 followed by K = 64+16g..64+16g+15; the scale operand of lane
// (r, g) is the scale of row r for K block g (K = 32g..32g+31), taken from byte op_sel of the
// register. The result register v of lane (r, g) is D[4g + v][r].
// The kernel feeds B rows as the first operand and A rows as the second, so a lane ends up with
// four consecutive n of one m: the epilogue is one 128-bit store per 16x16 tile and lane.
//
// Tiling. A workgroup of WAVES_M x WAVES_N wavefronts computes a BM x BN tile of C, K in steps of
// 128 bytes. A and B tiles (and one dword of four scale bytes per row) are staged through LDS,
// double-buffered: the global loads of step k+1 are issued before the MFMAs of step k and
// written to the other buffer afterwards, one barrier per step. LDS rows are 128 bytes; the
// 16-byte chunk index is XORed with (row/2)%8 so that the 16 lanes of a fragment read hit 16
// different bank groups.
#include "mxfp8_device.h"

namespace mxfp8 {

constexpr int BK = 128;  // K bytes per step = 4 scale blocks = one MFMA

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_> struct GemmCfg {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wavefront tile
    static constexpr int TM = WM / 16, TN = WN / 16;            // MFMA tiles per wavefront
    static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES + 4 * (BM + BN);
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int A_LOADS = A_BYTES / 16 / THREADS, B_LOADS = B_BYTES / 16 / THREADS;
    static_assert(A_BYTES % (16 * THREADS) == 0 && B_BYTES % (16 * THREADS) == 0, "tile/threads");
    static_assert(BM <= THREADS * 4 && BN <= THREADS * 4, "scale loads");
};

// Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2. Renumber them so
// that consecutive logical ids run on the same XCD, then walk the tile grid in column panels of
// `PANEL` tiles so that the workgroups resident on one XCD share A rows and B rows in its L2.
__device__ __forceinline__ void tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n, int &tm,
                                              int &tn)
{
    constexpr int XCDS = 8;
    int lid = bid;
    const int full = (nblocks / XCDS) * XCDS;
    if (bid < full)
        lid = (bid % XCDS) * (nblocks / XCDS) + bid / XCDS;
    constexpr int PANEL = 8;
    const int per_panel = PANEL * tiles_m;
    const int panel = lid / per_panel;
    const int in_panel = lid - panel * per_panel;
    const int width = min(PANEL, tiles_n - panel * PANEL);
    tm = in_panel / width;
    tn = panel * PANEL + in_panel % width;
}

template <class Cfg, bool OUT_BF16>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_kernel(
    const uint8_t *__restrict__ a_q, const uint8_t *__restrict__ a_s, const uint8_t *__restrict__ b_q,
    const uint8_t *__restrict__ b_s, int M, int N, int K, uint8_t *__restrict__ c, int64_t ldc_bytes,
    int tiles_m, int tiles_n, bool vec_store)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int BM = Cfg::BM, BN = Cfg::BN, TM = Cfg::TM, TN = Cfg::TN;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
    const int r16 = lane & 15, g = lane >> 4;

    int tile_m, tile_n;
    tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int nkb = K / kBlock;  // scale bytes per row
    const int KT = K / BK;

    // ---- global -> register staging (coalesced: 8 lanes cover one 128-byte row segment) ------
    const int ld_chunk = tid & 7;
    const int ld_row = tid >> 3;
    constexpr int ROWS_PER_PASS = Cfg::THREADS / 8;
    uint4 ra[Cfg::A_LOADS], rb[Cfg::B_LOADS];
    uint32_t rsa = 0, rsb = 0;
    const uint8_t *a_src[Cfg::A_LOADS];
    const uint8_t *b_src[Cfg::B_LOADS];
#pragma unroll
    for (int i = 0; i < Cfg::A_LOADS; ++i) {
        const int row = min(m0 + ld_row + i * ROWS_PER_PASS, M - 1);  // clamp: ragged tiles re-read a valid row
        a_src[i] = a_q + (int64_t)row * K + ld_chunk * 16;
    }
#pragma unroll
    for (int i = 0; i < Cfg::B_LOADS; ++i) {
        const int row = min(n0 + ld_row + i * ROWS_PER_PASS, N - 1);
        b_src[i] = b_q + (int64_t)row * K + ld_chunk * 16;
    }
    const uint8_t *sa_src = a_s + (int64_t)min(m0 + tid, M - 1) * nkb;
    const uint8_t *sb_src = b_s + (int64_t)min(n0 + tid, N - 1) * nkb;

    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < Cfg::A_LOADS; ++i)
            ra[i] = *reinterpret_cast<const uint4 *>(a_src[i] + (int64_t)kt * BK);
#pragma unroll
        for (int i = 0; i < Cfg::B_LOADS; ++i)
            rb[i] = *reinterpret_cast<const uint4 *>(b_src[i] + (int64_t)kt * BK);
        if (tid < BM)
            rsa = *reinterpret_cast<const uint32_t *>(sa_src + kt * 4);
        if (tid < BN)
            rsb = *reinterpret_cast<const uint32_t *>(sb_src + kt * 4);
    };
    auto store_lds = [&](int buf) {
        uint8_t *base = lds + buf * Cfg::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < Cfg::A_LOADS; ++i) {
            const int row = ld_row + i * ROWS_PER_PASS;
            *reinterpret_cast<uint4 *>(base + row * BK + swz(row, ld_chunk) * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < Cfg::B_LOADS; ++i) {
            const int row = ld_row + i * ROWS_PER_PASS;
            *reinterpret_cast<uint4 *>(base + Cfg::A_BYTES + row * BK + swz(row, ld_chunk) * 16) = rb[i];
        }
        uint32_t *sc = reinterpret_cast<uint32_t *>(base + Cfg::A_BYTES + Cfg::B_BYTES);
        if (tid < BM)
            sc[tid] = rsa;
        if (tid < BN)
            sc[BM + tid] = rsb;
    };

    v4f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf) {
        const uint8_t *base = lds + buf * Cfg::STAGE_BYTES;
        const uint8_t *as_ = base;
        const uint8_t *bs_ = base + Cfg::A_BYTES;
        const uint32_t *sc = reinterpret_cast<const uint32_t *>(base + Cfg::A_BYTES + Cfg::B_BYTES);
        v8i fa[TM];
        int sa[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm * Cfg::WM + i * 16 + r16;
            const v4i lo = *reinterpret_cast<const v4i *>(as_ + row * BK + swz(row, g) * 16);
            const v4i hi = *reinterpret_cast<const v4i *>(as_ + row * BK + swz(row, 4 + g) * 16);
            fa[i] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            sa[i] = (int)(sc[row] >> (8 * g));
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int row = wn * Cfg::WN + j * 16 + r16;
            const v4i lo = *reinterpret_cast<const v4i *>(bs_ + row * BK + swz(row, g) * 16);
            const v4i hi = *reinterpret_cast<const v4i *>(bs_ + row * BK + swz(row, 4 + g) * 16);
            const v8i fb = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            const int sb = (int)(sc[BM + row] >> (8 * g));
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb, fa[i], acc[i][j], 0, 0, 0, sb,
                                                                             0, sa[i]);
        }
    };

    if (KT > 0) {
        load_global(0);
        store_lds(0);
    }
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more)
            load_global(kt + 1);
        compute(kt & 1);
        if (more)
            store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: lane (r16, g) of tile (i, j) holds C[m0w + 16i + r16][n0w + 16j + 4g + 0..3]
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * Cfg::WM + i * 16 + r16;
        if (m >= M)
            continue;
        uint8_t *crow = c + (int64_t)m * ldc_bytes;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * Cfg::WN + j * 16 + 4 * g;
            const v4f v = acc[i][j];
            if (vec_store && n + 3 < N) {
                if constexpr (OUT_BF16) {
                    v2bf p0 = {(__bf16)v[0], (__bf16)v[1]}, p1 = {(__bf16)v[2], (__bf16)v[3]};
                    *reinterpret_cast<uint2 *>(crow + (int64_t)n * 2) =
                        make_uint2(__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1));
                } else {
                    *reinterpret_cast<float4 *>(crow + (int64_t)n * 4) = make_float4(v[0], v[1], v[2], v[3]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n + e < N) {
                        if constexpr (OUT_BF16)
                            *reinterpret_cast<__bf16 *>(crow + (int64_t)(n + e) * 2) = (__bf16)v[e];
                        else
                            *reinterpret_cast<float *>(crow + (int64_t)(n + e) * 4) = v[e];
                    }
            }
        }
    }
}

template <class Cfg, bool OUT_BF16>
static hipError_t launch_cfg(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                             int M, int N, int K, void *c, int64_t ldc, hipStream_t stream)
{
    const int tiles_m = (M + Cfg::BM - 1) / Cfg::BM, tiles_n = (N + Cfg::BN - 1) / Cfg::BN;
    auto kern = gemm_kernel<Cfg, OUT_BF16>;
    const int64_t ldc_bytes = ldc * (OUT_BF16 ? 2 : 4);
    // 128-bit (FP32) / 64-bit (BF16) stores need every row start aligned; otherwise element stores
    const bool vec_store = (reinterpret_cast<uintptr_t>(c) % 16 == 0) && (ldc_bytes % 16 == 0);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(Cfg::THREADS), Cfg::LDS_BYTES, stream,
                       a_q, a_s, b_q, b_s, M, N, K, static_cast<uint8_t *>(c), ldc_bytes, tiles_m, tiles_n, vec_store);
    return hipGetLastError();
}

hipError_t launch_gemm(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s, int64_t M,
                       int64_t N, int64_t K, void *c, bool c_bf16, int64_t ldc, hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2>;
    using Small = GemmCfg<128, 128, 2, 2>;
    // Small problems cannot fill 256 compute units with 256x256 tiles.
    const bool big = ((M + 255) / 256) * ((N + 255) / 256) >= 128;
    if (big)
        return c_bf16 ? launch_cfg<Big, true>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, ldc, stream)
                      : launch_cfg<Big, false>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, ldc, stream);
    return c_bf16 ? launch_cfg<Small, true>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, ldc, stream)
                  : launch_cfg<Small, false>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, ldc, stream);
}

}  // namespace mxfp8
