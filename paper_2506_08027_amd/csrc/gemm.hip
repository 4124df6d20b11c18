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
// 128 bytes (= one MFMA, four scale blocks). A and B tiles and one dword of scale bytes per row
// and step go from global memory straight into LDS (global_load_lds_dword{,x4}: no staging
// registers), two LDS buffers per operand; the software pipeline is described at the step lambda
// of the kernel. LDS rows are 128 bytes; the 16-byte chunk index is XORed with (row/2)%8 so that
// the 16 lanes of a fragment read hit 16 different bank groups. A direct-to-LDS load writes lane l
// of a wavefront to LDS offset 16*l, so the swizzle is applied on the global side: each lane
// fetches the chunk that belongs at its slot.
//
// Other operand formats on the same kernels (GemmCfg's FMT): plain BF16 operands for the product of the
// simulated path (two 16x16x32 BF16 instructions per K step and tile pair, no scales), and MXFP4 operands
// (two E2M1 codes per byte: a 128-byte K step is 256 elements, i.e. two 4-bit scaled instructions and two scale
// dwords per row). With 4-bit elements the instruction takes dwords 0..3 only, lane (r, g) holds K =
// 32g..32g+31 of row r and its own scale byte applies to them (pinned on the hardware by a test that runs
// single instructions on registers taken from memory).
#include "mxfp8_device.h"

namespace mxfp8 {

constexpr int BK = 128;  // K bytes per step = 4 scale blocks = one MFMA
constexpr int kStageBytes = 4608;  // per-wavefront LDS area of the persistent kernel's epilogue (16 rows x (256 + 32) bytes)

// Operand formats. kFmtFp8: MXFP8 operands with their scale bytes (the method itself), 128 elements and 4 scale
// blocks per 128-byte K step. kFmtBf16: plain BF16 operands, 64 per K step, no scales (the product of the
// simulated path of Section 3.1). kFmtFp4: MXFP4 operands (Table 1), two E2M1 codes per byte: 256 elements and
// 8 scale blocks (two scale dwords per row) per K step. Everything about tiles, buffers, data requests and the
// schedule is counted in BYTES of a K-contiguous operand row and is the same for all three.
constexpr int kFmtFp8 = 0, kFmtBf16 = 1, kFmtFp4 = 2;
// A_E5M2 / B_E5M2 (kFmtFp8 only): the elements of that operand are E5M2 instead of E4M3 (Section 3.2.2 compares the
// two per tensor type); nothing but the format fields of the matrix instruction changes.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int FMT_ = kFmtFp8, bool A_E5M2_ = false, bool B_E5M2_ = false> struct GemmCfg {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int FMT = FMT_;
    static constexpr bool A_E5M2 = A_E5M2_, B_E5M2 = B_E5M2_, ALL_E4M3 = FMT_ == kFmtFp8 && !A_E5M2_ && !B_E5M2_;
    static_assert(FMT_ == kFmtFp8 || (!A_E5M2_ && !B_E5M2_), "element formats belong to the MXFP8 product");
    static constexpr bool SCALED = FMT_ != kFmtBf16;
    static constexpr int SDW = FMT_ == kFmtFp4 ? 2 : 1;     // scale dwords per operand row and K step
    static constexpr int SBLK = FMT_ == kFmtFp4 ? 16 : 32;  // operand bytes per scale block
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wavefront tile
    static constexpr int TM = WM / 16, TN = WN / 16;            // MFMA tiles per wavefront
    static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK;
    // LDS map: A[2] | B[2] | A scales[2] | B scales[2]; a scale buffer holds, for each of the SDW scale dwords of
    // a K step, one dword (4 scale bytes) per tile row: [dword][row][4]
    static constexpr int SA_BYTES = BM * 4 * SDW, SB_BYTES = BN * 4 * SDW;
    static constexpr int A_OFF = 0, B_OFF = 2 * A_BYTES, SA_OFF = B_OFF + 2 * B_BYTES, SB_OFF = SA_OFF + 2 * SA_BYTES;
    static constexpr int LDS_BYTES = SB_OFF + 2 * SB_BYTES;
    static constexpr int LDS_BYTES_PERSISTENT = LDS_BYTES + WAVES * kStageBytes;  // + the epilogue's staging areas
    // one direct-to-LDS instruction moves 8 rows x 128 bytes (or 64 scale dwords) per wavefront
    static constexpr int A_LOADS = BM / 8 / WAVES, B_LOADS = BN / 8 / WAVES;
    static constexpr int SA_LOADS = SCALED ? SDW * ((BM / 64 + WAVES - 1) / WAVES) : 0, SB_LOADS = SCALED ? SDW * ((BN / 64 + WAVES - 1) / WAVES) : 0;
    static constexpr int NA = A_LOADS + SA_LOADS, NB = B_LOADS + SB_LOADS;  // DMA slots per step
    static_assert(BM % (8 * WAVES) == 0 && BN % (8 * WAVES) == 0, "tile rows per wavefront");
    static_assert(BM % 64 == 0 && BN % 64 == 0, "scale rows per instruction");
    static_assert(NB <= 2 * TM, "the B loads of the next step are issued with the MFMAs of the first column");
    static_assert(NA + NB < 64, "wait-count immediate");
};

// Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2. Renumber them so
// that consecutive logical ids run on the same XCD, then walk the tile grid in column panels of
// `PANEL` tiles so that the workgroups resident on one XCD share A rows and B rows in its L2.
__device__ __forceinline__ int xcd_logical_id(int bid, int nblocks)
{
    constexpr int XCDS = 8;
    const int full = (nblocks / XCDS) * XCDS;
    return bid < full ? (bid % XCDS) * (nblocks / XCDS) + bid / XCDS : bid;
}
__device__ __forceinline__ void panel_tile(int lid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int PANEL = 8;
    const int per_panel = PANEL * tiles_m;
    const int panel = lid / per_panel;
    const int in_panel = lid - panel * per_panel;
    const int width = min(PANEL, tiles_n - panel * PANEL);
    tm = in_panel / width;
    tn = panel * PANEL + in_panel % width;
}
__device__ __forceinline__ void tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n, int &tm,
                                              int &tn)
{
    panel_tile(xcd_logical_id(bid, nblocks), tiles_m, tiles_n, tm, tn);
}

// Nothing may be scheduled across this point: the instruction order below is the schedule.
#define MXFP8_PIN() __builtin_amdgcn_sched_barrier(0)
// s_waitcnt vmcnt(n), other counters untouched (gfx9 encoding: vmcnt is split over bits 3:0 and 15:14)
#define MXFP8_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// One K step of one 16x16 output tile. MXFP8: one scaled matrix instruction over 128 k (4 blocks per
// operand row, scale byte 0 of each lane's scale register). BF16: the lane's two 16-byte pieces are k
// 8g..8g+7 and 32+8g..32+8g+7 of the row's 64 values: two 16x16x32 instructions. MXFP4: the lane's two
// 16-byte pieces are scale blocks g and 4+g of the row's 8 (with 4-bit elements a lane holds one whole block
// and its own scale byte applies to it): two scaled instructions over 128 k each; the scale registers carry
// the byte of block g in bits 7:0 and that of block 4+g in bits 15:8.
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
template <class Cfg>
__device__ __forceinline__ v4f mma_step(const v8i &first, const v8i &second, v4f acc, int s_first, int s_second)
{
    constexpr int FMT = Cfg::FMT;
    if constexpr (FMT == kFmtFp8) {
        // format fields: 0 = E4M3, 1 = E5M2; the kernels feed B fragments as the first operand, A as the second
        return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(first, second, acc, Cfg::B_E5M2 ? 1 : 0, Cfg::A_E5M2 ? 1 : 0, 0,
                                                                s_first, 0, s_second);
    } else if constexpr (FMT == kFmtFp4) {
        const v8i f0 = {first[0], first[1], first[2], first[3], 0, 0, 0, 0}, f1 = {first[4], first[5], first[6], first[7], 0, 0, 0, 0};
        const v8i s0 = {second[0], second[1], second[2], second[3], 0, 0, 0, 0}, s1 = {second[4], second[5], second[6], second[7], 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(f0, s0, acc, 4, 4, 0, s_first & 0xFF, 0, s_second & 0xFF);
        return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(f1, s1, acc, 4, 4, 0, (int)((uint32_t)s_first >> 8), 0,
                                                                (int)((uint32_t)s_second >> 8));
    } else {
        const v4i f0 = {first[0], first[1], first[2], first[3]}, f1 = {first[4], first[5], first[6], first[7]};
        const v4i s0 = {second[0], second[1], second[2], second[3]}, s1 = {second[4], second[5], second[6], second[7]};
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, f0), __builtin_bit_cast(v8bf, s0), acc, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, f1), __builtin_bit_cast(v8bf, s1), acc, 0, 0, 0);
    }
}

// Expert groups of the grouped products (Appendix A.4), see gemm_persistent_kernel (rows of A grouped) and
// gemm_kernel (the reduction axis grouped).
struct GemmGroups {
    const int32_t *ends;  // device memory, `count` non-decreasing row numbers, the last one <= M
    int count;
    int64_t b_group_bytes, bs_group_bytes;
};

// Scale register of one fragment from a scale buffer in LDS ([dword][row][4], `rows` tile rows): MXFP8 takes the
// byte of the lane's K block, MXFP4 the bytes of blocks g and 4+g (same position in the two dwords of the row).
template <class Cfg> __device__ __forceinline__ int read_scale(const uint8_t *sbuf, int off, int rows)
{
    if constexpr (Cfg::FMT == kFmtFp4)
        return (int)sbuf[off] | ((int)sbuf[rows * 4 + off] << 8);
    else if constexpr (Cfg::FMT == kFmtFp8)
        return sbuf[off];
    else
        return 0;
}

// The kernel. LDS holds two A buffers, two B buffers and their scale dwords; the software pipeline
// is described at the step lambda below.
// KGROUPED (Appendix A.4, weight gradient of a mixture-of-experts layer): the reduction axis is the token
// axis, sorted by expert; expert e owns K range [group_ends[e-1], group_ends[e]) of both operands and gets its
// own output [M x N], `M * ldc` elements after the previous expert's. Workgroup = (expert, tile); the K range
// comes from device memory, is clamped to [previous end, K] and cut down to whole K steps (ends have to be
// multiples of 128 tokens); an expert without tokens stores zeros.
template <class Cfg, bool OUT_BF16, bool TILED, bool KGROUPED = false>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_kernel(
    const uint8_t *__restrict__ a_q, const uint8_t *__restrict__ a_s, const uint8_t *__restrict__ b_q,
    const uint8_t *__restrict__ b_s, int M, int N, int K, uint8_t *__restrict__ c_all, int64_t ldc_bytes,
    int tiles_m, int tiles_n, bool vec_store, GemmGroups groups)
{
    MXFP8_DYNAMIC_LDS(lds);
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform: lives in an SGPR
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
    const int r16 = lane & 15, g = lane >> 4;

    int tile_m, tile_n;
    int k0 = 0, k_len = K;  // the K range this workgroup reduces over
    uint8_t *c = c_all;
    if constexpr (KGROUPED) {
        const int per_expert = tiles_m * tiles_n;
        const int e = (int)blockIdx.x / per_expert;
        int prev = 0, end = 0;
        for (int i = 0; i <= e; ++i) {
            prev = end;
            end = min(max(groups.ends[i], prev), K);
        }
        k0 = prev / BK * BK;
        k_len = max(end / BK * BK - k0, 0);
        c += (int64_t)e * M * ldc_bytes;
        tile_of_block((int)blockIdx.x - e * per_expert, per_expert, tiles_m, tiles_n, tile_m, tile_n);
    } else {
        tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, tile_m, tile_n);
    }
    const int m0 = tile_m * Cfg::BM, n0 = tile_n * Cfg::BN;
    // K is the length of an operand row in BYTES (= elements for MXFP8, 2 x elements for BF16 operands)
    static_assert(!KGROUPED || Cfg::ALL_E4M3, "grouped products take MXFP8-E4M3 operands");
    const int nkb = K / Cfg::SBLK;  // scale bytes per row
    const int KT = k_len / BK;      // steps of this workgroup
    const int KT_row = K / BK;   // steps in a whole operand row (the pitch of the tiled scale layout)

    // ---- global -> LDS addressing: wavefront w owns 8-row groups w*LOADS.. of each tile; one
    // instruction fills 8 consecutive rows, lane l lands at row l/8, physical chunk l%8, and
    // fetches the logical chunk that the XOR swizzle stores there. Offsets are relative to the
    // tile origin (32-bit: a tile spans at most 256 rows of K bytes).
    const int ld_r = lane >> 3, ld_c = lane & 7;
    uint32_t a_goff[Cfg::A_LOADS], b_goff[Cfg::B_LOADS], as_goff[Cfg::SA_LOADS + 1], bs_goff[Cfg::SB_LOADS + 1];
#pragma unroll
    for (int i = 0; i < Cfg::A_LOADS; ++i) {
        const int row = (wave * Cfg::A_LOADS + i) * 8 + ld_r;
        const int chunk = ld_c ^ ((row >> 1) & 7);
        a_goff[i] = (uint32_t)min(row, M - 1 - m0) * (uint32_t)K + chunk * 16;  // ragged tiles re-read a valid row
    }
#pragma unroll
    for (int i = 0; i < Cfg::B_LOADS; ++i) {
        const int row = (wave * Cfg::B_LOADS + i) * 8 + ld_r;
        const int chunk = ld_c ^ ((row >> 1) & 7);
        b_goff[i] = (uint32_t)min(row, N - 1 - n0) * (uint32_t)K + chunk * 16;
    }
    // scale request i of a wavefront: scale dword i % SDW of the K step, for 64-row group a_grp(i) / b_grp(i)
    constexpr int SDW = Cfg::SDW;
    auto a_grp = [&](int i) __attribute__((always_inline)) { return (wave + (i / SDW) * Cfg::WAVES) % (Cfg::BM / 64); };
    auto b_grp = [&](int i) __attribute__((always_inline)) { return (wave + (i / SDW) * Cfg::WAVES) % (Cfg::BN / 64); };
#pragma unroll
    for (int i = 0; i < Cfg::SA_LOADS; ++i)
        as_goff[i] = (uint32_t)min(a_grp(i) * 64 + lane, M - 1 - m0) * (uint32_t)nkb;
#pragma unroll
    for (int i = 0; i < Cfg::SB_LOADS; ++i)
        bs_goff[i] = (uint32_t)min(b_grp(i) * 64 + lane, N - 1 - n0) * (uint32_t)nkb;
    const uint8_t *a_tile = a_q + (int64_t)m0 * K + k0, *b_tile = b_q + (int64_t)n0 * K + k0;
    const uint8_t *as_tile = a_s + (int64_t)m0 * nkb + k0 / Cfg::SBLK, *bs_tile = b_s + (int64_t)n0 * nkb + k0 / Cfg::SBLK;
    // Tiled scales: the 64 dwords of a (64-row group, K step) are contiguous, so the instruction that
    // reads one cache line per lane from row-major scales reads 256 consecutive bytes here. A ragged
    // last tile re-reads the last valid group: its rows are never stored.
    const uint8_t *as_grp[Cfg::SA_LOADS + 1], *bs_grp[Cfg::SB_LOADS + 1];
    if constexpr (TILED) {
#pragma unroll
        for (int i = 0; i < Cfg::SA_LOADS; ++i)
            as_grp[i] = a_s + ((int64_t)min(m0 / 64 + a_grp(i), (M + 63) / 64 - 1) * KT_row + k0 / BK) * (256 * SDW);
#pragma unroll
        for (int i = 0; i < Cfg::SB_LOADS; ++i)
            bs_grp[i] = b_s + ((int64_t)min(n0 / 64 + b_grp(i), (N + 63) / 64 - 1) * KT_row + k0 / BK) * (256 * SDW);
    }
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds);

    // DMA slot t (compile-time after unrolling) of the A / B loads of K step kt into buffer buf
    auto issue_a = [&](int t, int kt, int buf) __attribute__((always_inline)) {
        if (t < Cfg::A_LOADS) {
            dma_load<16>(a_tile + (int64_t)kt * BK, a_goff[t],
                         lds_base + Cfg::A_OFF + buf * Cfg::A_BYTES + (wave * Cfg::A_LOADS + t) * 1024);
        } else if (t < Cfg::NA) {
            const int i = t - Cfg::A_LOADS;
            // every wavefront issues the same number of requests (the wait counts rely on it):
            // with fewer 64-row groups than wavefronts some groups are simply fetched twice
            const int dw = i % SDW;
            if constexpr (TILED)
                dma_load<4>(as_grp[i] + ((int64_t)kt * SDW + dw) * 256, lane * 4,
                            lds_base + Cfg::SA_OFF + buf * Cfg::SA_BYTES + dw * Cfg::BM * 4 + a_grp(i) * 256);
            else
                dma_load<4>(as_tile + (kt * SDW + dw) * 4, as_goff[i],
                            lds_base + Cfg::SA_OFF + buf * Cfg::SA_BYTES + dw * Cfg::BM * 4 + a_grp(i) * 256);
        }
    };
    auto issue_b = [&](int t, int kt, int buf) __attribute__((always_inline)) {
        if (t < Cfg::B_LOADS) {
            dma_load<16>(b_tile + (int64_t)kt * BK, b_goff[t],
                         lds_base + Cfg::B_OFF + buf * Cfg::B_BYTES + (wave * Cfg::B_LOADS + t) * 1024);
        } else if (t < Cfg::NB) {
            const int i = t - Cfg::B_LOADS;
            const int dw = i % SDW;
            if constexpr (TILED)
                dma_load<4>(bs_grp[i] + ((int64_t)kt * SDW + dw) * 256, lane * 4,
                            lds_base + Cfg::SB_OFF + buf * Cfg::SB_BYTES + dw * Cfg::BN * 4 + b_grp(i) * 256);
            else
                dma_load<4>(bs_tile + (kt * SDW + dw) * 4, bs_goff[i],
                            lds_base + Cfg::SB_OFF + buf * Cfg::SB_BYTES + dw * Cfg::BN * 4 + b_grp(i) * 256);
        }
    };

    // ---- fragment addresses (bytes inside an A or B buffer): row*128 + swizzled 16-byte chunk for
    // the two K halves a lane holds; tile i sits 16 rows = 2048 bytes further (the swizzle term
    // (row/2)%8 does not change with multiples of 16 rows). Scale byte: row*4 + K block.
    const int a_row = wm * Cfg::WM + r16, b_row = wn * Cfg::WN + r16;
    const int a_off0 = a_row * BK + ((g ^ ((a_row >> 1) & 7)) << 4), a_off1 = a_row * BK + (((4 + g) ^ ((a_row >> 1) & 7)) << 4);
    const int b_off0 = b_row * BK + ((g ^ ((b_row >> 1) & 7)) << 4), b_off1 = b_row * BK + (((4 + g) ^ ((b_row >> 1) & 7)) << 4);
    const int a_soff = a_row * 4 + g, b_soff = b_row * 4 + g;
    auto read_frag = [&](const uint8_t *base, int off0, int off1) __attribute__((always_inline)) {
        const v4i lo = *reinterpret_cast<const v4i *>(base + off0);
        const v4i hi = *reinterpret_cast<const v4i *>(base + off1);
        return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    };

    v4f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    v8i fa[TM];  // A fragments and scale bytes of the current step (refilled in place, see below)
    int sa[TM];

    // ---- one K step (buffers cur = kt & 1, nxt = the other one) ----------------------------------
    // State on entry: the A fragments and A scale bytes of step kt are in registers (fa, sa); B(kt)
    // is in LDS buffer cur; A(kt+1) is in flight towards (or already in) A buffer nxt.
    //   column 0      : MFMAs start at once (only the first B fragment has to arrive); the B tile of
    //                   step kt+1 is requested into B buffer nxt, one DMA instruction per MFMA;
    //   columns 1..-2 : B fragments stream through two register sets; the A tile of step kt+2 is
    //                   requested into A buffer cur (its fragments were pulled into registers during
    //                   the previous step), in the second half of each column, when the prefetch
    //                   read of the next B fragment has drained from the LDS queue;
    //   barrier M     : wait until only the requests of this step are outstanding, i.e. A(kt+1) has
    //                   landed for every wavefront;
    //   last column   : after MFMA (i, last) the registers of A fragment i are dead and are refilled
    //                   in place with fragment i of A(kt+1): the fragment reads of the next step are
    //                   spread over this column instead of bursting at its start;
    //   barrier E     : wait until B(kt+1) has landed (only this step's A requests may be pending).
    // So B is fetched one step ahead, A almost two, with 96 KB in flight against 64 KB in use.
    constexpr int A_LO = (TN - 2) * (TM - TM / 2) >= Cfg::NA ? TM / 2 : 0;  // first MFMA of a column that issues
    static_assert((TN - 2) * (TM - A_LO) >= Cfg::NA, "A requests fit into columns 1..TN-2");
    auto step = [&](int kt) __attribute__((always_inline)) {
        const int cur = kt & 1, nxt = cur ^ 1;
        // past the end of K the prefetches fetch the last step again into buffers nobody reads any
        // more: every step runs the same branch-free code and the wait counts stay valid
        const int kt1 = min(kt + 1, KT - 1), kt2 = min(kt + 2, KT - 1);
        const uint8_t *bbuf = lds + Cfg::B_OFF + cur * Cfg::B_BYTES, *sbbuf = lds + Cfg::SB_OFF + cur * Cfg::SB_BYTES;
        const uint8_t *anext = lds + Cfg::A_OFF + nxt * Cfg::A_BYTES, *sanext = lds + Cfg::SA_OFF + nxt * Cfg::SA_BYTES;
        // B fragments stream through NFB register sets, fetched NFB-1 columns ahead of their use
        constexpr int NFB = 3;
        v8i fb[NFB];
        int sb[NFB];
#pragma unroll
        for (int j = 0; j < NFB - 1 && j < TN; ++j) {
            fb[j] = read_frag(bbuf, b_off0 + j * 2048, b_off1 + j * 2048);
            sb[j] = read_scale<Cfg>(sbbuf, b_soff + j * 64, Cfg::BN);
        }
        MXFP8_PIN();
        int a_slot = 0;  // compile-time after unrolling
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (j + NFB - 1 < TN) {
                fb[(j + NFB - 1) % NFB] = read_frag(bbuf, b_off0 + (j + NFB - 1) * 2048, b_off1 + (j + NFB - 1) * 2048);
                sb[(j + NFB - 1) % NFB] = read_scale<Cfg>(sbbuf, b_soff + (j + NFB - 1) * 64, Cfg::BN);
            }
            if (j == TN - 1) {
                MXFP8_WAIT_VMCNT(Cfg::NA + Cfg::NB);  // all but this step's requests: A(kt+1) is in LDS
                __syncthreads();
            }
            MXFP8_PIN();
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                acc[i][j] = mma_step<Cfg>(fb[j % NFB], fa[i], acc[i][j], sb[j % NFB], sa[i]);
                MXFP8_PIN();
                if (j == 0) {
                    issue_b(i, kt1, nxt);
                    if (i + TM < Cfg::NB)
                        issue_b(i + TM, kt1, nxt);
                } else if (j < TN - 1 && i >= A_LO) {
                    if (a_slot < Cfg::NA)
                        issue_a(a_slot, kt2, cur);
                    ++a_slot;
                }
                if (j == TN - 1) {
                    fa[i] = read_frag(anext, a_off0 + i * 2048, a_off1 + i * 2048);
                    sa[i] = read_scale<Cfg>(sanext, a_soff + i * 64, Cfg::BM);
                }
                MXFP8_PIN();
            }
        }
        MXFP8_WAIT_VMCNT(Cfg::NA);  // everything older than this step's A requests: B(kt+1) is in LDS
        __syncthreads();
    };

    if (KT > 0) {
#pragma unroll
        for (int t = 0; t < Cfg::NA; ++t)
            issue_a(t, 0, 0);
#pragma unroll
        for (int t = 0; t < Cfg::NB; ++t)
            issue_b(t, 0, 0);
#pragma unroll
        for (int t = 0; t < Cfg::NA; ++t)
            issue_a(t, min(1, KT - 1), 1);
        MXFP8_WAIT_VMCNT(0);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            fa[i] = read_frag(lds + Cfg::A_OFF, a_off0 + i * 2048, a_off1 + i * 2048);
            sa[i] = read_scale<Cfg>(lds + Cfg::SA_OFF, a_soff + i * 64, Cfg::BM);
        }
        __syncthreads();  // A buffer 0 is refilled by the requests of step 0 from here on
    }
    for (int kt = 0; kt < KT; ++kt)
        step(kt);
    MXFP8_WAIT_VMCNT(0);  // drain the redundant tail prefetches before the LDS allocation is released

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

// Workgroup barrier without the LDS fence of __syncthreads(): LDS reads issued before it may still be in
// flight afterwards. The persistent kernel uses it where a barrier only publishes DMA-written buffers
// (their arrival is tracked by vmcnt) and nothing that is still being read is handed back for overwriting.
// Where a buffer IS handed back (end of a K step) the reads that can still be in flight are awaited first
// (MXFP8_WAIT_VMCNT_AND_LDS): fragment reads that an already issued MFMA consumed have returned by
// construction, the in-place refills of the A fragments are the only ones left.
#define MXFP8_BARRIER() __builtin_amdgcn_s_barrier()
// s_waitcnt vmcnt(n) lgkmcnt(0): additionally every LDS read of this wavefront has returned
#define MXFP8_WAIT_VMCNT_AND_LDS(n) __builtin_amdgcn_s_waitcnt(0x0070 | ((n) & 15) | (((n) >> 4) << 14))

// ---- persistent variant --------------------------------------------------------------------------
// One workgroup per compute unit walks over several output tiles and keeps the K pipeline running
// across tile boundaries: the prefetches of the last two K steps of a tile, which the kernel above
// spends on re-reading the last step, fetch the first steps of the workgroup's next tile instead, so
// only the first tile of a workgroup has a prologue, and the epilogue stores of a tile drain while
// the operands of the next one are already in flight. Restricted to problems made of full tiles
// (M % BM == 0, N % BN == 0: every 8B-class layer shape) with K >= 2 steps and vector-storable C;
// without ragged tiles the DMA offsets inside a tile are the same for every tile.
// Wait counts: the epilogue's stores also count in vmcnt. Loads complete in order among themselves,
// so "at most n operations outstanding" still implies that all but the last n loads have landed,
// whatever the stores do; the immediates of the K step stay valid (they can only wait longer).
// FUSE_Q (BF16 output only; bit 0 = row-wise copy, bit 1 = column-wise copy): the epilogue also emits
// MXFP8 copies of the BF16-rounded output tile (Section 2: the output is re-quantized when the next layer
// needs it in MX format; Section 3.2: along rows and along columns; conversion of Section 3.3 /
// Appendix A.1, A.2 applied to the BF16 values), scales in the same layout as the inputs.
//   row-wise:    cq [M x N], cs = scales of C as an [M x N] operand. A 32-column block lies in two adjacent
//                MFMA tiles of one row, 8 values in each of the 4 lanes that share the row.
//   column-wise: cqT [N x M], csT = scales of C^T as an [N x M] operand. A 32-row block lies in two
//                vertically adjacent MFMA tiles, 2 values in each of the 16 lanes of a DPP row. The bytes
//                are transposed through the two LDS buffers that are idle between tiles (the B buffer the
//                finished step read and the A buffer whose fragments already sit in registers) and leave
//                as full lines of cqT.
#ifndef MXFP8_GEMM_SCHED
#define MXFP8_GEMM_SCHED 242  // B requests behind every 2nd MFMA, a gap of 2, A requests behind every 4th
#endif
// GROUPED (Appendix A.4, mixture-of-experts layers): the rows of A are tokens sorted by expert, rows
// [group_ends[e-1], group_ends[e]) belong to expert e, whose B operand starts b_group_bytes (scales:
// bs_group_bytes) after the previous expert's. group_ends lives in DEVICE memory (routing happens on the
// GPU), so the host cannot count the tiles: every workgroup sums them up itself, walks over its share and
// finds the expert of a tile by scanning the ends (wavefront-uniform scalar code, a few hundred cycles per
// 100 k-cycle tile). An expert's last tile may be partial: its surplus rows are computed from whatever
// rows follow (the next expert's, or re-reads of the last row of A) and not stored. N stays a multiple of
// the tile. Ends are clamped to [previous end, M], so bad ends cannot send a load out of A.
template <class Cfg, bool OUT_BF16, bool TILED, bool SPREAD, int FUSE_Q = 0, int SCHED = MXFP8_GEMM_SCHED, bool GROUPED = false>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_persistent_kernel(
    const uint8_t *__restrict__ a_q, const uint8_t *__restrict__ a_s, const uint8_t *__restrict__ b_q,
    const uint8_t *__restrict__ b_s, int M, int N, int K, uint8_t *__restrict__ c, int64_t ldc_bytes,
    int tiles_m, int tiles_n, uint8_t *__restrict__ cq, uint8_t *__restrict__ cs, uint8_t *__restrict__ cqT,
    uint8_t *__restrict__ csT, GemmGroups groups)
{
    static_assert(!GROUPED || (FUSE_Q == 0 && Cfg::ALL_E4M3), "grouped products: MXFP8-E4M3 operands, plain epilogue");
    static_assert(!FUSE_Q || (OUT_BF16 && (Cfg::TN == 8 || Cfg::TN == 4) && Cfg::TM == Cfg::TN), "fused output quantization");
    constexpr bool Q_ROW = (FUSE_Q & 1) != 0, Q_COL = (FUSE_Q & 2) != 0;
    static_assert(!Q_COL || Cfg::BM * Cfg::BN <= 2 * Cfg::B_BYTES, "transposed tile fits the two idle buffers");
    static_assert(!Cfg::SCALED || (Cfg::SA_LOADS == Cfg::SDW && Cfg::SB_LOADS == Cfg::SDW), "one scale request per wavefront, operand and scale dword");
    static_assert(Cfg::ALL_E4M3 || FUSE_Q == 0, "output quantization belongs to the MXFP8-E4M3 product");
    MXFP8_DYNAMIC_LDS(lds);
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
    const int r16 = lane & 15, g = lane >> 4;
    constexpr int SDW = Cfg::SDW;
    const int nkb = K / Cfg::SBLK;
    const int KT = K / BK;
    int ntiles = tiles_m * tiles_n;
    if constexpr (GROUPED) {
        ntiles = 0;
        for (int e = 0, prev = 0; e < groups.count; ++e) {
            const int end = min(max(groups.ends[e], prev), M);
            ntiles += (end - prev + Cfg::BM - 1) / Cfg::BM * tiles_n;
            prev = end;
        }
    }
    const int stride = gridDim.x;
    // >= 1 when the host knows the number of tiles (the grid has at most that many workgroups)
    const int my_tiles = (ntiles - (int)blockIdx.x + stride - 1) / stride;
    if (GROUPED && my_tiles <= 0)
        return;  // the whole workgroup, before any barrier

    // ---- DMA offsets inside an operand tile (see the kernel above). Without ragged rows they do not
    // depend on the tile, and with square tiles the A and the B tile use the same ones.
    static_assert(Cfg::BM == Cfg::BN, "A and B tiles share their DMA offsets");
    const int ld_r = lane >> 3, ld_c = lane & 7;
    uint32_t goff[Cfg::A_LOADS];
#pragma unroll
    for (int i = 0; i < Cfg::A_LOADS; ++i) {
        const int row = (wave * Cfg::A_LOADS + i) * 8 + ld_r;
        goff[i] = (uint32_t)row * (uint32_t)K + (ld_c ^ ((row >> 1) & 7)) * 16;
    }
    const int grp = wave % (Cfg::BM / 64);  // 64-row group of each tile whose scale dwords this wavefront fetches
    const uint32_t sgoff = TILED ? lane * 4 : (uint32_t)(grp * 64 + lane) * (uint32_t)nkb;
    const int s_step = (TILED ? 256 : 4) * SDW;  // bytes from the scale dwords of one K step to the next
    constexpr int s_dword = TILED ? 256 : 4;     // ... and from one scale dword of a K step to its next one
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds);

    // operand pointers of a tile at K step 0 (wavefront-uniform)
    struct Tile {
        const uint8_t *a, *b, *as, *bs;
        int m0, n0;
        int rows;  // GROUPED: rows of the tile that belong to its expert (stored)
        int lim;   // GROUPED: last row of the tile, counted from m0, that may be read from A
    };
    auto tile_at = [&](int index) __attribute__((always_inline)) {
        int tm, tn;
        Tile t;
        const uint8_t *bq = b_q, *bsc = b_s;
        if constexpr (GROUPED) {
            // The workgroups that run side by side have consecutive ids: they work on the same expert (all
            // XCDs then stream the same B operand), and inside the expert's tiles the XCD-aware order applies.
            int u = (int)blockIdx.x + index * stride;
            int e = 0, prev = 0, end = 0, tiles_e = 0;
            for (; e < groups.count; ++e) {  // u < ntiles = the sum of the groups' tiles: the scan ends inside
                end = min(max(groups.ends[e], prev), M);
                tiles_e = (end - prev + Cfg::BM - 1) / Cfg::BM * tiles_n;
                if (u < tiles_e)
                    break;
                u -= tiles_e;
                prev = end;
            }
            panel_tile(xcd_logical_id(u, tiles_e), tiles_e / tiles_n, tiles_n, tm, tn);
            t.m0 = prev + tm * Cfg::BM;
            t.rows = min(Cfg::BM, end - t.m0);
            t.lim = M - 1 - t.m0;
            bq += e * groups.b_group_bytes;
            bsc += e * groups.bs_group_bytes;
        } else {
            tile_of_block((int)blockIdx.x + index * stride, ntiles, tiles_m, tiles_n, tm, tn);
            t.m0 = tm * Cfg::BM;
            t.rows = Cfg::BM;
            t.lim = Cfg::BM;
        }
        t.n0 = tn * Cfg::BN;
        t.a = a_q + (int64_t)t.m0 * K;
        t.b = bq + (int64_t)t.n0 * K;
        if constexpr (TILED) {
            // (grouped: group starts are multiples of 64 rows; 64-row groups past the end of A re-read the last one)
            const int ag = GROUPED ? min(t.m0 / 64 + grp, (M + 63) / 64 - 1) : t.m0 / 64 + grp;
            t.as = a_s + (int64_t)ag * KT * (256 * SDW);
            t.bs = bsc + (int64_t)(t.n0 / 64 + grp) * KT * (256 * SDW);
        } else {
            t.as = a_s + (int64_t)t.m0 * nkb;
            t.bs = bsc + (int64_t)t.n0 * nkb;
        }
        return t;
    };

    // DMA slot t of the A / B requests of one K step, from the step's source pointers into buffer buf.
    // GROUPED: rows of the A tile past `lim` (the end of A) re-read row lim.
    const int row0 = wave * Cfg::A_LOADS * 8 + ld_r;  // this lane's row in DMA slot 0
    auto issue_a = [&](int t, const uint8_t *src, const uint8_t *ssrc, int buf, int lim) __attribute__((always_inline)) {
        if (t < Cfg::A_LOADS) {
            uint32_t off = goff[t];
            if constexpr (GROUPED)
                off -= (uint32_t)max(row0 + 8 * t - lim, 0) * (uint32_t)K;
            dma_load<16>(src, off, lds_base + Cfg::A_OFF + buf * Cfg::A_BYTES + (wave * Cfg::A_LOADS + t) * 1024);
        } else if (t < Cfg::NA) {
            uint32_t off = sgoff;
            if constexpr (GROUPED && !TILED)
                off -= (uint32_t)max(grp * 64 + lane - lim, 0) * (uint32_t)nkb;
            const int dw = t - Cfg::A_LOADS;
            dma_load<4>(ssrc + dw * s_dword, off, lds_base + Cfg::SA_OFF + buf * Cfg::SA_BYTES + dw * Cfg::BM * 4 + grp * 256);
        }
    };
    auto issue_b = [&](int t, const uint8_t *src, const uint8_t *ssrc, int buf) __attribute__((always_inline)) {
        if (t < Cfg::B_LOADS)
            dma_load<16>(src, goff[t], lds_base + Cfg::B_OFF + buf * Cfg::B_BYTES + (wave * Cfg::B_LOADS + t) * 1024);
        else if (t < Cfg::NB)
            dma_load<4>(ssrc + (t - Cfg::B_LOADS) * s_dword, sgoff,
                        lds_base + Cfg::SB_OFF + buf * Cfg::SB_BYTES + (t - Cfg::B_LOADS) * Cfg::BN * 4 + grp * 256);
    };

    const int a_row = wm * Cfg::WM + r16, b_row = wn * Cfg::WN + r16;
    const int a_off0 = a_row * BK + ((g ^ ((a_row >> 1) & 7)) << 4), a_off1 = a_row * BK + (((4 + g) ^ ((a_row >> 1) & 7)) << 4);
    const int b_off0 = b_row * BK + ((g ^ ((b_row >> 1) & 7)) << 4), b_off1 = b_row * BK + (((4 + g) ^ ((b_row >> 1) & 7)) << 4);
    const int a_soff = a_row * 4 + g, b_soff = b_row * 4 + g;
    auto read_frag = [&](const uint8_t *base, int off0, int off1) __attribute__((always_inline)) {
        const v4i lo = *reinterpret_cast<const v4i *>(base + off0);
        const v4i hi = *reinterpret_cast<const v4i *>(base + off1);
        return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    };

    v4f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};
    v8i fa[TM];
    int sa[TM];

    // One K step, same schedule as in the kernel above; the requests go to the sources handed in:
    // (b_src, bs_src) = B tile and scales of the workgroup's NEXT step, (a_src, as_src) = A tile and
    // scales of the step after that, either of which may belong to the next output tile.
    constexpr int A_LO = (TN - 2) * (TM - TM / 2) >= Cfg::NA ? TM / 2 : 0;
    static_assert((TN - 2) * (TM - A_LO) >= Cfg::NA, "A requests fit into columns 1..TN-2");
    auto step = [&](int cur, const uint8_t *b_src, const uint8_t *bs_src, const uint8_t *a_src,
                    const uint8_t *as_src, int a_lim) __attribute__((always_inline)) {
        const int nxt = cur ^ 1;
        const uint8_t *bbuf = lds + Cfg::B_OFF + cur * Cfg::B_BYTES, *sbbuf = lds + Cfg::SB_OFF + cur * Cfg::SB_BYTES;
        const uint8_t *anext = lds + Cfg::A_OFF + nxt * Cfg::A_BYTES, *sanext = lds + Cfg::SA_OFF + nxt * Cfg::SA_BYTES;
        constexpr int NFB = 3;  // B fragment register sets, read NFB-1 columns ahead
        v8i fb[NFB];
        int sb[NFB];
#pragma unroll
        for (int j = 0; j < NFB - 1 && j < TN; ++j) {
            fb[j] = read_frag(bbuf, b_off0 + j * 2048, b_off1 + j * 2048);
            sb[j] = read_scale<Cfg>(sbbuf, b_soff + j * 64, Cfg::BN);
        }
        MXFP8_PIN();
        int a_slot = 0;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (j + NFB - 1 < TN) {
                fb[(j + NFB - 1) % NFB] = read_frag(bbuf, b_off0 + (j + NFB - 1) * 2048, b_off1 + (j + NFB - 1) * 2048);
                sb[(j + NFB - 1) % NFB] = read_scale<Cfg>(sbbuf, b_soff + (j + NFB - 1) * 64, Cfg::BN);
            }
            if (j == TN - 1) {
                MXFP8_WAIT_VMCNT(Cfg::NA + Cfg::NB);
                MXFP8_BARRIER();
            }
            MXFP8_PIN();
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                acc[i][j] = mma_step<Cfg>(fb[j % NFB], fa[i], acc[i][j], sb[j % NFB], sa[i]);
                MXFP8_PIN();
                if constexpr (SPREAD) {
                    // SCHED = 100 * gap + 10 * A spacing + B spacing (in MFMAs)
                    constexpr int B_EVERY = SCHED % 10, A_EVERY = SCHED / 10 % 10, GAP = SCHED / 100;
                    constexpr int A_FIRST = B_EVERY * Cfg::NB + GAP;  // MFMA after which the first A request goes out
                    static_assert(A_FIRST + A_EVERY * (Cfg::NA - 1) < (TN - 1) * TM, "all requests before the last column");
                    const int m = j * TM + i;  // compile-time after unrolling
                    if (m % B_EVERY == 0 && m / B_EVERY < Cfg::NB)
                        issue_b(m / B_EVERY, b_src, bs_src, nxt);
                    else if (m >= A_FIRST && (m - A_FIRST) % A_EVERY == 0 && (m - A_FIRST) / A_EVERY < Cfg::NA)
                        issue_a((m - A_FIRST) / A_EVERY, a_src, as_src, cur, a_lim);
                } else if (j == 0) {
                    issue_b(i, b_src, bs_src, nxt);
                    if (i + TM < Cfg::NB)
                        issue_b(i + TM, b_src, bs_src, nxt);
                } else if (j < TN - 1 && i >= A_LO) {
                    if (a_slot < Cfg::NA)
                        issue_a(a_slot, a_src, as_src, cur, a_lim);
                    ++a_slot;
                }
                if (j == TN - 1) {
                    fa[i] = read_frag(anext, a_off0 + i * 2048, a_off1 + i * 2048);
                    sa[i] = read_scale<Cfg>(sanext, a_soff + i * 64, Cfg::BM);
                }
                MXFP8_PIN();
            }
        }
        // end of the step: B(k+1) has landed; B buffer cur and A buffer nxt go back to the DMA, so this
        // wavefront's refill reads of A buffer nxt must have returned before anybody passes the barrier
        MXFP8_WAIT_VMCNT_AND_LDS(Cfg::NA);
        MXFP8_BARRIER();
    };

    Tile cur_tile = tile_at(0);
    // prologue of the workgroup's first tile: A(0), B(0) into buffers 0, A(1) into A buffer 1
#pragma unroll
    for (int t = 0; t < Cfg::NA; ++t)
        issue_a(t, cur_tile.a, cur_tile.as, 0, cur_tile.lim);
#pragma unroll
    for (int t = 0; t < Cfg::NB; ++t)
        issue_b(t, cur_tile.b, cur_tile.bs, 0);
#pragma unroll
    for (int t = 0; t < Cfg::NA; ++t)
        issue_a(t, cur_tile.a + BK, cur_tile.as + s_step, 1, cur_tile.lim);
    MXFP8_WAIT_VMCNT(0);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        fa[i] = read_frag(lds + Cfg::A_OFF, a_off0 + i * 2048, a_off1 + i * 2048);
        sa[i] = read_scale<Cfg>(lds + Cfg::SA_OFF, a_soff + i * 64, Cfg::BM);
    }
    __syncthreads();

    int par = 0;  // LDS buffer parity of the workgroup's running step count
    for (int ti = 0; ti < my_tiles; ++ti) {
        const bool has_next = ti + 1 < my_tiles;
        const Tile next_tile = has_next ? tile_at(ti + 1) : cur_tile;
        for (int kt = 0; kt < KT; ++kt) {
            // source of the step after this one (B) and of the one after that (A): this tile, else the
            // first steps of the next tile, else (last tile) this tile's last step once more
            const uint8_t *b_src, *bs_src, *a_src, *as_src;
            int a_lim = cur_tile.lim;
            if (kt + 1 < KT) {
                b_src = cur_tile.b + (int64_t)(kt + 1) * BK;
                bs_src = cur_tile.bs + (int64_t)(kt + 1) * s_step;
            } else if (has_next) {
                b_src = next_tile.b;
                bs_src = next_tile.bs;
            } else {
                b_src = cur_tile.b + (int64_t)(KT - 1) * BK;
                bs_src = cur_tile.bs + (int64_t)(KT - 1) * s_step;
            }
            if (kt + 2 < KT) {
                a_src = cur_tile.a + (int64_t)(kt + 2) * BK;
                as_src = cur_tile.as + (int64_t)(kt + 2) * s_step;
            } else if (has_next) {
                a_src = next_tile.a + (int64_t)(kt + 2 - KT) * BK;
                as_src = next_tile.as + (int64_t)(kt + 2 - KT) * s_step;
                a_lim = next_tile.lim;
            } else {
                a_src = cur_tile.a + (int64_t)(KT - 1) * BK;
                as_src = cur_tile.as + (int64_t)(KT - 1) * s_step;
            }
            step(par, b_src, bs_src, a_src, as_src, a_lim);
            par ^= 1;
        }
        // ---- epilogue of this tile; the A requests of the next tile's second step are in flight.
        // Row groups (16 rows of the wavefront's part) are finished one after the other (pinned), each through
        // the wavefront's staging area, so that the converted values of only one row group are live at a
        // time next to the A fragments of the next tile.
        constexpr int ESZ = OUT_BF16 ? 2 : 4;
        if constexpr (Q_COL)
            __syncthreads();  // every wavefront's fragment refills have left the A buffer that is reused below
        uint8_t *ctile = c + (int64_t)cur_tile.m0 * ldc_bytes + (int64_t)cur_tile.n0 * ESZ;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            uint8_t *crow = ctile + (int64_t)(i * 16) * ldc_bytes;
            // the values of this row group are still in accumulator registers at this point: keeps the
            // compiler from moving all 256 of them into ordinary registers at the top of the epilogue
#pragma unroll
            for (int j = 0; j < TN; ++j)
                MXFP8_KEEP_IN_ACC(acc[i][j]);
            if constexpr (Q_ROW) {
                // BF16 rows and their MXFP8 copy both leave through the wavefront's staging area (see the plain
                // epilogue below for why): first the 16 BF16 rows, then, in the same area, the 16 byte rows.
                const int64_t m = cur_tile.m0 + wm * Cfg::WM + i * 16 + r16;        // this lane's row of C
                const int n_wave = cur_tile.n0 + wn * Cfg::WN;                       // first column of the wavefront
                constexpr int ROWB = Cfg::WN * 2, PITCH = ROWB + 32;                 // BF16 row and its staged pitch
                constexpr int QPITCH = Cfg::WN + 16;                                 // staged pitch of a byte row
                static_assert(16 * PITCH <= kStageBytes && (16 * ROWB) % 1024 == 0 && (16 * Cfg::WN) % 1024 == 0, "staging area");
                uint8_t *stage = lds + Cfg::LDS_BYTES + wave * kStageBytes;
                uint32_t scales = 0;                                                 // scale bytes of the row's blocks
                uint32_t q[TN];
#pragma unroll
                for (int blk = 0; blk < TN / 2; ++blk) {
                    uint32_t h[4];  // BF16 pairs: columns 4g..4g+3 of tile 2*blk, then of tile 2*blk+1
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const v4f v = acc[i][2 * blk + t];
                        v2bf p0 = {(__bf16)v[0], (__bf16)v[1]}, p1 = {(__bf16)v[2], (__bf16)v[3]};
                        h[2 * t] = __builtin_bit_cast(uint32_t, p0);
                        h[2 * t + 1] = __builtin_bit_cast(uint32_t, p1);
                        *reinterpret_cast<uint2 *>(stage + r16 * PITCH + ((2 * blk + t) * 16 + 4 * g) * 2) = make_uint2(h[2 * t], h[2 * t + 1]);
                    }
                    // block amax on the magnitude bits: 8 values here, then the 3 other lanes of the row
                    uint32_t am = pk_max_u16(pk_max_u16(h[0] & 0x7FFF7FFFu, h[1] & 0x7FFF7FFFu),
                                             pk_max_u16(h[2] & 0x7FFF7FFFu, h[3] & 0x7FFF7FFFu));
                    am = umax(am & 0xFFFFu, am >> 16);
                    am = umax(am, (uint32_t)__shfl_xor((int)am, 16, 64));
                    am = umax(am, (uint32_t)__shfl_xor((int)am, 32, 64));
                    const uint32_t sb = scale_byte_from_bf16_bits(am);
                    const float sc = scale_operand(sb);
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        uint32_t qt = cvt2_bf16(cvt2_bf16(0, h[2 * t], sc, false), h[2 * t + 1], sc, true);
                        if (sb >= 254) {  // NaN or Inf in the block: rare
                            if (sb == 0xFF) {
                                qt = 0x7F7F7F7Fu;
                            } else {
                                uint32_t f = 0;
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    const uint32_t bits = (e & 1) ? h[2 * t + e / 2] >> 16 : h[2 * t + e / 2] & 0xFFFFu;
                                    f |= inf_byte_bf16(bits, (qt >> (8 * e)) & 0xFFu) << (8 * e);
                                }
                                qt = f;
                            }
                        }
                        q[2 * blk + t] = qt;
                    }
                    scales |= sb << (8 * blk);
                }
                __builtin_amdgcn_wave_barrier();  // the reads below see the other lanes' writes (LDS serves a wavefront in order)
#pragma unroll
                for (int t = 0; t < 16 * ROWB / 1024; ++t) {
                    const int lin = t * 1024 + lane * 16, row = lin / ROWB, colb = lin % ROWB;
                    const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * PITCH + colb);
                    *reinterpret_cast<uint4 *>(crow + (int64_t)(wm * Cfg::WM + row) * ldc_bytes + wn * ROWB + colb) = v;
                }
                __builtin_amdgcn_wave_barrier();  // the byte rows overwrite the area after these reads
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    *reinterpret_cast<uint32_t *>(stage + r16 * QPITCH + j * 16 + 4 * g) = q[j];
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int t = 0; t < 16 * Cfg::WN / 1024; ++t) {
                    const int lin = t * 1024 + lane * 16, row = lin / Cfg::WN, colb = lin % Cfg::WN;
                    const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * QPITCH + colb);
                    *reinterpret_cast<uint4 *>(cq + (cur_tile.m0 + wm * Cfg::WM + i * 16 + row) * (int64_t)N + n_wave + colb) = v;
                }
                __builtin_amdgcn_wave_barrier();  // (the next row group overwrites the area after these reads)
                if (g == 0) {  // the TN/2 scale bytes of this row and wavefront: one dword or halfword
                    const int64_t nb = N / kBlock, b0 = n_wave / kBlock;
                    uint8_t *sp = TILED ? cs + (((m >> 6) * ((nb + 3) / 4) + (b0 >> 2)) * 64 + (m & 63)) * 4 + (b0 & 3)
                                        : cs + m * nb + b0;
                    if constexpr (TN / 2 == 4)
                        *reinterpret_cast<uint32_t *>(sp) = scales;
                    else
                        *reinterpret_cast<uint16_t *>(sp) = (uint16_t)scales;
                }
            } else {
                // Row group i of this wavefront (16 rows x WN columns) goes through a wavefront-private LDS area
                // so that it leaves as whole rows: a lane holds 4 consecutive columns of one row per MFMA tile,
                // and storing those directly costs one partial cache line per row and instruction (the address
                // unit of the compute unit then needs ~7 us per 256 x 256 tile, during which the matrix pipes
                // wait behind their own stores). Staged, every store instruction writes 1 KB of contiguous rows.
                constexpr int ROWB = Cfg::WN * ESZ;                            // bytes of one row of the wavefront's part
                constexpr int PITCH = ROWB + 32;                               // staged row pitch: spreads the rows over the banks
                constexpr int RPP = ROWB * 16 <= 4096 ? 16 : 4096 / ROWB;      // rows per pass (at most 4 KB staged)
                static_assert(RPP * PITCH <= kStageBytes && (RPP * ROWB) % 1024 == 0, "staging area");
                uint8_t *stage = lds + Cfg::LDS_BYTES + wave * kStageBytes;
#pragma unroll
                for (int pass = 0; pass < 16 / RPP; ++pass) {
                    if (RPP == 16 || r16 / RPP == pass) {
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const v4f v = acc[i][j];
                            uint8_t *dst = stage + (r16 % RPP) * PITCH + (j * 16 + 4 * g) * ESZ;
                            if constexpr (OUT_BF16) {
                                v2bf p0 = {(__bf16)v[0], (__bf16)v[1]}, p1 = {(__bf16)v[2], (__bf16)v[3]};
                                *reinterpret_cast<uint2 *>(dst) =
                                    make_uint2(__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1));
                            } else {
                                *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                            }
                        }
                    }
                    __builtin_amdgcn_wave_barrier();  // the reads below see the other lanes' writes (LDS serves a wavefront in order)
#pragma unroll
                    for (int t = 0; t < RPP * ROWB / 1024; ++t) {
                        const int lin = t * 1024 + lane * 16, row = lin / ROWB, colb = lin % ROWB;
                        const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * PITCH + colb);
                        if (!GROUPED || wm * Cfg::WM + i * 16 + pass * RPP + row < cur_tile.rows)
                            *reinterpret_cast<uint4 *>(crow + (int64_t)(wm * Cfg::WM + pass * RPP + row) * ldc_bytes +
                                                       wn * ROWB + colb) = v;
                    }
                    __builtin_amdgcn_wave_barrier();  // (the next pass overwrites the area after these reads)
                }
            }
            MXFP8_PIN();
        }
        if constexpr (Q_COL) {
            // Idle LDS between tiles: B buffer par^1 (read by the step that just ended) and A buffer par (its
            // fragments are in registers). Transposed tile [column][BM row bytes]; the first half of the
            // columns in the B buffer, the second half in the A buffer when one buffer is too small. The
            // 16-byte chunk of a column line is XORed with (column / 4) so that the four lanes of a row,
            // whose columns are 4 apart, write different banks.
            constexpr bool SPLIT = Cfg::BM * Cfg::BN > Cfg::B_BYTES;
            constexpr int COLS_PER_REGION = SPLIT ? Cfg::BN / 2 : Cfg::BN;
            constexpr int CHUNKS = Cfg::BM / 16;  // 16-byte chunks per column line
            uint8_t *region0 = lds + Cfg::B_OFF + (par ^ 1) * Cfg::B_BYTES;
            uint8_t *region1 = lds + Cfg::A_OFF + par * Cfg::A_BYTES;
            auto line_of = [&](int n_tile) __attribute__((always_inline)) {
                return (SPLIT && n_tile >= COLS_PER_REGION ? region1 : region0) + (n_tile % COLS_PER_REGION) * Cfg::BM;
            };
            const int64_t nbT = M / kBlock;                                   // scale blocks per row of C^T
            const int64_t bT0 = (cur_tile.m0 + wm * Cfg::WM) / kBlock;        // first row block of this wavefront
#pragma unroll
            for (int j = 0; j < TN; ++j) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    MXFP8_KEEP_IN_ACC(acc[i][j]);  // (see the row loop above)
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int n_tile = wn * Cfg::WN + j * 16 + 4 * g + 2 * half;  // columns n_tile and n_tile + 1
                    uint8_t *line0 = line_of(n_tile), *line1 = line_of(n_tile + 1);
                    const int sw0 = (n_tile >> 2) & (CHUNKS - 1);                 // same for n_tile + 1
                    uint32_t scales0 = 0, scales1 = 0;
#pragma unroll
                    for (int rb = 0; rb < TM / 2; ++rb) {
                        // rows r16 and 16 + r16 of the 32-row block, as BF16 pairs (column n_tile low, n_tile + 1 high)
                        const v4f va = acc[2 * rb][j], vb = acc[2 * rb + 1][j];
                        v2bf pa = {(__bf16)va[2 * half], (__bf16)va[2 * half + 1]}, pb = {(__bf16)vb[2 * half], (__bf16)vb[2 * half + 1]};
                        const uint32_t xa = __builtin_bit_cast(uint32_t, pa), xb = __builtin_bit_cast(uint32_t, pb);
                        uint32_t am = pk_max_u16(xa & 0x7FFF7FFFu, xb & 0x7FFF7FFFu);
                        am = pk_max_u16(am, dpp_xor1(am));
                        am = pk_max_u16(am, dpp_xor2(am));
                        am = pk_max_u16(am, dpp_half_mirror(am));
                        am = pk_max_u16(am, dpp_mirror(am));
                        const uint32_t sb0 = scale_byte_from_bf16_bits(am & 0xFFFFu), sb1 = scale_byte_from_bf16_bits(am >> 16);
                        // (row r16, row 16 + r16) of one column as a BF16 pair
                        const uint32_t c0 = __builtin_amdgcn_perm(xb, xa, 0x05040100u), c1 = __builtin_amdgcn_perm(xb, xa, 0x07060302u);
                        uint32_t q0 = cvt2_bf16(0, c0, scale_operand(sb0), false) & 0xFFFFu;
                        uint32_t q1 = cvt2_bf16(0, c1, scale_operand(sb1), false) & 0xFFFFu;
                        if (sb0 >= 254)
                            q0 = sb0 == 0xFF ? 0x7F7Fu
                                             : inf_byte_bf16(c0 & 0xFFFFu, q0 & 0xFFu) | (inf_byte_bf16(c0 >> 16, q0 >> 8) << 8);
                        if (sb1 >= 254)
                            q1 = sb1 == 0xFF ? 0x7F7Fu
                                             : inf_byte_bf16(c1 & 0xFFFFu, q1 & 0xFFu) | (inf_byte_bf16(c1 >> 16, q1 >> 8) << 8);
                        const int m_lo = wm * Cfg::WM + rb * 32 + r16, m_hi = m_lo + 16;  // rows inside the tile
                        line0[(((m_lo >> 4) ^ sw0) << 4) + (m_lo & 15)] = (uint8_t)q0;
                        line0[(((m_hi >> 4) ^ sw0) << 4) + (m_hi & 15)] = (uint8_t)(q0 >> 8);
                        line1[(((m_lo >> 4) ^ sw0) << 4) + (m_lo & 15)] = (uint8_t)q1;
                        line1[(((m_hi >> 4) ^ sw0) << 4) + (m_hi & 15)] = (uint8_t)(q1 >> 8);
                        scales0 |= sb0 << (8 * rb);
                        scales1 |= sb1 << (8 * rb);
                    }
                    if (r16 == 0) {  // the TM/2 scale bytes of two columns of C^T: a dword or halfword each
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            const int64_t n = cur_tile.n0 + n_tile + t;
                            uint8_t *sp = TILED ? csT + (((n >> 6) * ((nbT + 3) / 4) + (bT0 >> 2)) * 64 + (n & 63)) * 4 + (bT0 & 3)
                                                : csT + n * nbT + bT0;
                            if constexpr (TM / 2 == 4)
                                *reinterpret_cast<uint32_t *>(sp) = t ? scales1 : scales0;
                            else
                                *reinterpret_cast<uint16_t *>(sp) = (uint16_t)(t ? scales1 : scales0);
                        }
                    }
                }
                MXFP8_PIN();
            }
            __syncthreads();  // the transposed tile is complete
#pragma unroll
            for (int pass = 0; pass < Cfg::BN * CHUNKS / Cfg::THREADS; ++pass) {
                const int chunk = pass * Cfg::THREADS + tid;
                const int n_tile = chunk / CHUNKS, part = chunk % CHUNKS;
                const uint4 v = *reinterpret_cast<const uint4 *>(line_of(n_tile) + ((part ^ ((n_tile >> 2) & (CHUNKS - 1))) << 4));
                *reinterpret_cast<uint4 *>(cqT + (int64_t)(cur_tile.n0 + n_tile) * M + cur_tile.m0 + part * 16) = v;
            }
            __syncthreads();  // nobody requests the next tiles into these buffers while they are still read
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};
        cur_tile = next_tile;
    }
    MXFP8_WAIT_VMCNT(0);  // the redundant prefetches of the last steps must land before LDS is released
}

// Number of workgroups of a persistent launch: one per compute unit of the current device, at most
// `max_workgroups` when the caller gives a positive bound, never more than there are tiles.
static hipError_t persistent_grid(int ntiles, int max_workgroups, int &grid)
{
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess)
        return e;
    grid = cus > 0 ? cus : 1;
    if (max_workgroups > 0 && max_workgroups < grid)
        grid = max_workgroups;
    if (ntiles < grid)
        grid = ntiles;
    return hipSuccess;
}

// The K-step schedule that spreads the requests over the step is the faster one on an MI355X wherever
// its spacing fits the tile (measured on the 8B-class layer shapes: +3 % over issuing them in bursts).
template <class Cfg> constexpr bool spread_fits()
{
    return 2 * Cfg::NB + 2 + 4 * (Cfg::NA - 1) < (Cfg::TN - 1) * Cfg::TM;
}
// The schedule of a configuration: the default spacing where it fits, else (two more requests per operand
// with MXFP4's second scale dword) A requests behind every 3rd MFMA pair, else bursts (0).
template <class Cfg> constexpr int sched_for()
{
    if (spread_fits<Cfg>())
        return MXFP8_GEMM_SCHED;
    return 2 * Cfg::NB + 2 + 3 * (Cfg::NA - 1) < (Cfg::TN - 1) * Cfg::TM ? 232 : 0;
}

template <class Cfg, bool OUT_BF16, bool TILED>
static hipError_t launch_cfg(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                             int M, int N, int K, void *c, int64_t ldc, int max_workgroups, hipStream_t stream)
{
    const int tiles_m = (M + Cfg::BM - 1) / Cfg::BM, tiles_n = (N + Cfg::BN - 1) / Cfg::BN;
    const int64_t ldc_bytes = ldc * (OUT_BF16 ? 2 : 4);
    // 128-bit (FP32) / 64-bit (BF16) stores need every row start aligned; otherwise element stores
    const bool vec_store = (reinterpret_cast<uintptr_t>(c) % 16 == 0) && (ldc_bytes % 16 == 0);
    // Problems made of full tiles run on the persistent kernel (its epilogue addresses a tile's rows with
    // 32-bit offsets from the tile origin); everything else takes one workgroup per tile.
    if (M % Cfg::BM == 0 && N % Cfg::BN == 0 && K >= 2 * BK && vec_store && ldc_bytes * Cfg::BM < (int64_t(1) << 31)) {
        int grid = 0;
        hipError_t e = persistent_grid(tiles_m * tiles_n, max_workgroups, grid);
        if (e != hipSuccess)
            return e;
        constexpr int sched = sched_for<Cfg>();
        auto kern = gemm_persistent_kernel<Cfg, OUT_BF16, TILED, sched != 0, 0, sched != 0 ? sched : MXFP8_GEMM_SCHED>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                Cfg::LDS_BYTES_PERSISTENT);
        if (e != hipSuccess)
            return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Cfg::THREADS), Cfg::LDS_BYTES_PERSISTENT, stream, a_q, a_s, b_q, b_s, M, N, K,
                           static_cast<uint8_t *>(c), ldc_bytes, tiles_m, tiles_n, static_cast<uint8_t *>(nullptr),
                           static_cast<uint8_t *>(nullptr), static_cast<uint8_t *>(nullptr),
                           static_cast<uint8_t *>(nullptr), GemmGroups{nullptr, 0, 0, 0});
        return hipGetLastError();
    }
    auto kern = gemm_kernel<Cfg, OUT_BF16, TILED>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(Cfg::THREADS), Cfg::LDS_BYTES, stream,
                       a_q, a_s, b_q, b_s, M, N, K, static_cast<uint8_t *>(c), ldc_bytes, tiles_m, tiles_n, vec_store,
                       GemmGroups{nullptr, 0, 0, 0});
    return hipGetLastError();
}

template <class Cfg>
static hipError_t launch_any(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s, int M,
                             int N, int K, void *c, bool c_bf16, bool tiled, int64_t ldc, int max_workgroups,
                             hipStream_t stream)
{
    if (tiled)
        return c_bf16 ? launch_cfg<Cfg, true, true>(a_q, a_s, b_q, b_s, M, N, K, c, ldc, max_workgroups, stream)
                      : launch_cfg<Cfg, false, true>(a_q, a_s, b_q, b_s, M, N, K, c, ldc, max_workgroups, stream);
    return c_bf16 ? launch_cfg<Cfg, true, false>(a_q, a_s, b_q, b_s, M, N, K, c, ldc, max_workgroups, stream)
                  : launch_cfg<Cfg, false, false>(a_q, a_s, b_q, b_s, M, N, K, c, ldc, max_workgroups, stream);
}

hipError_t launch_gemm(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s, int64_t M,
                       int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc, int max_workgroups,
                       hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2>;
    using Small = GemmCfg<128, 128, 2, 2>;
    // Small problems cannot fill 256 compute units with 256x256 tiles.
    const bool big = ((M + 255) / 256) * ((N + 255) / 256) >= 128;
    if (big)
        return launch_any<Big>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, c_bf16, tiled_scales, ldc, max_workgroups,
                               stream);
    return launch_any<Small>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, c_bf16, tiled_scales, ldc, max_workgroups,
                             stream);
}

// Grouped product over expert-sorted rows of A (see GemmGroups). Always the persistent kernel: N a multiple of
// the tile (256 when the problem is large and N allows it, else 128), K >= 2 steps, C vector-storable; returns
// hipErrorInvalidConfiguration (nothing launched) otherwise. The host does not know the number of tiles: the
// grid is one workgroup per compute unit (or max_workgroups), capped by the largest number there can be.
template <class Cfg, bool OUT_BF16, bool TILED>
static hipError_t launch_grouped_cfg(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                                     const GemmGroups &groups, int M, int N, int K, void *c, int64_t ldc,
                                     int max_workgroups, hipStream_t stream)
{
    const int64_t ldc_bytes = ldc * (OUT_BF16 ? 2 : 4);
    const bool vec_store = (reinterpret_cast<uintptr_t>(c) % 16 == 0) && (ldc_bytes % 16 == 0);
    if (N % Cfg::BN || K < 2 * BK || !vec_store || ldc_bytes * Cfg::BM >= (int64_t(1) << 31))
        return hipErrorInvalidConfiguration;
    const int tiles_n = N / Cfg::BN;
    const int64_t most_tiles = ((int64_t)(M + Cfg::BM - 1) / Cfg::BM + groups.count) * tiles_n;
    int grid = 0;
    hipError_t e = persistent_grid((int)(most_tiles < 0x7FFFFFFF ? most_tiles : 0x7FFFFFFF), max_workgroups, grid);
    if (e != hipSuccess)
        return e;
    auto kern = gemm_persistent_kernel<Cfg, OUT_BF16, TILED, spread_fits<Cfg>(), 0, MXFP8_GEMM_SCHED, true>;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            Cfg::LDS_BYTES_PERSISTENT);
    if (e != hipSuccess)
        return e;
    uint8_t *none = nullptr;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Cfg::THREADS), Cfg::LDS_BYTES_PERSISTENT, stream, a_q, a_s, b_q, b_s, M, N, K,
                       static_cast<uint8_t *>(c), ldc_bytes, 0, tiles_n, none, none, none, none, groups);
    return hipGetLastError();
}

// Weight-gradient form of the grouped product (see gemm_kernel, KGROUPED): one workgroup per (expert, tile).
template <class Cfg, bool OUT_BF16, bool TILED>
static hipError_t launch_kgrouped_cfg(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                                      const GemmGroups &groups, int M, int N, int K, void *c, int64_t ldc, hipStream_t stream)
{
    const int tiles_m = (M + Cfg::BM - 1) / Cfg::BM, tiles_n = (N + Cfg::BN - 1) / Cfg::BN;
    const int64_t ldc_bytes = ldc * (OUT_BF16 ? 2 : 4);
    const bool vec_store = (reinterpret_cast<uintptr_t>(c) % 16 == 0) && (ldc_bytes % 16 == 0) && ((int64_t)M * ldc_bytes) % 16 == 0;
    const int64_t grid = (int64_t)groups.count * tiles_m * tiles_n;
    if (grid > 0x7FFFFFFF)
        return hipErrorInvalidConfiguration;
    auto kern = gemm_kernel<Cfg, OUT_BF16, TILED, true>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Cfg::THREADS), Cfg::LDS_BYTES, stream, a_q, a_s, b_q, b_s, M, N, K,
                       static_cast<uint8_t *>(c), ldc_bytes, tiles_m, tiles_n, vec_store, groups);
    return hipGetLastError();
}

hipError_t launch_gemm_kgrouped(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                                const int32_t *group_ends, int groups, int64_t M, int64_t N, int64_t K, void *c, bool c_bf16,
                                bool tiled_scales, int64_t ldc, hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2>;
    using Small = GemmCfg<128, 128, 2, 2>;
    const GemmGroups g{group_ends, groups, 0, 0};
    const bool big = ((M + 255) / 256) * ((N + 255) / 256) * groups >= 128;
    const int m = (int)M, n = (int)N, k = (int)K;
#define MXFP8_KGROUPED(CFG)                                                                                        \
    (c_bf16 ? (tiled_scales ? launch_kgrouped_cfg<CFG, true, true>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, stream)   \
                            : launch_kgrouped_cfg<CFG, true, false>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, stream)) \
            : (tiled_scales ? launch_kgrouped_cfg<CFG, false, true>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, stream)  \
                            : launch_kgrouped_cfg<CFG, false, false>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, stream)))
    return big ? MXFP8_KGROUPED(Big) : MXFP8_KGROUPED(Small);
#undef MXFP8_KGROUPED
}

hipError_t launch_gemm_grouped(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                               const int32_t *group_ends, int groups, int64_t b_group_bytes, int64_t bs_group_bytes,
                               int64_t M, int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc,
                               int max_workgroups, hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2>;
    using Small = GemmCfg<128, 128, 2, 2>;
    const GemmGroups g{group_ends, groups, b_group_bytes, bs_group_bytes};
    const bool big = N % 256 == 0 && ((M + 255) / 256) * (N / 256) >= 128;
    const int m = (int)M, n = (int)N, k = (int)K;
#define MXFP8_GROUPED(CFG)                                                                                                     \
    (c_bf16 ? (tiled_scales ? launch_grouped_cfg<CFG, true, true>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, max_workgroups, stream)   \
                            : launch_grouped_cfg<CFG, true, false>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, max_workgroups, stream)) \
            : (tiled_scales ? launch_grouped_cfg<CFG, false, true>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, max_workgroups, stream)  \
                            : launch_grouped_cfg<CFG, false, false>(a_q, a_s, b_q, b_s, g, m, n, k, c, ldc, max_workgroups, stream)))
    return big ? MXFP8_GROUPED(Big) : MXFP8_GROUPED(Small);
#undef MXFP8_GROUPED
}

// MXFP8 product with the element format of each operand chosen by the caller (E4M3 or E5M2: Section 3.2.2).
template <bool A5, bool B5>
static hipError_t launch_gemm_elements_t(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s, int64_t M,
                                         int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc,
                                         int max_workgroups, hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2, kFmtFp8, A5, B5>;
    using Small = GemmCfg<128, 128, 2, 2, kFmtFp8, A5, B5>;
    const bool big = ((M + 255) / 256) * ((N + 255) / 256) >= 128;
    if (big)
        return launch_any<Big>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, c_bf16, tiled_scales, ldc, max_workgroups, stream);
    return launch_any<Small>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)K, c, c_bf16, tiled_scales, ldc, max_workgroups, stream);
}

hipError_t launch_gemm_elements(const uint8_t *a_q, const uint8_t *a_s, bool a_e5m2, const uint8_t *b_q, const uint8_t *b_s,
                                bool b_e5m2, int64_t M, int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc,
                                int max_workgroups, hipStream_t stream)
{
    if (a_e5m2)
        return b_e5m2 ? launch_gemm_elements_t<true, true>(a_q, a_s, b_q, b_s, M, N, K, c, c_bf16, tiled_scales, ldc, max_workgroups, stream)
                      : launch_gemm_elements_t<true, false>(a_q, a_s, b_q, b_s, M, N, K, c, c_bf16, tiled_scales, ldc, max_workgroups, stream);
    if (b_e5m2)
        return launch_gemm_elements_t<false, true>(a_q, a_s, b_q, b_s, M, N, K, c, c_bf16, tiled_scales, ldc, max_workgroups, stream);
    return launch_gemm(a_q, a_s, b_q, b_s, M, N, K, c, c_bf16, tiled_scales, ldc, max_workgroups, stream);
}

// Product of two MXFP4 operands (Table 1: E2M1 elements, two per byte), [M x K/2] and [N x K/2] bytes with K/32
// scale bytes per row: the same block-scaled sum (Section 2, Appendix A.3) on the 4-bit form of the scaled matrix
// instruction. K is counted in elements here and in bytes inside the kernels.
hipError_t launch_gemm_fp4(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s, int64_t M,
                           int64_t N, int64_t K, void *c, bool c_bf16, bool tiled_scales, int64_t ldc, int max_workgroups,
                           hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2, kFmtFp4>;
    using Small = GemmCfg<128, 128, 2, 2, kFmtFp4>;
    const bool big = ((M + 255) / 256) * ((N + 255) / 256) >= 128;
    if (big)
        return launch_any<Big>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)(K / 2), c, c_bf16, tiled_scales, ldc, max_workgroups,
                               stream);
    return launch_any<Small>(a_q, a_s, b_q, b_s, (int)M, (int)N, (int)(K / 2), c, c_bf16, tiled_scales, ldc, max_workgroups,
                             stream);
}

// Product of two BF16 operands, [M x K] and [N x K], both K-contiguous, FP32 accumulation: the GEMM of the
// simulated path (Section 3.1). Same kernels as the MXFP8 product with the BF16 matrix instruction and no
// scales; K is counted in elements here and in bytes inside the kernels.
hipError_t launch_gemm_bf16(const uint8_t *a, const uint8_t *b, int64_t M, int64_t N, int64_t K, void *c, bool c_bf16,
                            int64_t ldc, int max_workgroups, hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2, kFmtBf16>;
    using Small = GemmCfg<128, 128, 2, 2, kFmtBf16>;
    const bool big = ((M + 255) / 256) * ((N + 255) / 256) >= 128;
    const uint8_t *none = nullptr;
    const int m = (int)M, n = (int)N, kbytes = (int)(2 * K);
    if (big)
        return c_bf16 ? launch_cfg<Big, true, false>(a, none, b, none, m, n, kbytes, c, ldc, max_workgroups, stream)
                      : launch_cfg<Big, false, false>(a, none, b, none, m, n, kbytes, c, ldc, max_workgroups, stream);
    return c_bf16 ? launch_cfg<Small, true, false>(a, none, b, none, m, n, kbytes, c, ldc, max_workgroups, stream)
                  : launch_cfg<Small, false, false>(a, none, b, none, m, n, kbytes, c, ldc, max_workgroups, stream);
}

// GEMM with BF16 output and MXFP8 copies of that output (axis bit 0: row-wise, bit 1: column-wise) from
// the same epilogue. Runs on the persistent kernel, hence full tiles only: returns
// hipErrorInvalidConfiguration (nothing launched) when M or N is not a multiple of the tile (256 when the
// problem has at least 128 such tiles, else 128) or K has fewer than two steps.
template <class Cfg, bool TILED, int AXIS>
static hipError_t launch_fused_cfg(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                                   int M, int N, int K, void *c, int64_t ldc, uint8_t *cq, uint8_t *cs, uint8_t *cqT,
                                   uint8_t *csT, int max_workgroups, hipStream_t stream)
{
    const int64_t ldc_bytes = ldc * 2;
    if (M % Cfg::BM || N % Cfg::BN || K < 2 * BK || ldc_bytes * Cfg::BM >= (int64_t(1) << 31))
        return hipErrorInvalidConfiguration;
    const int tiles_m = M / Cfg::BM, tiles_n = N / Cfg::BN;
    auto kern = gemm_persistent_kernel<Cfg, true, TILED, spread_fits<Cfg>(), AXIS>;
    int grid = 0;
    hipError_t e = persistent_grid(tiles_m * tiles_n, max_workgroups, grid);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                Cfg::LDS_BYTES_PERSISTENT);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Cfg::THREADS), Cfg::LDS_BYTES_PERSISTENT, stream, a_q, a_s, b_q, b_s, M, N, K,
                       static_cast<uint8_t *>(c), ldc_bytes, tiles_m, tiles_n, cq, cs, cqT, csT, GemmGroups{nullptr, 0, 0, 0});
    return hipGetLastError();
}

template <class Cfg, bool TILED, class... Args> static hipError_t launch_fused_axis(int axis, Args... args)
{
    switch (axis) {
    case 1: return launch_fused_cfg<Cfg, TILED, 1>(args...);
    case 2: return launch_fused_cfg<Cfg, TILED, 2>(args...);
    default: return launch_fused_cfg<Cfg, TILED, 3>(args...);
    }
}

hipError_t launch_gemm_fused(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q, const uint8_t *b_s,
                             int64_t M, int64_t N, int64_t K, void *c, int64_t ldc, int axis, uint8_t *cq,
                             uint8_t *cs, uint8_t *cqT, uint8_t *csT, bool tiled_scales, int max_workgroups,
                             hipStream_t stream)
{
    using Big = GemmCfg<256, 256, 2, 2>;
    using Small = GemmCfg<128, 128, 2, 2>;
    const bool big = ((M + 255) / 256) * ((N + 255) / 256) >= 128;
    const int m = (int)M, n = (int)N, k = (int)K;
    if (big)
        return tiled_scales ? launch_fused_axis<Big, true>(axis, a_q, a_s, b_q, b_s, m, n, k, c, ldc, cq, cs, cqT, csT, max_workgroups, stream)
                            : launch_fused_axis<Big, false>(axis, a_q, a_s, b_q, b_s, m, n, k, c, ldc, cq, cs, cqT, csT, max_workgroups, stream);
    return tiled_scales ? launch_fused_axis<Small, true>(axis, a_q, a_s, b_q, b_s, m, n, k, c, ldc, cq, cs, cqT, csT, max_workgroups, stream)
                        : launch_fused_axis<Small, false>(axis, a_q, a_s, b_q, b_s, m, n, k, c, ldc, cq, cs, cqT, csT, max_workgroups, stream);
}

}  // namespace mxfp8
