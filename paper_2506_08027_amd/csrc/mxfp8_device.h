// Device-side helpers shared by the MXFP8 kernels (gfx950 only).
//
// Number formats (Section 2, Table 1): elements are OCP E4M3 (1-4-3, bias 7, max 448, NaN =
// S.1111.111); a scale byte s stands for X = 2^(s-127), 0xFF for NaN; blocks have 32 elements.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mxfp8 {

typedef short v2s __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef unsigned short v2us __attribute__((ext_vector_type(2)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kBlock = 32;

// ---- cross-lane moves inside a row of 16 lanes (DPP, no LDS traffic) -------------------------
// quad_perm [1,0,3,2] / [2,3,0,1]: exchange with lane^1 / lane^2; row_half_mirror: lane i <-> 7-i
// inside each group of 8 (after the two quad steps every lane of a quad holds the quad result, so
// the mirror delivers the other quad of the same 8 lanes).
__device__ __forceinline__ uint32_t dpp_xor1(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t dpp_xor2(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t dpp_half_mirror(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true);
}

// row_mirror: lane i <-> 15-i inside a row of 16 lanes (after a reduction over each group of 8 this
// delivers the other group)
__device__ __forceinline__ uint32_t dpp_mirror(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true);
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// max of the two 16-bit halves, both halves at once (v_pk_max_u16)
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    v2us x = __builtin_bit_cast(v2us, a), y = __builtin_bit_cast(v2us, b);
    v2us r = __builtin_elementwise_max(x, y);
    return __builtin_bit_cast(uint32_t, r);
}

// ---- scale byte from the block amax, in the bit space (Algorithm 1 / Appendix A.1) ----------
// For amax = 1.m * 2^(e-127) the smallest n with amax <= 448 * 2^n is e-127-8, plus one when
// 1.m > 1.75; adding (2.0 - 1.75) - 1ulp to the mantissa carries into the exponent field exactly
// in that case. The lower clamp (byte 0 = 2^-127) covers zero and every FP32 subnormal.
// abs_bits = |amax| as FP32 bits. Inf -> 254 (the clamp of Algorithm 1), NaN -> 0xFF.
__device__ __forceinline__ uint32_t scale_byte_from_f32_bits(uint32_t abs_bits)
{
    int s = (int)((abs_bits + 0x1FFFFFu) >> 23) - 8;
    s = s < 0 ? 0 : s;
    if (abs_bits >= 0x7F800000u)
        s = abs_bits > 0x7F800000u ? 0xFF : 254;
    return (uint32_t)s;
}
// Same rule on BF16 bits (the upper half of the FP32 pattern; the lower mantissa bits are zero).
__device__ __forceinline__ uint32_t scale_byte_from_bf16_bits(uint32_t abs_bits16)
{
    int s = (int)((abs_bits16 + 0x1Fu) >> 7) - 8;
    s = s < 0 ? 0 : s;
    if (abs_bits16 >= 0x7F80u)
        s = abs_bits16 > 0x7F80u ? 0xFF : 254;
    return (uint32_t)s;
}

// ---- ablation arms (Table 1: E5M2 elements; Section 3.3: the OCP v1 scale rule the recipe replaces) ----
// MODE bit 0: elements are E5M2 (1-5-2, bias 15, max 57344 = 1.75 * 2^15, code 0x7B) instead of E4M3;
// MODE bit 1: the scale exponent is floor(log2(amax)) - emax (amax / max rounded DOWN to a power of two)
//             instead of Algorithm 1's round-up, so that block maxima above 1.75 * 2^e saturate.
// MODE 0 is the recipe and takes the functions above.
constexpr int kModeE5M2 = 1, kModeOcpRule = 2;
template <int MODE> constexpr uint32_t max_code() { return (MODE & kModeE5M2) ? 0x7Bu : 0x7Eu; }
template <int MODE> constexpr int emax() { return (MODE & kModeE5M2) ? 15 : 8; }
template <int MODE> __device__ __forceinline__ uint32_t scale_byte_mode_f32_bits(uint32_t abs_bits)
{
    // round-up rule: the mantissa carry of Algorithm 1's bit form; OCP rule: the exponent field itself
    int s = (int)(((MODE & kModeOcpRule) ? abs_bits : abs_bits + 0x1FFFFFu) >> 23) - emax<MODE>();
    s = s < 0 ? 0 : s;
    if (abs_bits >= 0x7F800000u)
        s = abs_bits > 0x7F800000u ? 0xFF : 254;
    return (uint32_t)s;
}
template <int MODE> __device__ __forceinline__ uint32_t scale_byte_mode_bf16_bits(uint32_t abs_bits16)
{
    int s = (int)(((MODE & kModeOcpRule) ? abs_bits16 : abs_bits16 + 0x1Fu) >> 7) - emax<MODE>();
    s = s < 0 ? 0 : s;
    if (abs_bits16 >= 0x7F80u)
        s = abs_bits16 > 0x7F80u ? 0xFF : 254;
    return (uint32_t)s;
}

// The conversion instructions divide by 2^(exponent field of the scale operand - 127) and read an
// exponent field of 0 as 2^-127, so the scale byte shifted into the exponent field is the operand.
__device__ __forceinline__ float scale_operand(uint32_t scale_byte)
{
    return __uint_as_float(scale_byte << 23);
}

// ---- element conversion (Appendix A.2): RNE to E4M3 of V / X --------------------------------
// v_cvt_scalef32_pk_fp8_{f32,bf16} round to nearest even, keep the sign of zero and of
// underflows and produce subnormals, but answer NaN for |V/X| > 464 instead of saturating.
// With the round-up scale no finite block reaches that; only +-Inf inputs do, and those are
// patched to +-448 by the callers (fix_inf_*).
__device__ __forceinline__ uint32_t cvt2_f32(uint32_t old, float a, float b, float scale, bool hi)
{
    v2s o = __builtin_bit_cast(v2s, old);
    v2s r = hi ? __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(o, a, b, scale, true)
               : __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(o, a, b, scale, false);
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint32_t cvt2_bf16(uint32_t old, uint32_t pair, float scale, bool hi)
{
    v2s o = __builtin_bit_cast(v2s, old);
    v2bf p = __builtin_bit_cast(v2bf, pair);
    v2s r = hi ? __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(o, p, scale, true)
               : __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(o, p, scale, false);
    return __builtin_bit_cast(uint32_t, r);
}

// E5M2 forms of the two conversions (v_cvt_scalef32_pk_bf8_{f32,bf16}): same operands, same rounding.
__device__ __forceinline__ uint32_t cvt2_e5m2_f32(uint32_t old, float a, float b, float scale, bool hi)
{
    v2s o = __builtin_bit_cast(v2s, old);
    v2s r = hi ? __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(o, a, b, scale, true)
               : __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(o, a, b, scale, false);
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint32_t cvt2_e5m2_bf16(uint32_t old, uint32_t pair, float scale, bool hi)
{
    v2s o = __builtin_bit_cast(v2s, old);
    v2bf p = __builtin_bit_cast(v2bf, pair);
    v2s r = hi ? __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(o, p, scale, true)
               : __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(o, p, scale, false);
    return __builtin_bit_cast(uint32_t, r);
}

// Saturation for the ablation arms (Appendix A.2: what exceeds the FP8 maximum after rounding is clamped to
// it): the converters answer with a code above the largest finite one (NaN, or Inf for E5M2) whenever the
// scaled value rounds beyond the maximum; such a byte, and the byte of an infinite input, becomes
// sign | largest finite code, the sign taken from the input. Only for blocks without NaN.
template <int MODE> __device__ __forceinline__ uint32_t saturate_byte(uint32_t q, bool negative, bool input_inf)
{
    return ((q & 0x7Fu) > max_code<MODE>() || input_inf) ? (negative ? 0x80u : 0u) | max_code<MODE>() : q;
}

// Saturating rule for infinities: the element byte becomes sign | 0x7E (+-448).
__device__ __forceinline__ uint32_t inf_byte_f32(uint32_t bits, uint32_t q)
{
    return (bits & 0x7FFFFFFFu) == 0x7F800000u ? ((bits >> 24) & 0x80u) | 0x7Eu : q;
}
__device__ __forceinline__ uint32_t inf_byte_bf16(uint32_t bits16, uint32_t q)
{
    return (bits16 & 0x7FFFu) == 0x7F80u ? ((bits16 >> 8) & 0x80u) | 0x7Eu : q;
}

// ---- streaming accesses ------------------------------------------------------------------------
// The quantizer reads its source once and writes its outputs once: nontemporal loads and stores keep that
// stream from displacing other data in the caches (measured on an MI355X: 3-4 % more bandwidth).
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 stream_load(const uint4 *p)
{
    const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void stream_store(uint4 *p, uint4 v)
{
    __builtin_nontemporal_store(v4u{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u *>(p));
}
__device__ __forceinline__ void stream_store(uint2 *p, uint2 v)
{
    __builtin_nontemporal_store(v2u{v.x, v.y}, reinterpret_cast<v2u *>(p));
}
__device__ __forceinline__ void stream_store(uint32_t *p, uint32_t v) { __builtin_nontemporal_store(v, p); }

// ---- what exists only on the GPU --------------------------------------------------------------
// The CPU tests compile these kernel sources as host C++ against an execution model of their own;
// that build defines MXFP8_HOST_MODEL and brings its own versions of the items below.
#ifndef MXFP8_HOST_MODEL
// The workgroup's dynamically sized LDS block (size given at launch).
#define MXFP8_DYNAMIC_LDS(name) extern __shared__ __attribute__((aligned(1024))) uint8_t name[]
// States that x lives in accumulator registers (AGPRs) at this point of the program.
#define MXFP8_KEEP_IN_ACC(x) asm volatile("" : "+a"(x))

// Global memory -> LDS without passing through registers: lane l of the wavefront fetches BYTES
// bytes from base + voff (its own address) and the hardware writes them to LDS address
// lds_addr + l*BYTES (lds_addr is wavefront-uniform and travels in M0).
// Emitted as inline assembly on purpose: the compiler's wait-count pass treats a pending LDS-DMA
// load as "may complete out of order with LDS reads" and then turns every wait on an LDS read
// into a wait for ALL outstanding LDS reads, which would serialise the fragment prefetch.
// Completion is tracked by hand with s_waitcnt vmcnt(n) in front of the barriers.
template <int BYTES>
__device__ __forceinline__ void dma_load(const uint8_t *base, uint32_t voff, uint32_t lds_addr)
{
    const uint32_t m0v = lds_addr;  // callers pass a wavefront-uniform (scalar) address
    static_assert(BYTES == 16 || BYTES == 4, "dword or dwordx4");
    if constexpr (BYTES == 16)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(m0v)
                     : "memory");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(base), "s"(m0v)
                     : "memory");
}
#endif  // MXFP8_HOST_MODEL

}  // namespace mxfp8
