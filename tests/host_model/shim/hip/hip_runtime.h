// Stand-in for <hip/hip_runtime.h> when the kernel sources of this library are compiled as host
// C++ for the CPU execution model in tests/host_model/wavesim.h (test infrastructure only).
// It supplies the language extensions, vector types, built-in variables, the handful of runtime
// calls the launchers use, and host versions of the gfx950 instructions the kernels call.
#pragma once
#define MXFP8_HOST_MODEL 1

#include "../../wavesim.h"

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __shared__ static  // one workgroup runs at a time, so a static array is that workgroup's LDS

struct alignas(8) uint2 {
    uint32_t x, y;
};
struct alignas(16) uint4 {
    uint32_t x, y, z, w;
};
struct alignas(16) float4 {
    float x, y, z, w;
};
inline uint2 make_uint2(uint32_t x, uint32_t y) { return uint2{x, y}; }
inline uint4 make_uint4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) { return uint4{x, y, z, w}; }
inline float4 make_float4(float x, float y, float z, float w) { return float4{x, y, z, w}; }

template <class T> constexpr T min(T a, T b) { return b < a ? b : a; }
template <class T> constexpr T max(T a, T b) { return a < b ? b : a; }

inline float __uint_as_float(uint32_t u)
{
    float f;
    memcpy(&f, &u, 4);
    return f;
}
inline uint32_t __float_as_uint(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

#define threadIdx (::wavesim::me().tid)
#define blockIdx (::wavesim::g.bid)
#define blockDim (::wavesim::g.block)
#define gridDim (::wavesim::g.grid)
#define __syncthreads() ::wavesim::block_sync()
#define __shfl_xor(v, mask, width) ::wavesim::shfl_xor((v), (mask))

#define __builtin_amdgcn_readfirstlane(x) ::wavesim::readfirstlane(x)
#define __builtin_amdgcn_s_waitcnt(imm) ::wavesim::s_waitcnt(imm)
#define __builtin_amdgcn_sched_barrier(mask) ((void)0)
#define __builtin_amdgcn_s_barrier() ::wavesim::block_sync()
#define __builtin_amdgcn_wave_barrier() ::wavesim::wave_sync()
#define __builtin_amdgcn_update_dpp(old, src, ctrl, row_mask, bank_mask, bound_ctrl) \
    ::wavesim::update_dpp((old), (src), (ctrl), (row_mask), (bank_mask), (bound_ctrl))
#define __builtin_amdgcn_perm(s0, s1, sel) ::wavesim::perm((s0), (s1), (sel))
#define __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(old, a, b, scale, hi) \
    ::wavesim::cvt_scalef32_pk_fp8_f32((old), (a), (b), (scale), (hi))
#define __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(old, p, scale, hi) \
    ::wavesim::cvt_scalef32_pk_fp8_bf16((old), (p), (scale), (hi))
#define __builtin_amdgcn_cvt_pk_f32_fp8(q, hi) ::wavesim::cvt_pk_f32_fp8((q), (hi))
#define __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(a, b, scale) ::wavesim::cvt_scalef32_2xpk16_6bit((a), (b), (scale), 2, 3)
#define __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(a, b, scale) ::wavesim::cvt_scalef32_2xpk16_6bit((a), (b), (scale), 3, 2)
#define __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(old, a, b, scale, sel) \
    ::wavesim::cvt_scalef32_pk_fp4_f32((old), (a), (b), (scale), (sel))
#define __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(old, a, b, scale, hi) \
    ::wavesim::cvt_scalef32_pk_bf8_f32((old), (a), (b), (scale), (hi))
#define __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(old, p, scale, hi) \
    ::wavesim::cvt_scalef32_pk_bf8_bf16((old), (p), (scale), (hi))
#define __builtin_amdgcn_cvt_pk_f32_bf8(q, hi) ::wavesim::cvt_pk_f32_bf8((q), (hi))
#define __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(...) ::wavesim::mfma_scale_16x16x128(__VA_ARGS__)
#define __builtin_amdgcn_mfma_f32_16x16x32_bf16(...) ::wavesim::mfma_16x16x32_bf16(__VA_ARGS__)

// ---- runtime calls of the launchers --------------------------------------------------------------
typedef void *hipStream_t;
enum hipError_t { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorInvalidConfiguration = 9 };
enum hipFuncAttribute { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
inline hipError_t hipFuncSetAttribute(const void *, hipFuncAttribute, int) { return hipSuccess; }
inline hipError_t hipGetLastError() { return hipSuccess; }
enum hipDeviceAttribute_t { hipDeviceAttributeMultiprocessorCount = 63 };
inline hipError_t hipGetDevice(int *dev)
{
    *dev = 0;
    return hipSuccess;
}
inline hipError_t hipDeviceGetAttribute(int *value, hipDeviceAttribute_t, int)
{
    const char *e = getenv("WAVESIM_CUS");  // tests shrink the device so that persistent grids loop at small sizes
    *value = e ? atoi(e) : 256;              // compute units of an MI355X
    return hipSuccess;
}
#define hipLaunchKernelGGL(kern, grid, block, shmem, stream, ...)                            \
    do {                                                                                     \
        (void)(stream);                                                                      \
        ::wavesim::launch((grid), (block), (shmem), [=]() { kern(__VA_ARGS__); });           \
    } while (0)

// ---- the pieces of mxfp8_device.h that exist only on the GPU -----------------------------------
#define MXFP8_KEEP_IN_ACC(x) ((void)0)  // a register-allocation hint
// dynamic LDS: the block allocated for this launch
#define MXFP8_DYNAMIC_LDS(name) uint8_t *const name = ::wavesim::g.lds
namespace mxfp8 {
template <int BYTES> inline void dma_load(const uint8_t *base, uint32_t voff, uint32_t lds_addr)
{
    static_assert(BYTES == 4 || BYTES == 16, "dword or dwordx4");
    ::wavesim::dma_issue(base, voff, lds_addr, BYTES);
}
}  // namespace mxfp8
