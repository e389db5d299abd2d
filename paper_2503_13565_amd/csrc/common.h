// Device-side helpers shared by the gfx950 kernels of the MXFP4 weight-only-quantised
// linear layer (arXiv 2503.13565, section 3.4.3).  Wave size is 64 everywhere.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <atomic>

namespace mxfp4 {

constexpr int kWave = 64;
constexpr int kBlockElems = 32;      // elements per scale block along K
constexpr int kBlockBytes = 16;      // packed bytes per scale block

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// E8M0 scale byte -> FP32 2^(byte-127).  Byte 0 is 2^-127 (an FP32 subnormal), byte 0xFF is NaN.
__device__ __forceinline__ float e8m0_to_f32(uint32_t byte)
{
    uint32_t bits = byte << 23;
    bits = (byte == 0u) ? 0x00400000u : bits;
    bits = (byte == 0xFFu) ? 0x7FC00000u : bits;
    return __uint_as_float(bits);
}

// FP32 -> BF16 bit pattern, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// The gate of the gated MLP: silu(g) * u with silu(g) = g / (1 + e^-g), in FP32.  The limits
// come out of the arithmetic: e^-g = inf gives -0 for very negative g, e^-g = 0 gives g.
__device__ __forceinline__ float silu_gate(float g, float u) { return g / (1.f + __expf(-g)) * u; }

// One E2M1 nibble (sign<<3 | eem) -> FP32, by bit assembly: codes 0 and 1 are 0 and 0.5, a
// normal code eem is 1.m * 2^(ee-1).
__device__ __forceinline__ float e2m1_to_f32(uint32_t nib)
{
    uint32_t c = nib & 7u;
    uint32_t bits = (((c >> 1) + 126u) << 23) | ((c & 1u) << 22);
    bits = (c == 1u) ? 0x3F000000u : bits;
    bits = (c == 0u) ? 0u : bits;
    return __uint_as_float(bits | ((nib & 8u) << 28));
}

template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kCtrl, 0xF, 0xF, false));
}

// Sum over the 64 lanes of a wave in a fixed order; every lane returns the total.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_f32<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f32<0x141>(v);   // row_half_mirror
    v += dpp_f32<0x140>(v);   // row_mirror: all 16 lanes of a row now hold the row's sum
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// Workgroup barrier that waits for LDS traffic only.  __syncthreads() would also drain the
// vector-memory counter and with it the weight loads that are deliberately in flight.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

typedef __attribute__((ext_vector_type(2))) unsigned short u16x2_t;

// Sixteen codes of the 2-bit format (one dword, code j in bits 2j, 2j + 1) -> eight BF16 pairs.  A
// code is sign << 1 | magnitude, which are the top two bits of the BF16 number +-2.0 or +-0: a
// pair of codes moves to bits 15:14 and 31:30 of a dword by one packed 16-bit shift of the half that
// holds them, and a mask.  The product then carries 2 X per unit and is scaled by X / 2 afterwards.
__device__ __forceinline__ void decode_t2(uint32_t c, uint32_t* out8)
{
    const uint32_t lo = __builtin_amdgcn_perm(c, c, 0x01000100u);   // codes 0..7 in both halves
    const uint32_t hi = __builtin_amdgcn_perm(c, c, 0x03020302u);   // codes 8..15 in both halves
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const u16x2_t sh = {(unsigned short)(14 - 4 * p), (unsigned short)(12 - 4 * p)};
        const u16x2_t a = __builtin_bit_cast(u16x2_t, lo) << sh;
        const u16x2_t b = __builtin_bit_cast(u16x2_t, hi) << sh;
        out8[p] = __builtin_bit_cast(uint32_t, a) & 0xC000C000u;
        out8[4 + p] = __builtin_bit_cast(uint32_t, b) & 0xC000C000u;
    }
}

// Wait until every vector-memory operation of this wave has completed (s_waitcnt vmcnt(0),
// other counters untouched; gfx9 encoding).  A real waitcnt instruction rather than inline
// assembly, so that the compiler's own wait insertion knows nothing is pending afterwards.
__device__ __forceinline__ void drain_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Host side: a measurement switch (an environment variable that picks a launch shape or a kernel so
// that two of them can be timed in one run).  The library as shipped reads none of them; they exist
// only in builds with -DMXFP4_MEASUREMENT_KNOBS.
inline const char* knob(const char* name)
{
#ifdef MXFP4_MEASUREMENT_KNOBS
    return getenv(name);
#else
    (void)name;
    return nullptr;
#endif
}

// Host side: lets a kernel use more than the default 64 KiB of dynamic LDS.  The attribute belongs
// to the kernel on the current device, so there is one flag per device; each kernel instance keeps a
// static object of its own.  Threads that race here set the same attribute twice, which is harmless.
struct LdsLimit {
    static constexpr int kDevices = 64;
    std::atomic<bool> done[kDevices] = {};
    hipError_t raise(const void* kernel, int bytes)
    {
        int d = 0;
        hipError_t e = hipGetDevice(&d);
        if (e != hipSuccess)
            return e;
        const bool tracked = d >= 0 && d < kDevices;
        if (tracked && done[d].load(std::memory_order_relaxed))
            return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess && tracked)
            done[d].store(true, std::memory_order_relaxed);
        return e;
    }
};

}  // namespace mxfp4
