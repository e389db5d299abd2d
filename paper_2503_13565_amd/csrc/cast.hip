// BF16 -> MXFP4 direct cast and its inverse for gfx950 (arXiv 2503.13565, section 3.4.3:
// the two-step quantisation; E2M1 elements, one E8M0 scale per 32 elements along K).
//
// Four lanes share one 32-element block: each lane loads 16 bytes (8 elements), the block maximum
// is taken across the quad with DPP on the integer magnitudes, the scale byte is integer
// arithmetic on the BF16 exponent, and each lane writes one packed dword; a wave therefore reads
// 1 KiB and writes 256 B, contiguous, per piece, and the 64 scale bytes of four pieces as one run.  The elements are rounded by the gfx950 scaled BF16->FP4
// convert, or by an integer-only rule on the bit patterns that gives the same bits.
#include "common.h"
#include "kernels.h"

namespace mxfp4 {

// Code (eem) of one element from its 15 magnitude bits and the block's scale byte.
// With sig the 8-bit significand and d = exponent - scale byte (d <= 2 for every element of
// the block that produced the scale), F = |v|/X in units of 2^-10 is sig << (d+3).  The
// quantum of E2M1 is 0.5 below 2 and doubles per binade above; F is rounded to it to nearest
// even and the result is re-based to the code, saturating at 7.
__device__ __forceinline__ uint32_t quantise_e2m1(uint32_t mag, int scale_byte)
{
    const uint32_t exp = mag >> 7;
    const uint32_t man = mag & 0x7Fu;
    const uint32_t sig = exp ? (0x80u | man) : man;
    const int sh3 = (int)(exp ? exp : 1u) - scale_byte + 3;
    if (sh3 < 0)
        return 0u;                                   // below 2^-3 of X: rounds to zero
    const uint32_t F = sig << sh3;
    const int top = 31 - __clz((int)F);              // -1 for F == 0
    const int shq = (top > 10 ? top : 10) - 1;       // log2 of the quantum in F units
    const uint32_t rounded = (F + ((1u << (shq - 1)) - 1u) + ((F >> shq) & 1u)) >> shq;
    const uint32_t code = rounded + 2u * (uint32_t)(shq - 9);
    return code > 7u ? 7u : code;
}

// One 8-element group (16 bytes of BF16) of a block per lane; the four lanes of a quad hold one
// 32-element block.  kHw: elements are rounded by the gfx950 scaled BF16->FP4 convert (one
// instruction per element pair; checked on the device against the integer rule above for every
// finite BF16 value and every scale byte); otherwise by the integer rule.
template <bool kHw>
__device__ __forceinline__ void cast_group(const u32x4_t v, uint32_t* packed_out, int* scale_out)
{
    const uint32_t d[4] = {v[0], v[1], v[2], v[3]};
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t lo = d[i] & 0x7FFFu, hi = (d[i] >> 16) & 0x7FFFu;
        amax = max(amax, max(lo, hi));
    }
    // block maximum over the 4 lanes of the quad (BF16 magnitude order = integer order)
    amax = max(amax, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)amax, 0xB1, 0xF, 0xF, false));
    amax = max(amax, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)amax, 0x4E, 0xF, 0xF, false));

    uint32_t packed = 0;
    int scale_byte;
    if (amax >= 0x7F80u) {
        scale_byte = 0xFF;                           // NaN or Inf in the block
    } else {
        scale_byte = (int)(amax >> 7) - 2;           // biased exponent of amax, minus 2
        scale_byte = scale_byte < 0 ? 0 : scale_byte;
        if constexpr (kHw) {
            // the convert divides by 2^(exponent field - 127) of its scale operand (field 0 is 2^-127)
            const float scale = __uint_as_float((uint32_t)scale_byte << 23);
            const uint32_t d0 = d[0], d1 = d[1], d2 = d[2], d3 = d[3];
            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, __builtin_bit_cast(bf16x2_t, d0), scale, 0);
            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, __builtin_bit_cast(bf16x2_t, d1), scale, 1);
            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, __builtin_bit_cast(bf16x2_t, d2), scale, 2);
            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, __builtin_bit_cast(bf16x2_t, d3), scale, 3);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = d[i] & 0xFFFFu, hi = d[i] >> 16;
                const uint32_t nlo = quantise_e2m1(lo & 0x7FFFu, scale_byte) | ((lo >> 15) << 3);
                const uint32_t nhi = quantise_e2m1(hi & 0x7FFFu, scale_byte) | ((hi >> 15) << 3);
                packed |= (nlo | (nhi << 4)) << (8 * i);
            }
        }
    }
    *packed_out = packed;
    *scale_out = scale_byte;
}

// Persistent walk over chunks of 256 groups (4 KiB of BF16, 64 blocks): wave w of the grid takes
// chunks w, w + waves, ...; its four loads per lane are the chunk's four consecutive 1 KiB pieces.
// A chunk's 64 scale bytes are contiguous in s: the quads leave them in 64 bytes of LDS of the
// wave's own and lanes 0..3 store them as one 64-byte run (byte stores, 16 per wave instruction,
// cost the memory system a partial write each).  A wave's LDS operations run in order, so no barrier
// is needed.  kFlat: rows are contiguous (ldw == K), so a group's address needs no division.
template <bool kHw, bool kFlat>
__global__ __launch_bounds__(256) void direct_cast_kernel(const uint16_t* __restrict__ w,
                                                          int64_t n_rows, int k, int64_t ldw,
                                                          uint32_t* __restrict__ q,
                                                          uint8_t* __restrict__ s)
{
    constexpr int kU = 4;
    __shared__ __align__(16) uint8_t sbytes[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int groups_per_row = k >> 3;               // 8-element groups; a multiple of 4
    const int64_t total = n_rows * groups_per_row;   // a multiple of 4
    const int64_t chunks = (total + 255) >> 8;
    const int64_t waves = (int64_t)gridDim.x * 4;
    const bool s_aligned = (reinterpret_cast<uintptr_t>(s) & 15) == 0;       // else byte stores throughout
    for (int64_t c = (int64_t)blockIdx.x * 4 + wave; c < chunks; c += waves) {
        const int64_t g0 = c * 256 + lane;
        u32x4_t v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            int64_t gid = g0 + u * 64;
            gid = gid < total ? gid : c * 256;       // surplus slots repeat the chunk's first group (never stored)
            int64_t off = gid * 8;
            if constexpr (!kFlat) {
                const int64_t row = gid / groups_per_row;
                off = row * ldw + (gid - row * groups_per_row) * 8;
            }
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(w + off));
        }
        const bool whole = s_aligned && c * 256 + 256 <= total;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int64_t gid = g0 + u * 64;
            uint32_t packed;
            int scale_byte;
            cast_group<kHw>(v[u], &packed, &scale_byte);   // whole quads take part in the DPP steps
            if (gid < total) {
                __builtin_nontemporal_store(packed, q + gid);
                if ((lane & 3) == 0) {
                    if (whole)
                        sbytes[wave][u * 16 + (lane >> 2)] = (uint8_t)scale_byte;
                    else
                        s[gid >> 2] = (uint8_t)scale_byte;
                }
            }
        }
        if (whole && lane < 4) {
            const u32x4_t line = *reinterpret_cast<const u32x4_t*>(&sbytes[wave][lane * 16]);
            __builtin_nontemporal_store(line, reinterpret_cast<u32x4_t*>(s + c * 64) + lane);
        }
    }
}

// q, s -> BF16 (scale * magnitude, exact while the product is a normal BF16).  One lane per
// packed dword (8 elements).  kHw selects the gfx950 scaled FP4->BF16 convert instead of bit
// assembly, so that the instruction's semantics can be checked in isolation.
template <bool kHw>
__global__ __launch_bounds__(256) void dequant_kernel(const uint32_t* __restrict__ q,
                                                      const uint8_t* __restrict__ s,
                                                      int64_t n_rows, int k, uint16_t* __restrict__ w,
                                                      int64_t ldw)
{
    const int groups_per_row = k >> 3;
    const int64_t total = n_rows * groups_per_row;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total)
        return;
    const int64_t row = gid / groups_per_row;
    const int cg = (int)(gid - row * groups_per_row);
    const uint32_t packed = q[gid];
    const float scale = e8m0_to_f32(s[gid >> 2]);
    uint32_t out[4];
    if constexpr (kHw) {
        bf16x2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(packed, scale, 0);
        bf16x2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(packed, scale, 1);
        bf16x2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(packed, scale, 2);
        bf16x2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(packed, scale, 3);
        out[0] = __builtin_bit_cast(uint32_t, p0);
        out[1] = __builtin_bit_cast(uint32_t, p1);
        out[2] = __builtin_bit_cast(uint32_t, p2);
        out[3] = __builtin_bit_cast(uint32_t, p3);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t byte = (packed >> (8 * i)) & 0xFFu;
            const float lo = e2m1_to_f32(byte & 0xFu) * scale;
            const float hi = e2m1_to_f32(byte >> 4) * scale;
            out[i] = (uint32_t)f32_to_bf16_rne(lo) | ((uint32_t)f32_to_bf16_rne(hi) << 16);
        }
    }
    *reinterpret_cast<uint4*>(w + row * ldw + (int64_t)cg * 8) = make_uint4(out[0], out[1], out[2], out[3]);
}

hipError_t launch_direct_cast(const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q, void* s,
                              bool bits, hipStream_t stream)
{
    const int64_t total = n_rows * (k / 8);
    if (total == 0)
        return hipSuccess;
    int64_t blocks = (total + 1023) / 1024;          // a workgroup's four waves take a chunk of 256 groups each
    static const int per_cu = [] {
        const char* e = knob("MXFP4_CAST_WGS");      // measurement only
        return e && atoi(e) > 0 ? atoi(e) : 8;
    }();
    const int64_t resident = 256 * per_cu;           // 8 workgroups of 4 waves per CU on the target part
    if (blocks > resident)
        blocks = resident;
    const bool flat = ldw == k;
    auto kern = bits ? (flat ? direct_cast_kernel<false, true> : direct_cast_kernel<false, false>)
                     : (flat ? direct_cast_kernel<true, true> : direct_cast_kernel<true, false>);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t*)w, n_rows, (int)k,
                       ldw, (uint32_t*)q, (uint8_t*)s);
    return hipGetLastError();
}

hipError_t launch_dequant(const void* q, const void* s, int64_t n_rows, int64_t k, void* w, int64_t ldw,
                          bool hw_convert, hipStream_t stream)
{
    const int64_t total = n_rows * (k / 8);
    if (total == 0)
        return hipSuccess;
    const int64_t blocks = (total + 255) / 256;
    if (hw_convert)
        hipLaunchKernelGGL(dequant_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const uint32_t*)q, (const uint8_t*)s, n_rows, (int)k, (uint16_t*)w, ldw);
    else
        hipLaunchKernelGGL(dequant_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const uint32_t*)q, (const uint8_t*)s, n_rows, (int)k, (uint16_t*)w, ldw);
    return hipGetLastError();
}

}  // namespace mxfp4
