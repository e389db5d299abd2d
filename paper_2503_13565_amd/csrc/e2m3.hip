// A 6-bit draft format on the same path (arXiv 2503.13565, sections 1 and 5: other bit widths as
// drop-ins for the 4-bit draft; the cast is the two-step rule of section 3.4.3): E2M3 elements
// (1 sign, 2 exponent bits with bias 1, 3 mantissa bits, magnitudes m/8 and (1 + m/8) 2^(e-1),
// largest 7.5, no infinities, no NaN), one E8M0 scale per 32 elements along K.
// Layout: the 32 codes (sign << 5 | eemmm) of a block are a little-endian bit string of 192 bits,
// code i in bits 6i .. 6i+5: q6 [N, K/32 * 24] bytes; scales [N, K/32].  6.25 bits per weight.
//
// gfx950 converts a whole block at once: v_cvt_scalef32_pk32_fp6_bf16 (32 BF16 in 16 registers ->
// 6 registers of codes) and v_cvt_scalef32_pk32_bf16_fp6 back, both with the block's scale.  One
// lane therefore owns a block in the cast (64 bytes in, 24 bytes out) as it does in the product
// (gemv_reg.hip, where a lane's 24-byte load and one convert replace the 16-byte load and the
// eight converts of the 4-bit format).  The integer rule gives the same bits.
#include "common.h"
#include "kernels.h"

namespace mxfp4 {

namespace {

typedef __attribute__((ext_vector_type(32))) __bf16 bf16x32_t;
typedef __attribute__((ext_vector_type(6))) unsigned int u32x6_t;
typedef __attribute__((ext_vector_type(16))) unsigned int u32x16_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;

// Code (eemmm) of one element from its 15 magnitude bits and the block's scale byte.  With sig the
// 8-bit significand, r = |v| / X = sig * 2^(e - 7), e = exponent field - scale byte (<= 2).  F is r
// in units of 2^-14; the quantum of E2M3 is 1/8 below 2 and doubles per binade above; F is rounded
// to it to nearest even and re-based to the code, saturating at 31 (7.5).
__device__ __forceinline__ uint32_t quantise_e2m3(uint32_t mag, int scale_byte)
{
    const uint32_t exp = mag >> 7;
    const uint32_t man = mag & 0x7Fu;
    const uint32_t sig = exp ? (0x80u | man) : man;
    const int sh = (int)(exp ? exp : 1u) - scale_byte + 7;
    if (sh < 0 || sig == 0u)
        return 0u;                                   // below 2^-7: rounds to zero
    const uint32_t F = sig << sh;                    // sh <= 9: below 2^17
    const int top = 31 - __clz((int)F);
    const int shq = (top > 14 ? top : 14) - 3;       // log2 of the quantum in F units
    const uint32_t rounded = (F + ((1u << (shq - 1)) - 1u) + ((F >> shq) & 1u)) >> shq;
    const uint32_t code = rounded + ((uint32_t)(shq - 11) << 3);
    return code > 31u ? 31u : code;
}

// One lane casts one 32-element block.
template <bool kHw>
__global__ __launch_bounds__(256) void e2m3_cast_kernel(const uint16_t* __restrict__ w, int64_t n_rows, int k,
                                                        int64_t ldw, u32x2_t* __restrict__ q6,
                                                        uint8_t* __restrict__ s)
{
    const int nblk = k >> 5;
    const int64_t total = n_rows * nblk;
    for (int64_t blk = (int64_t)blockIdx.x * 256 + threadIdx.x; blk < total; blk += (int64_t)gridDim.x * 256) {
        const int64_t row = blk / nblk;
        const u32x4_t* src = reinterpret_cast<const u32x4_t*>(w + row * ldw + (blk - row * nblk) * 32);
        uint32_t d[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const u32x4_t v = __builtin_nontemporal_load(src + i);
            d[4 * i] = v[0];
            d[4 * i + 1] = v[1];
            d[4 * i + 2] = v[2];
            d[4 * i + 3] = v[3];
        }
        uint32_t amax = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            amax = max(amax, max(d[i] & 0x7FFFu, (d[i] >> 16) & 0x7FFFu));
        uint32_t out[6] = {0u, 0u, 0u, 0u, 0u, 0u};
        int scale_byte;
        if (amax >= 0x7F80u) {
            scale_byte = 0xFF;                       // NaN or Inf in the block
        } else {
            scale_byte = (int)(amax >> 7) - 2;       // biased exponent of amax, minus 2
            scale_byte = scale_byte < 0 ? 0 : scale_byte;
            if constexpr (kHw) {
                // the magnitudes are clamped to 7.5 X first, so the convert never sees an overflow
                const uint32_t top = (((uint32_t)scale_byte + 2u) << 7) | 0x70u;
                u32x16_t c;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t lo = min(d[i] & 0x7FFFu, top) | (d[i] & 0x8000u);
                    const uint32_t hi = min((d[i] >> 16) & 0x7FFFu, top) | ((d[i] >> 16) & 0x8000u);
                    c[i] = lo | (hi << 16);
                }
                const float scale = __uint_as_float((uint32_t)scale_byte << 23);
                const u32x6_t r = __builtin_amdgcn_cvt_scalef32_pk32_fp6_bf16(__builtin_bit_cast(bf16x32_t, c), scale);
#pragma unroll
                for (int i = 0; i < 6; ++i)
                    out[i] = r[i];
            } else {
#pragma unroll
                for (int e = 0; e < 32; ++e) {
                    const uint32_t h = (e & 1) ? d[e >> 1] >> 16 : d[e >> 1] & 0xFFFFu;
                    const uint32_t code = quantise_e2m3(h & 0x7FFFu, scale_byte) | ((h >> 15) << 5);
                    const int bit = 6 * e, dw = bit >> 5, sft = bit & 31;
                    out[dw] |= code << sft;
                    if (sft > 26)
                        out[dw + 1] |= code >> (32 - sft);
                }
            }
        }
        q6[blk * 3] = u32x2_t{out[0], out[1]};
        q6[blk * 3 + 1] = u32x2_t{out[2], out[3]};
        q6[blk * 3 + 2] = u32x2_t{out[4], out[5]};
        s[blk] = (uint8_t)scale_byte;
    }
}

// q6, s -> BF16 (exact while the product is a normal BF16): one lane per block, by the scaled
// FP6->BF16 convert, so that the instruction's semantics can be checked in isolation.
__global__ __launch_bounds__(256) void e2m3_dequant_kernel(const u32x2_t* __restrict__ q6,
                                                           const uint8_t* __restrict__ s, int64_t n_rows, int k,
                                                           uint16_t* __restrict__ w, int64_t ldw)
{
    const int nblk = k >> 5;
    const int64_t total = n_rows * nblk;
    const int64_t blk = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blk >= total)
        return;
    const int64_t row = blk / nblk;
    const u32x2_t a = q6[blk * 3], b = q6[blk * 3 + 1], c = q6[blk * 3 + 2];
    const u32x6_t packed = {a[0], a[1], b[0], b[1], c[0], c[1]};
    const float scale = e8m0_to_f32(s[blk]);
    const u32x16_t out = __builtin_bit_cast(u32x16_t, __builtin_amdgcn_cvt_scalef32_pk32_bf16_fp6(packed, scale));
    uint4* dst = reinterpret_cast<uint4*>(w + row * ldw + (blk - row * nblk) * 32);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        dst[i] = make_uint4(out[4 * i], out[4 * i + 1], out[4 * i + 2], out[4 * i + 3]);
}

}  // namespace

hipError_t launch_e2m3_cast(const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q6, void* s,
                            bool integer_rule, hipStream_t stream)
{
    const int64_t total = n_rows * (k / 32);
    if (total == 0)
        return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 8)
        blocks = 256 * 8;
    auto kern = integer_rule ? e2m3_cast_kernel<false> : e2m3_cast_kernel<true>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t*)w, n_rows, (int)k, ldw,
                       (u32x2_t*)q6, (uint8_t*)s);
    return hipGetLastError();
}

hipError_t launch_e2m3_dequant(const void* q6, const void* s, int64_t n_rows, int64_t k, void* w, int64_t ldw,
                               hipStream_t stream)
{
    const int64_t total = n_rows * (k / 32);
    if (total == 0)
        return hipSuccess;
    hipLaunchKernelGGL(e2m3_dequant_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const u32x2_t*)q6, (const uint8_t*)s, n_rows, (int)k, (uint16_t*)w, ldw);
    return hipGetLastError();
}

}  // namespace mxfp4
