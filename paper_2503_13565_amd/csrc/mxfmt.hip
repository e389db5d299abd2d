// Further draft formats on the same path (arXiv 2503.13565, sections 1, 3.2 and 5: 8-bit and
// lower-bit quantisation as drop-ins for the 4-bit draft; the cast is the two-step rule of section
// 3.4.3 with another element format, the product is Eq. 2 with FP32 accumulation):
//   id 1  E5M2  1 sign, 5 exponent bits (bias 15), 2 mantissa bits, largest finite 57344; 8 bits
//   id 2  E3M2  1 sign, 3 exponent bits (bias 3), 2 mantissa bits, largest 28, no Inf/NaN; 6 bits
//   id 3  T2    1 sign, 1 magnitude bit: {0, +-1} times the block scale (a ternary draft); 2 bits
// each with one E8M0 scale per 32 elements along K: X = 2^(floor(log2 amax) - emax), emax = 15, 4, 0.
// Layout: the 32 codes of a block (sign in the top bit of a code) are a little-endian bit string,
// code i in bits b i .. b i + b - 1: q [N, K/32 * 4 b] bytes (32, 24, 8 bytes per block), scales
// [N, K/32].  8.25, 6.25 and 2.25 bits per weight.
//
// One lane owns one block everywhere here.  Cast: 64 bytes in, 4 b bytes out; elements by the
// gfx950 scaled converts (v_cvt_scalef32_pk_bf8_bf16, v_cvt_scalef32_pk32_bf6_bf16) after clamping
// to the largest magnitude, or by an ALU rule that gives the same bits (the only rule T2 has).
// Product: the activations sit in LDS as [row][quarter of a block][block], so that the 64 lanes of a
// wave read consecutive 16 bytes; a lane loads its block and scale byte, decodes to 16 BF16 pairs
// (scaled converts for E5M2 and E3M2; T2 by shifts, see decode()) and runs v_dot2_f32_bf16 against
// the block's 32 activations; rows are summed over the wave.  Where a row has fewer than 64 blocks
// and their count is a power of two (K <= 1024: attention-head sized rows) a wave step covers
// 64 / (K/32) rows instead of one, and the sum is over the lanes of a row only.
#include "common.h"
#include "kernels.h"

namespace mxfp4 {

namespace {

typedef __attribute__((ext_vector_type(32))) __bf16 bf16x32_t;
typedef __attribute__((ext_vector_type(2))) short s16x2_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
typedef __attribute__((ext_vector_type(6))) unsigned int u32x6_t;
typedef __attribute__((ext_vector_type(16))) unsigned int u32x16_t;

constexpr int kOobF = 0x7FFFFFF0;        // lane offset beyond any descriptor: the load returns zero

template <int F>
struct Fmt;
template <>
struct Fmt<1> {
    static constexpr int kBits = 8, kMb = 2, kBias = 15, kEmax = 15, kTop = 123;
};
template <>
struct Fmt<2> {
    static constexpr int kBits = 6, kMb = 2, kBias = 3, kEmax = 4, kTop = 31;
};
template <>
struct Fmt<3> {
    static constexpr int kBits = 2, kMb = 1, kBias = 0, kEmax = 0, kTop = 1;
};

// Magnitude code of one element from its 15 BF16 magnitude bits and the block's scale byte.
// r = |v| / X = sig * 2^(e - 7) with sig the 8-bit significand and e = exponent field - scale byte,
// built exactly as an FP32 number.  In the format's normal range the FP32 pattern is rounded to kMb
// mantissa bits to nearest even (a carry moves into the exponent) and re-based; below it the code is
// r in units of the subnormal quantum, rounded to nearest even.  Saturates at the top code.
template <int F>
__device__ __forceinline__ uint32_t quantise(uint32_t mag, int scale_byte)
{
    using T = Fmt<F>;
    const uint32_t exp = mag >> 7;
    const uint32_t man = mag & 0x7Fu;
    const uint32_t sig = exp ? (0x80u | man) : man;
    const int fe = (int)(exp ? exp : 1u) - scale_byte + 120;     // biased FP32 exponent of 2^(e - 7)
    if (fe < 1 || sig == 0u)
        return 0u;                                                // r < 2^-119: rounds to zero
    const float r = (float)sig * __uint_as_float((uint32_t)fe << 23);
    const uint32_t u = __float_as_uint(r);
    uint32_t code;
    if ((int)(u >> 23) - 127 >= 1 - T::kBias) {
        constexpr int sh = 23 - T::kMb;
        code = ((u + ((1u << (sh - 1)) - 1u) + ((u >> sh) & 1u)) >> sh) - ((uint32_t)(127 - T::kBias) << T::kMb);
    } else {
        code = (uint32_t)__builtin_rintf(r * (float)(1 << (T::kBias + T::kMb - 1)));
    }
    return code > (uint32_t)T::kTop ? (uint32_t)T::kTop : code;
}

// One lane casts one 32-element block.
template <int F, bool kHw>
__global__ __launch_bounds__(256) void mx_cast_kernel(const uint16_t* __restrict__ w, int64_t n_rows, int k,
                                                      int64_t ldw, uint32_t* __restrict__ q,
                                                      uint8_t* __restrict__ s)
{
    using T = Fmt<F>;
    constexpr int kDw = T::kBits;                    // dwords per block
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
        uint32_t out[kDw];
#pragma unroll
        for (int i = 0; i < kDw; ++i)
            out[i] = 0u;
        int scale_byte;
        if (amax >= 0x7F80u) {
            scale_byte = 0xFF;                       // NaN or Inf in the block
        } else {
            scale_byte = (int)(amax >> 7) - T::kEmax;
            scale_byte = scale_byte < 0 ? 0 : scale_byte;
            if constexpr (kHw && F != 3) {
                // the magnitudes are clamped to 1.75 * 2^emax X first, so the convert never sees an overflow
                const uint32_t top = (((uint32_t)(scale_byte + T::kEmax)) << 7) | 0x60u;
                u32x16_t c;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t lo = min(d[i] & 0x7FFFu, top) | (d[i] & 0x8000u);
                    const uint32_t hi = min((d[i] >> 16) & 0x7FFFu, top) | ((d[i] >> 16) & 0x8000u);
                    c[i] = lo | (hi << 16);
                }
                const float scale = __uint_as_float((uint32_t)scale_byte << 23);
                if constexpr (F == 1) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        s16x2_t r = {0, 0};
                        const uint32_t pair = c[i];
                        r = __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(r, __builtin_bit_cast(bf16x2_t, pair), scale, false);
                        out[i >> 1] |= (uint32_t)(uint16_t)r[0] << (16 * (i & 1));
                    }
                } else {
                    const u32x6_t r = __builtin_amdgcn_cvt_scalef32_pk32_bf6_bf16(__builtin_bit_cast(bf16x32_t, c), scale);
#pragma unroll
                    for (int i = 0; i < 6; ++i)
                        out[i] = r[i];
                }
            } else {
#pragma unroll
                for (int e = 0; e < 32; ++e) {
                    const uint32_t h = (e & 1) ? d[e >> 1] >> 16 : d[e >> 1] & 0xFFFFu;
                    const uint32_t code = quantise<F>(h & 0x7FFFu, scale_byte) | ((h >> 15) << (T::kBits - 1));
                    const int bit = T::kBits * e, dw = bit >> 5, sft = bit & 31;
                    out[dw] |= code << sft;
                    if (sft + T::kBits > 32)
                        out[dw + 1] |= code >> (32 - sft);
                }
            }
        }
        u32x2_t* dst = reinterpret_cast<u32x2_t*>(q + blk * kDw);
#pragma unroll
        for (int i = 0; i < kDw / 2; ++i)
            dst[i] = u32x2_t{out[2 * i], out[2 * i + 1]};
        s[blk] = (uint8_t)scale_byte;
    }
}

// q, s -> BF16: one lane per block.  E5M2 and E3M2 by the scaled converts (exact while the product
// is a normal BF16), T2 by bit assembly (exact always).
template <int F>
__global__ __launch_bounds__(256) void mx_dequant_kernel(const uint32_t* __restrict__ q, const uint8_t* __restrict__ s,
                                                         int64_t n_rows, int k, uint16_t* __restrict__ w, int64_t ldw)
{
    using T = Fmt<F>;
    constexpr int kDw = T::kBits;
    const int nblk = k >> 5;
    const int64_t total = n_rows * nblk;
    const int64_t blk = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blk >= total)
        return;
    const int64_t row = blk / nblk;
    uint32_t in[kDw];
    const u32x2_t* src = reinterpret_cast<const u32x2_t*>(q + blk * kDw);
#pragma unroll
    for (int i = 0; i < kDw / 2; ++i) {
        const u32x2_t v = src[i];
        in[2 * i] = v[0];
        in[2 * i + 1] = v[1];
    }
    const uint32_t sb = s[blk];
    uint32_t out[16];
    if constexpr (F == 1) {
        const float scale = e8m0_to_f32(sb);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            out[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(in[i], scale, false));
            out[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(in[i], scale, true));
        }
    } else if constexpr (F == 2) {
        const float scale = e8m0_to_f32(sb);
        const u32x6_t packed = {in[0], in[1], in[2], in[3], in[4], in[5]};
        const u32x16_t r = __builtin_bit_cast(u32x16_t, __builtin_amdgcn_cvt_scalef32_pk32_bf16_bf6(packed, scale));
#pragma unroll
        for (int i = 0; i < 16; ++i)
            out[i] = r[i];
    } else {
        // X as BF16: 2^(sb - 127); byte 0 is the subnormal 2^-127, byte 0xFF makes every element NaN
        const uint32_t xb = sb == 0u ? 0x0040u : sb << 7;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t c4 = (in[i >> 3] >> (4 * (i & 7))) & 0xFu;
            uint32_t lo = ((c4 & 1u) ? xb : 0u) | ((c4 & 2u) << 14);
            uint32_t hi = ((c4 & 4u) ? xb : 0u) | ((c4 & 8u) << 12);
            if (sb == 0xFFu)
                lo = hi = 0x7FC0u;
            out[i] = lo | (hi << 16);
        }
    }
    uint4* dst = reinterpret_cast<uint4*>(w + row * ldw + (blk - row * nblk) * 32);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        dst[i] = make_uint4(out[4 * i], out[4 * i + 1], out[4 * i + 2], out[4 * i + 3]);
}

struct FPos {
    int g;      // row group
    int t;      // step along K (`seg` blocks per step)
};

// MT activation rows per pass, R row slots per wave step, NW waves per workgroup; two register
// buffers of one step each.  A wave step covers `seg` = 2^segshift blocks of P = 64 / seg weight
// rows per slot (seg = 64: one row per slot, several steps along K; seg = K/32 < 64: one step).
// `out` as in the other product kernels (y, or the argmax partials).
template <int F, int MT, int R, int NW>
__global__ __launch_bounds__(NW * 64) void mx_gemv_kernel(GemmArgs a, int m0, int segshift)
{
    using T = Fmt<F>;
    constexpr int kBb = T::kBits * 4;                                // bytes per block
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                  // [MT][4][K / 32] chunks of 8 activations
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nblk = a.k >> 5;
    const int xchunks = a.k >> 3;
    const int seg = 1 << segshift;
    const int P = 64 >> segshift;
    const int lrow = lane >> segshift, lb = lane & (seg - 1);
    const int steps = (nblk + seg - 1) >> segshift;
    const int n_groups = (a.n + R * P - 1) / (R * P);
    const int total_waves = gridDim.x * NW;
    const int first_group = (int)blockIdx.x * NW + wave;
    const bool argmax = a.part_val != nullptr;

    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.q), 0,
                                                                        a.n * nblk * kBb, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.s), 0, a.n * nblk,
                                                                        0x00020000);
    auto valid = [&](const FPos& p) { return p.g < n_groups; };
    auto advance = [&](FPos& p) {
        if (++p.t == steps) {
            p.t = 0;
            p.g += total_waves;
        }
    };
    // Always the same loads per step: past the wave's last position, beyond a ragged last step and
    // beyond the last weight row the lane offset is out of the descriptor's range (no memory touched,
    // zero back: zero codes under scale byte 0).
    // Two register buffers of one step each: the first 16 bytes of a block (8 for the 2-bit format),
    // the rest of it (8-bit: 16 bytes, 6-bit: 8 bytes) and the scale byte, per row slot.
    u32x4_t qa[2][R];
    u32x4_t qb[2][F == 1 ? R : 1];
    u32x2_t qc[2][F == 1 ? 1 : R];
    uint32_t qs[2][R];
    auto issue = [&](const FPos& p, const int d) {
        const int g = valid(p) ? p.g : 0;
        const int b = p.t * seg + lb;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = (g * R + r) * P + lrow;
            const bool live = valid(p) && row < a.n && b < nblk;
            const int blk = row * nblk + b;
            const int off = live ? blk * kBb : kOobF;
            if constexpr (F == 1) {
                qa[d][r] = __builtin_amdgcn_raw_buffer_load_b128(rq, off, 0, 2);
                qb[d][r] = __builtin_amdgcn_raw_buffer_load_b128(rq, off, 16, 2);
            } else if constexpr (F == 2) {
                qa[d][r] = __builtin_amdgcn_raw_buffer_load_b128(rq, off, 0, 2);
                qc[d][r] = __builtin_amdgcn_raw_buffer_load_b64(rq, off, 16, 2);
            } else {
                qc[d][r] = __builtin_amdgcn_raw_buffer_load_b64(rq, off, 0, 2);
            }
            qs[d][r] = __builtin_amdgcn_raw_buffer_load_b8(rs, live ? blk : kOobF, 0, 0);
        }
    };

    FPos pos[2];
    FPos load{first_group, 0};
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        pos[d] = load;
        issue(load, d);
        advance(load);
    }
    for (int c = tid; c < xchunks; c += NW * 64) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const int msrc = min(m0 + m, a.m - 1);                   // ragged M: repeat the last row
            const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
            xs[(m * 4 + (c & 3)) * nblk + (c >> 2)] = xp[c];
        }
    }
    lds_barrier();

    float best_val[MT];
    int best_idx[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        best_val[m] = -INFINITY;
        best_idx[m] = 0x7FFFFFFF;
    }
    float acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MT; ++m)
            acc[r][m] = 0.f;

    auto compute = [&](const FPos& p, const int d) {
        const int b = min(p.t * seg + lb, nblk - 1);                  // beyond the tail the weights are zero
        u32x4_t xv[MT][4];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xv[m][j] = xs[(m * 4 + j) * nblk + b];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            uint32_t wv[16];
            float late = 1.f;
            if constexpr (F == 1) {
                // the convert reads only the exponent field of its scale operand (as E8M0)
                const float sc = __uint_as_float(qs[d][r] << 23);
                const u32x4_t lo4 = qa[d][r], hi4 = qb[d][r];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t wd = i < 4 ? lo4[i & 3] : hi4[i & 3];
                    wv[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(wd, sc, false));
                    wv[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(wd, sc, true));
                }
            } else if constexpr (F == 2) {
                const float sc = __uint_as_float(qs[d][r] << 23);
                const u32x4_t lo4 = qa[d][r];
                const u32x2_t hi2 = qc[d][r];
                const u32x6_t packed = {lo4[0], lo4[1], lo4[2], lo4[3], hi2[0], hi2[1]};
                const u32x16_t w6 = __builtin_bit_cast(u32x16_t, __builtin_amdgcn_cvt_scalef32_pk32_bf16_bf6(packed, sc));
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    wv[i] = w6[i];
            } else {
                const u32x2_t c2 = qc[d][r];
                decode_t2(c2[0], wv);
                decode_t2(c2[1], wv + 8);
                // X / 2 = 2^(sb - 128); bytes 0 and 1 give FP32 subnormals, 0xFF gives NaN
                const uint32_t sb = qs[d][r];
                uint32_t bits = sb >= 2u ? (sb - 1u) << 23 : 0x00200000u << sb;
                bits = sb == 0xFFu ? 0x7FC00000u : bits;
                late = __uint_as_float(bits);
            }
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float v = F == 3 ? 0.f : acc[r][m];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    // through a scalar: a bit cast applied directly to a vector element reads element 0
                    const uint32_t xd = xv[m][i >> 2][i & 3];
                    v = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, wv[i]),
                                                        __builtin_bit_cast(bf16x2_t, xd), v, false);
                }
                acc[r][m] = F == 3 ? __builtin_fmaf(v, late, acc[r][m]) : v;
            }
        }
        if (p.t == steps - 1) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = (p.g * R + r) * P + lrow;
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    float v = acc[r][m];
                    acc[r][m] = 0.f;
                    if (segshift == 6) {
                        v = wave_sum(v);
                    } else {
                        for (int o = seg >> 1; o > 0; o >>= 1)        // the lanes of one row, same order in each
                            v += __shfl_xor(v, o);
                    }
                    if (argmax) {
                        if (row < a.n && v > best_val[m]) {           // rows ascend: lowest index wins ties
                            best_val[m] = v;
                            best_idx[m] = row;
                        }
                    } else if (lb == 0 && row < a.n && m0 + m < a.m) {
                        a.y[(int64_t)(m0 + m) * a.ldy + row] = f32_to_bf16_rne(v);
                    }
                }
            }
        }
    };

    // Every trip issues the same loads whether or not buffer 1 still had work, so that every path
    // into the loop head carries the same queue of outstanding loads.
    while (valid(pos[0])) {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            if (d == 0 || valid(pos[d]))
                compute(pos[d], d);
            pos[d] = load;
            issue(load, d);
            advance(load);
        }
    }

    if (argmax) {
        // lanes hold different rows in the packed form: best of the wave, lowest index on ties
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            for (int o = 32; o > 0; o >>= 1) {
                const float v = __shfl_xor(best_val[m], o);
                const int i = __shfl_xor(best_idx[m], o);
                if (v > best_val[m] || (v == best_val[m] && i < best_idx[m])) {
                    best_val[m] = v;
                    best_idx[m] = i;
                }
            }
        }
        __syncthreads();
        float* wval = reinterpret_cast<float*>(smem);
        int* widx = reinterpret_cast<int*>(smem) + NW * MT;
        if (lane == 0) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                wval[wave * MT + m] = best_val[m];
                widx[wave * MT + m] = best_idx[m];
            }
        }
        __syncthreads();
        if (tid < MT && m0 + tid < a.m) {
            float bv = wval[tid];
            int bi = widx[tid];
            for (int w = 1; w < NW; ++w) {
                const float v = wval[w * MT + tid];
                const int i = widx[w * MT + tid];
                if (v > bv || (v == bv && i < bi)) {
                    bv = v;
                    bi = i;
                }
            }
            a.part_val[(int64_t)(m0 + tid) * a.parts + blockIdx.x] = bv;
            a.part_idx[(int64_t)(m0 + tid) * a.parts + blockIdx.x] = bi;
        }
    }
}

template <int F, int MT, int R, int NW>
hipError_t launch_k(const GemmArgs& a, int m0, int segshift, int blocks, size_t lds, int max_lds, hipStream_t stream)
{
    auto kern = mx_gemv_kernel<F, MT, R, NW>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), max_lds); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, stream, a, m0, segshift);
    return hipGetLastError();
}

template <int F, int MT>
hipError_t launch_mt(const GemmArgs& a, int m0, int segshift, bool many_rows, int nw, int blocks, size_t lds,
                     int max_lds, hipStream_t stream)
{
    constexpr int kR = F == 3 ? 4 : 2;              // row slots per step when the matrix has rows to spare
    if (nw == 8)
        return many_rows ? launch_k<F, MT, kR, 8>(a, m0, segshift, blocks, lds, max_lds, stream)
                         : launch_k<F, MT, 1, 8>(a, m0, segshift, blocks, lds, max_lds, stream);
    return many_rows ? launch_k<F, MT, kR, 16>(a, m0, segshift, blocks, lds, max_lds, stream)
                     : launch_k<F, MT, 1, 16>(a, m0, segshift, blocks, lds, max_lds, stream);
}

template <int F>
hipError_t launch_fmt(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    constexpr int kR = F == 3 ? 4 : 2;
    const int nblk = a.k >> 5;
    int segshift = 6;
    if (nblk < 64 && (nblk & (nblk - 1)) == 0)
        for (segshift = 0; (1 << segshift) < nblk; ++segshift) {
        }
    const int rows_per_slot = 64 >> segshift;
    // several row slots per step unless the matrix is so short that SIMDs would idle
    const bool many_rows = (a.n + kR * rows_per_slot - 1) / (kR * rows_per_slot) >= dev.cus * 16;
    const int r = many_rows ? kR : 1;
    const int n_groups = (a.n + r * rows_per_slot - 1) / (r * rows_per_slot);
    int first_blocks = 0;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        int mt = left > 2 ? 4 : (left > 1 ? 2 : 1);
        while (mt > 1 && (size_t)mt * a.k * 2 > (size_t)dev.lds_bytes)
            mt >>= 1;
        const size_t x_bytes = (size_t)mt * a.k * 2;
        const size_t lds = x_bytes < 1024 ? 1024 : x_bytes;          // the argmax combine needs a few bytes
        const int per_cu = 2 * lds <= (size_t)dev.lds_bytes ? 2 : 1;
        const int nw = per_cu == 2 ? 8 : 16;                          // 16 waves per compute unit
        int blocks = (n_groups + nw - 1) / nw;
        if (blocks > dev.cus * per_cu)
            blocks = dev.cus * per_cu;
        if (blocks > gemv_max_parts(dev))
            blocks = gemv_max_parts(dev);
        // the argmax partial arrays are indexed by workgroup: no pass may use more than the first
        if (m0 == 0)
            first_blocks = blocks;
        else if (a.part_val != nullptr && blocks > first_blocks)
            blocks = first_blocks;
        hipError_t e;
        switch (mt) {
        case 4:
            e = launch_mt<F, 4>(a, m0, segshift, many_rows, nw, blocks, lds, dev.lds_bytes, stream);
            break;
        case 2:
            e = launch_mt<F, 2>(a, m0, segshift, many_rows, nw, blocks, lds, dev.lds_bytes, stream);
            break;
        default:
            e = launch_mt<F, 1>(a, m0, segshift, many_rows, nw, blocks, lds, dev.lds_bytes, stream);
            break;
        }
        if (e != hipSuccess)
            return e;
        m0 += mt;
    }
    if (parts_used)
        *parts_used = first_blocks;
    return hipSuccess;
}

template <int F>
hipError_t launch_cast_f(const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q, void* s, bool integer_rule,
                         hipStream_t stream)
{
    const int64_t total = n_rows * (k / 32);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 8)
        blocks = 256 * 8;
    auto kern = integer_rule ? mx_cast_kernel<F, false> : mx_cast_kernel<F, true>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t*)w, n_rows, (int)k, ldw,
                       (uint32_t*)q, (uint8_t*)s);
    return hipGetLastError();
}

template <int F>
hipError_t launch_dequant_f(const void* q, const void* s, int64_t n_rows, int64_t k, void* w, int64_t ldw,
                            hipStream_t stream)
{
    const int64_t total = n_rows * (k / 32);
    hipLaunchKernelGGL(mx_dequant_kernel<F>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const uint32_t*)q, (const uint8_t*)s, n_rows, (int)k, (uint16_t*)w, ldw);
    return hipGetLastError();
}

}  // namespace

int mxfmt_block_bytes(int fmt) { return fmt == 1 ? 32 : (fmt == 2 ? 24 : (fmt == 3 ? 8 : 0)); }

hipError_t launch_mxfmt_cast(int fmt, const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q, void* s,
                             bool integer_rule, hipStream_t stream)
{
    if (n_rows * (k / 32) == 0)
        return hipSuccess;
    switch (fmt) {
    case 1:
        return launch_cast_f<1>(w, n_rows, k, ldw, q, s, integer_rule, stream);
    case 2:
        return launch_cast_f<2>(w, n_rows, k, ldw, q, s, integer_rule, stream);
    case 3:
        return launch_cast_f<3>(w, n_rows, k, ldw, q, s, true, stream);
    default:
        return hipErrorInvalidValue;
    }
}

hipError_t launch_mxfmt_dequant(int fmt, const void* q, const void* s, int64_t n_rows, int64_t k, void* w,
                                int64_t ldw, hipStream_t stream)
{
    if (n_rows * (k / 32) == 0)
        return hipSuccess;
    switch (fmt) {
    case 1:
        return launch_dequant_f<1>(q, s, n_rows, k, w, ldw, stream);
    case 2:
        return launch_dequant_f<2>(q, s, n_rows, k, w, ldw, stream);
    case 3:
        return launch_dequant_f<3>(q, s, n_rows, k, w, ldw, stream);
    default:
        return hipErrorInvalidValue;
    }
}

// The activation copy of one row must fit the LDS.
bool mxfmt_can_run(const GemmArgs& a, const DeviceInfo& dev) { return (size_t)a.k * 2 <= (size_t)dev.lds_bytes; }

hipError_t launch_mxfmt_gemv(int fmt, const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    switch (fmt) {
    case 1:
        return launch_fmt<1>(a, dev, parts_used, stream);
    case 2:
        return launch_fmt<2>(a, dev, parts_used, stream);
    case 3:
        return launch_fmt<3>(a, dev, parts_used, stream);
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace mxfp4
