// An 8-bit draft format on the same path (arXiv 2503.13565, sections 1, 3.2 and 5 name 8-bit
// quantisation as a drop-in for the 4-bit draft; the cast is the two-step rule of section 3.4.3
// with the 8-bit element format): E4M3 elements (1 sign, 4 exponent bits with bias 7, 3 mantissa
// bits, largest magnitude 448, S.1111.111 = NaN), one E8M0 scale per 32 elements along K.
// Layout: q8 [N, K] one byte per element, scales [N, K/32].
//
// Cast: as the 4-bit cast (four lanes share a block, 16 bytes of BF16 per lane, block maximum by
// DPP, scale byte = exponent of the maximum minus 8), elements rounded by the gfx950 scaled
// BF16->FP8 convert after clamping the magnitude to 448 X (so that the instruction never sees an
// overflow), or by an integer rule on the bit patterns that gives the same bits.
// Product: the skeleton of the BF16 GEMV: a wave walks groups of R weight rows, one 16-byte load
// per lane and row (16 weights = half a scale block, 1 KiB per wave instruction), the lane's scale
// byte by a byte load, activations staged once per workgroup in LDS, scaled FP8->BF16 converts
// (two weights each) and v_dot2_f32_bf16 with FP32 accumulation.  At one byte per weight the
// vector ALUs keep up with memory for up to four activation rows per pass (8 converts + 8 dot2 per
// row and 16 bytes); more rows take more passes.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

namespace {

typedef __attribute__((ext_vector_type(2))) short s16x2_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;

constexpr int kOob8 = 0x7FFFFFF0;        // lane offset beyond any descriptor: the load returns zero

// Code (eeeemmm) of one element from its 15 magnitude bits and the block's scale byte.  With sig
// the 8-bit significand, r = |v| / X = sig * 2^(e - 7), e = exponent field - scale byte.  F is r in
// units of 2^-17; the quantum of E4M3 is 2^-9 below 2^-6 and 2^(binade - 3) above; F is rounded to
// it to nearest even and re-based to the code, saturating at 126 (448).
__device__ __forceinline__ uint32_t quantise_e4m3(uint32_t mag, int scale_byte)
{
    const uint32_t exp = mag >> 7;
    const uint32_t man = mag & 0x7Fu;
    const uint32_t sig = exp ? (0x80u | man) : man;
    const int sh = (int)(exp ? exp : 1u) - scale_byte + 10;
    if (sh < 0 || sig == 0u)
        return 0u;                                   // below 2^-10: rounds to zero
    const uint32_t F = sig << sh;                    // sh <= 18: below 2^26
    const int top = 31 - __clz((int)F);
    const int shq = (top > 11 ? top : 11) - 3;       // log2 of the quantum in F units
    const uint32_t rounded = (F + ((1u << (shq - 1)) - 1u) + ((F >> shq) & 1u)) >> shq;
    const uint32_t code = rounded + ((uint32_t)(shq - 8) << 3);
    return code > 126u ? 126u : code;
}

template <bool kHw>
__device__ __forceinline__ void cast_group8(const u32x4_t v, u32x2_t* out, int* scale_out)
{
    const uint32_t d[4] = {v[0], v[1], v[2], v[3]};
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        amax = max(amax, max(d[i] & 0x7FFFu, (d[i] >> 16) & 0x7FFFu));
    amax = max(amax, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)amax, 0xB1, 0xF, 0xF, false));
    amax = max(amax, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)amax, 0x4E, 0xF, 0xF, false));

    u32x2_t packed = {0u, 0u};
    int scale_byte;
    if (amax >= 0x7F80u) {
        scale_byte = 0xFF;                           // NaN or Inf in the block
    } else {
        scale_byte = (int)(amax >> 7) - 8;           // biased exponent of amax, minus 8
        scale_byte = scale_byte < 0 ? 0 : scale_byte;
        if constexpr (kHw) {
            const float scale = __uint_as_float((uint32_t)scale_byte << 23);
            const uint32_t top = (((uint32_t)scale_byte + 8u) << 7) | 0x60u;      // 448 X as BF16 magnitude bits
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = min(d[i] & 0x7FFFu, top) | (d[i] & 0x8000u);
                const uint32_t hi = min((d[i] >> 16) & 0x7FFFu, top) | ((d[i] >> 16) & 0x8000u);
                const uint32_t pair = lo | (hi << 16);
                s16x2_t r = {0, 0};
                r = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(r, __builtin_bit_cast(bf16x2_t, pair), scale, false);
                const uint32_t two = (uint32_t)(uint16_t)r[0];
                if (i < 2)
                    packed[0] |= two << (16 * i);
                else
                    packed[1] |= two << (16 * (i - 2));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = d[i] & 0xFFFFu, hi = d[i] >> 16;
                const uint32_t blo = quantise_e4m3(lo & 0x7FFFu, scale_byte) | ((lo >> 15) << 7);
                const uint32_t bhi = quantise_e4m3(hi & 0x7FFFu, scale_byte) | ((hi >> 15) << 7);
                const uint32_t two = blo | (bhi << 8);
                if (i < 2)
                    packed[0] |= two << (16 * i);
                else
                    packed[1] |= two << (16 * (i - 2));
            }
        }
    }
    *out = packed;
    *scale_out = scale_byte;
}

template <bool kHw>
__global__ __launch_bounds__(256) void e4m3_cast_kernel(const uint16_t* __restrict__ w, int64_t n_rows, int k,
                                                        int64_t ldw, u32x2_t* __restrict__ q8,
                                                        uint8_t* __restrict__ s)
{
    constexpr int kU = 4;
    const int groups_per_row = k >> 3;               // 8-element groups; a multiple of 4
    const int64_t total = n_rows * groups_per_row;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t g0 = (int64_t)blockIdx.x * 256 + threadIdx.x; g0 < total; g0 += kU * stride) {
        u32x4_t v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            int64_t gid = g0 + u * stride;
            gid = gid < total ? gid : g0;            // surplus slots repeat the first (never stored)
            const int64_t row = gid / groups_per_row;
            v[u] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4_t*>(w + row * ldw + (gid - row * groups_per_row) * 8));
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int64_t gid = g0 + u * stride;
            u32x2_t packed;
            int scale_byte;
            cast_group8<kHw>(v[u], &packed, &scale_byte);  // whole quads take part in the DPP steps
            if (gid < total) {
                q8[gid] = packed;
                if ((gid & 3) == 0)
                    s[gid >> 2] = (uint8_t)scale_byte;
            }
        }
    }
}

// q8, s -> BF16 (exact while the product is a normal BF16): one lane per 8 elements, by the
// scaled FP8->BF16 convert, so that the instruction's semantics can be checked in isolation.
__global__ __launch_bounds__(256) void e4m3_dequant_kernel(const u32x2_t* __restrict__ q8,
                                                           const uint8_t* __restrict__ s, int64_t n_rows, int k,
                                                           uint16_t* __restrict__ w, int64_t ldw)
{
    const int groups_per_row = k >> 3;
    const int64_t total = n_rows * groups_per_row;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total)
        return;
    const int64_t row = gid / groups_per_row;
    const int cg = (int)(gid - row * groups_per_row);
    const u32x2_t packed = q8[gid];
    const uint32_t sb = s[gid >> 2];
    const float scale = e8m0_to_f32(sb);
    const uint32_t p0 = packed[0], p1 = packed[1];
    const bf16x2_t a0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(p0, scale, false);
    const bf16x2_t a1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(p0, scale, true);
    const bf16x2_t a2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(p1, scale, false);
    const bf16x2_t a3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(p1, scale, true);
    *reinterpret_cast<uint4*>(w + row * ldw + (int64_t)cg * 8) =
        make_uint4(__builtin_bit_cast(uint32_t, a0), __builtin_bit_cast(uint32_t, a1),
                   __builtin_bit_cast(uint32_t, a2), __builtin_bit_cast(uint32_t, a3));
}

struct E8Pos {
    int g;      // row group
    int t;      // step along K (64 chunks of 16 elements per step)
};

// MT activation rows per pass, R weight rows per group, NW waves per workgroup; two register
// buffers of one step each.  `out` as in the other product kernels (y, or the argmax partials).
template <int MT, int R, int NW>
__global__ __launch_bounds__(NW * 64) void e4m3_gemv_kernel(GemmArgs a, int m0)
{
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                  // [MT][K / 8] chunks of 8 activations
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int xchunks = a.k >> 3;
    const int chunks = a.k >> 4;                                     // 16-element weight chunks per row
    const int nblk = a.k >> 5;
    const int steps = (chunks + 63) >> 6;
    const int tail = chunks - (steps - 1) * 64;                      // chunks in the last step (1..64)
    const int n_groups = (a.n + R - 1) / R;
    const int total_waves = gridDim.x * NW;
    const int first_group = (int)blockIdx.x * NW + wave;
    const bool argmax = a.part_val != nullptr;

    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.q), 0, a.n * a.k,
                                                                        0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.s), 0, a.n * nblk,
                                                                        0x00020000);
    struct Item {
        u32x4_t w[R];
        uint32_t sc[R];
    };
    auto valid = [&](const E8Pos& p) { return p.g < n_groups; };
    auto advance = [&](E8Pos& p) {
        if (++p.t == steps) {
            p.t = 0;
            p.g += total_waves;
        }
    };
    // Always 2 R loads per step: past the wave's last position, and for the lanes beyond a ragged
    // last step, the lane offset is out of the descriptor's range (no memory touched, zero back).
    auto issue = [&](const E8Pos& p, Item& it) {
        const bool live = valid(p) && (p.t < steps - 1 || lane < tail);
        const int g = valid(p) ? p.g : 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = min(g * R + r, a.n - 1);                  // ragged N: re-read the last row
            it.w[r] = __builtin_amdgcn_raw_buffer_load_b128(rq, live ? lane * 16 : kOob8, row * a.k + p.t * 1024, 2);
            it.sc[r] = __builtin_amdgcn_raw_buffer_load_b8(rs, live ? (lane >> 1) : kOob8, row * nblk + p.t * 32, 0);
        }
    };

    Item buf[2];
    E8Pos pos[2];
    E8Pos load{first_group, 0};
    {
        constexpr int T = NW * 64;
        constexpr int kSlots = 8 / MT;                               // 8 activation loads in flight per batch
        u32x4_t xr[MT][kSlots];
        auto x_load = [&](int c0) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const int msrc = min(m0 + m, a.m - 1);               // ragged M: repeat the last row
                const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
#pragma unroll
                for (int i = 0; i < kSlots; ++i)
                    xr[m][i] = xp[min(c0 + i * T, xchunks - 1)];
            }
        };
        auto x_store = [&](int c0) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int i = 0; i < kSlots; ++i)
                    xs[m * xchunks + min(c0 + i * T, xchunks - 1)] = xr[m][i];   // clamped duplicates rewrite the same data
        };
        x_load(tid);
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            pos[d] = load;
            issue(load, buf[d]);
            advance(load);
        }
        x_store(tid);
        for (int c0 = tid + kSlots * T; c0 < xchunks; c0 += kSlots * T) {
            x_load(c0);
            x_store(c0);
        }
    }
    lds_barrier();

    float best_val[MT];
    int best_idx[MT];
    float res[MT];               // finished outputs, one per lane: slot i = i-th finished row of this wave
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        best_val[m] = -INFINITY;
        best_idx[m] = 0x7FFFFFFF;
        res[m] = 0.f;
    }
    int slots = 0, flushed_groups = 0;
    float acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MT; ++m)
            acc[r][m] = 0.f;

    auto flush = [&]() {
        if (lane < slots) {
            const int j = lane / R, r = lane - j * R;
            const int row = (first_group + (flushed_groups + j) * total_waves) * R + r;
            if (row < a.n) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    if (m0 + m < a.m)
                        a.y[(int64_t)(m0 + m) * a.ldy + row] = f32_to_bf16_rne(res[m]);
            }
        }
        flushed_groups += slots / R;
        slots = 0;
        drain_vmem();
    };

    auto compute = [&](const E8Pos& p, const Item& it) {
        const int c = min(p.t * 64 + lane, chunks - 1);               // beyond the tail the weights are zero
        u32x4_t xv[MT][2];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            xv[m][0] = xs[m * xchunks + 2 * c];
            xv[m][1] = xs[m * xchunks + 2 * c + 1];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            // the convert reads only the exponent field of its scale operand (as E8M0)
            const float sc = __uint_as_float(it.sc[r] << 23);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t wd = it.w[r][j];                       // four weights
                const bf16x2_t w_lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wd, sc, false);
                const bf16x2_t w_hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wd, sc, true);
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    // through scalars: a bit cast applied directly to a vector element reads element 0
                    const uint32_t x_lo = xv[m][j >> 1][(j & 1) * 2], x_hi = xv[m][j >> 1][(j & 1) * 2 + 1];
                    float v = acc[r][m];
                    v = __builtin_amdgcn_fdot2_f32_bf16(w_lo, __builtin_bit_cast(bf16x2_t, x_lo), v, false);
                    v = __builtin_amdgcn_fdot2_f32_bf16(w_hi, __builtin_bit_cast(bf16x2_t, x_hi), v, false);
                    acc[r][m] = v;
                }
            }
        }
        if (p.t == steps - 1) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = p.g * R + r;
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    const float v = wave_sum(acc[r][m]);
                    acc[r][m] = 0.f;
                    if (argmax) {
                        if (row < a.n && v > best_val[m]) {           // rows ascend: lowest index wins ties
                            best_val[m] = v;
                            best_idx[m] = row;
                        }
                    } else {
                        res[m] = (lane == slots + r) ? v : res[m];
                    }
                }
            }
            if (!argmax) {
                slots += R;
                if (slots + R > 64)
                    flush();
            }
        }
    };

    // Every trip issues the same loads whether or not buffer 1 still had work, so that every path
    // into the loop head carries the same queue of outstanding loads.
    while (valid(pos[0])) {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            if (d == 0 || valid(pos[d]))
                compute(pos[d], buf[d]);
            pos[d] = load;
            issue(load, buf[d]);
            advance(load);
        }
    }
    if (!argmax && slots > 0)
        flush();

    if (argmax) {
        __syncthreads();
        float* wv = reinterpret_cast<float*>(smem);
        int* wi = reinterpret_cast<int*>(smem) + NW * MT;
        if (lane == 0) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                wv[wave * MT + m] = best_val[m];
                wi[wave * MT + m] = best_idx[m];
            }
        }
        __syncthreads();
        if (tid < MT && m0 + tid < a.m) {
            float bv = wv[tid];
            int bi = wi[tid];
            for (int w = 1; w < NW; ++w) {
                const float v = wv[w * MT + tid];
                const int i = wi[w * MT + tid];
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

template <int MT, int R, int NW>
hipError_t launch_k(const GemmArgs& a, int m0, int blocks, size_t lds, int max_lds, hipStream_t stream)
{
    auto kern = e4m3_gemv_kernel<MT, R, NW>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), max_lds); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, stream, a, m0);
    return hipGetLastError();
}

template <int MT>
hipError_t launch_rows(const GemmArgs& a, int m0, int r, int nw, int blocks, size_t lds, int max_lds,
                       hipStream_t stream)
{
#define MXFP4_E4M3_CASE(NW_)                                                              \
    if (nw == NW_)                                                                        \
        return r == 2 ? launch_k<MT, 2, NW_>(a, m0, blocks, lds, max_lds, stream)         \
                      : launch_k<MT, 1, NW_>(a, m0, blocks, lds, max_lds, stream);
    MXFP4_E4M3_CASE(4)
    MXFP4_E4M3_CASE(8)
    MXFP4_E4M3_CASE(16)
#undef MXFP4_E4M3_CASE
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_e4m3_cast(const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q8, void* s,
                            bool integer_rule, hipStream_t stream)
{
    const int64_t total = n_rows * (k / 8);
    if (total == 0)
        return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 8)
        blocks = 256 * 8;
    auto kern = integer_rule ? e4m3_cast_kernel<false> : e4m3_cast_kernel<true>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t*)w, n_rows, (int)k, ldw,
                       (u32x2_t*)q8, (uint8_t*)s);
    return hipGetLastError();
}

hipError_t launch_e4m3_dequant(const void* q8, const void* s, int64_t n_rows, int64_t k, void* w, int64_t ldw,
                               hipStream_t stream)
{
    const int64_t total = n_rows * (k / 8);
    if (total == 0)
        return hipSuccess;
    hipLaunchKernelGGL(e4m3_dequant_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const u32x2_t*)q8, (const uint8_t*)s, n_rows, (int)k, (uint16_t*)w, ldw);
    return hipGetLastError();
}

// The activation copy of one row must fit the LDS.
bool e4m3_can_run(const GemmArgs& a, const DeviceInfo& dev) { return (size_t)a.k * 2 <= (size_t)dev.lds_bytes; }

hipError_t launch_e4m3_gemv(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    // two rows per group unless the matrix is so short that SIMDs would idle
    const int r = (a.n + 1) / 2 >= dev.cus * 16 ? 2 : 1;
    const int n_groups = (a.n + r - 1) / r;
    int first_blocks = 0;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        static const int max_mt = [] {
            const char* e = knob("MXFP4_E4M3_MAX_ROWS");           // measurement only
            return e ? atoi(e) : 8;
        }();
        int mt = left > 4 && max_mt >= 8 ? 8 : (left > 2 ? 4 : (left > 1 ? 2 : 1));
        while (mt > 1 && (size_t)mt * a.k * 2 > (size_t)dev.lds_bytes)
            mt >>= 1;
        const size_t lds = (size_t)mt * a.k * 2 < 256 ? 256 : (size_t)mt * a.k * 2;   // the argmax combine needs a few bytes
        int per_cu = (int)((size_t)dev.lds_bytes / lds);
        per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
        const int nw = per_cu >= 3 ? 4 : (per_cu == 2 ? 8 : 16);     // 16 waves per compute unit
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
        case 8:
            e = launch_rows<8>(a, m0, r, nw, blocks, lds, dev.lds_bytes, stream);
            break;
        case 4:
            e = launch_rows<4>(a, m0, r, nw, blocks, lds, dev.lds_bytes, stream);
            break;
        case 2:
            e = launch_rows<2>(a, m0, r, nw, blocks, lds, dev.lds_bytes, stream);
            break;
        default:
            e = launch_rows<1>(a, m0, r, nw, blocks, lds, dev.lds_bytes, stream);
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

}  // namespace mxfp4
