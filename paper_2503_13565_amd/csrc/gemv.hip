// Bandwidth-bound skinny product y = x * dequant(W)^T on the vector ALUs of gfx950, for one
// or two activation rows at a time (arXiv 2503.13565, section 3.4.3 and Eq. 2; section 4.4:
// the GEMM with 1..8 tokens must run at memory speed).
//
// Mapping.  A lane owns whole 32-element scale blocks: one 16-byte load brings a block's 32
// nibbles, one byte load its scale, so a wave instruction reads 1 KiB of contiguous packed
// weights.  A wave walks a group of R consecutive weight rows, 64 blocks per step, keeping
// FP32 partial sums per (row, activation row); the lanes' partials are summed with DPP at the
// end of the row group.  Activations are staged once per workgroup in LDS, laid out so that
// the 16-byte chunk j of consecutive blocks is contiguous (conflict-free 128-bit reads), and
// are shared by all R rows of the step.  Workgroups are persistent: row groups are dealt
// round-robin to all waves of the grid.  Loads for the next step are issued before the
// current step is computed (two register buffers).
//
// Decode variants (template kDecode):
//   kCvt  - v_cvt_scalef32_pk_bf16_fp4: one instruction turns a byte (2 nibbles) and the
//           block scale into two scaled BF16 weights; v_dot2_f32_bf16 multiplies-adds them.
//   kLut  - LDS-resident table byte -> two unscaled BF16 weights, replicated per bank so
//           every lane reads its own bank; the scale is applied to the 32-element partial
//           sum (late scaling, Eq. 2).
//   kBits - plain integer/FP32 bit assembly; slow, kept as the in-library cross-check.
#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

enum { kBits = MXFP4_PATH_VALU_BITS, kCvt = MXFP4_PATH_VALU_CVT, kLut = MXFP4_PATH_VALU_LUT };

constexpr int kLutBytes = 256 * 32 * 4;   // 256 byte values x 32 banks x one dword

template <int R>
struct Item {
    uint4 q[R];         // packed nibbles of this lane's block, one per row of the group
    uint32_t s[R];      // scale bytes
};

struct Pos {
    int g;              // row group
    int t;              // step along K (64 blocks per step)
};

template <int MT, int R, int kDecode, bool kTail, bool kArgmax>
__global__ __launch_bounds__(256) void gemv_kernel(GemmArgs a, int m0)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint4* xs = reinterpret_cast<uint4*>(smem);                      // [MT][4][nblk] chunks
    uint32_t* lut = reinterpret_cast<uint32_t*>(smem + (size_t)MT * a.k * 2);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nblk = a.k >> 5;

    // Stage the activation rows: chunk c (8 elements) of row m goes to [m][c & 3][c >> 2].
    {
        const int chunks = a.k >> 3;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const int msrc = min(m0 + m, a.m - 1);                   // ragged M: repeat the last row
            const uint4* xr = reinterpret_cast<const uint4*>(a.x + (int64_t)msrc * a.ldx);
            for (int c = tid; c < chunks; c += 256)
                xs[(m * 4 + (c & 3)) * nblk + (c >> 2)] = xr[c];
        }
        if constexpr (kDecode == kLut) {
            for (int e = tid; e < 256 * 32; e += 256) {
                const uint32_t byte = (uint32_t)e >> 5;
                const uint32_t lo = __float_as_uint(e2m1_to_f32(byte & 0xFu)) >> 16;
                const uint32_t hi = __float_as_uint(e2m1_to_f32(byte >> 4)) >> 16;
                lut[e] = lo | (hi << 16);
            }
        }
    }
    __syncthreads();

    const int steps = (nblk + 63) >> 6;
    const int n_groups = (a.n + R - 1) / R;
    const int total_waves = gridDim.x * 4;
    const int64_t q_row_bytes = a.k >> 1;

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

    auto valid = [&](const Pos& p) { return p.g < n_groups; };
    auto advance = [&](Pos& p) {
        if (++p.t == steps) {
            p.t = 0;
            p.g += total_waves;
        }
    };
    auto issue = [&](const Pos& p, Item<R>& it) {
        const int b = p.t * 64 + lane;
        const int bc = kTail ? min(b, nblk - 1) : b;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = min(p.g * R + r, a.n - 1);                // ragged N: re-read the last row
            it.q[r] = *reinterpret_cast<const uint4*>(a.q + row * q_row_bytes + (int64_t)bc * 16);
            it.s[r] = a.s[(int64_t)row * nblk + bc];
        }
    };
    auto compute = [&](const Pos& p, Item<R>& it) {
        const int b = p.t * 64 + lane;
        const int bc = kTail ? min(b, nblk - 1) : b;
        uint4 xv[MT][4];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xv[m][j] = xs[(m * 4 + j) * nblk + bc];
        if (kTail && b >= nblk) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                it.q[r] = make_uint4(0, 0, 0, 0);                     // all nibbles +0
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float sc = e8m0_to_f32(it.s[r]);
            const uint32_t qd[4] = {it.q[r].x, it.q[r].y, it.q[r].z, it.q[r].w};
            float part[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m)
                part[m] = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t xd[MT][4];
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    xd[m][0] = xv[m][j].x;
                    xd[m][1] = xv[m][j].y;
                    xd[m][2] = xv[m][j].z;
                    xd[m][3] = xv[m][j].w;
                }
                if constexpr (kDecode == kCvt) {
                    bf16x2_t w[4];
                    w[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd[j], sc, 0);
                    w[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd[j], sc, 1);
                    w[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd[j], sc, 2);
                    w[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd[j], sc, 3);
#pragma unroll
                    for (int p4 = 0; p4 < 4; ++p4)
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[r][m] = __builtin_amdgcn_fdot2_f32_bf16(
                                w[p4], __builtin_bit_cast(bf16x2_t, xd[m][p4]), acc[r][m], false);
                } else if constexpr (kDecode == kLut) {
                    const uint32_t* bank = lut + (lane & 31);
#pragma unroll
                    for (int p4 = 0; p4 < 4; ++p4) {
                        const uint32_t byte = (qd[j] >> (8 * p4)) & 0xFFu;
                        const uint32_t w2 = bank[byte * 32];
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            part[m] = __builtin_amdgcn_fdot2_f32_bf16(
                                __builtin_bit_cast(bf16x2_t, w2), __builtin_bit_cast(bf16x2_t, xd[m][p4]),
                                part[m], false);
                    }
                } else {
#pragma unroll
                    for (int p4 = 0; p4 < 4; ++p4) {
                        const uint32_t byte = (qd[j] >> (8 * p4)) & 0xFFu;
                        const float wlo = e2m1_to_f32(byte & 0xFu), whi = e2m1_to_f32(byte >> 4);
#pragma unroll
                        for (int m = 0; m < MT; ++m) {
                            part[m] = fmaf(wlo, bf16_bits_to_f32(xd[m][p4] & 0xFFFFu), part[m]);
                            part[m] = fmaf(whi, bf16_bits_to_f32(xd[m][p4] >> 16), part[m]);
                        }
                    }
                }
            }
            if constexpr (kDecode != kCvt) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    acc[r][m] = fmaf(sc, part[m], acc[r][m]);         // late scaling, Eq. 2
            }
        }
        if (p.t == steps - 1) {
            // end of the row group: sum the lanes' partials, write or compare
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = p.g * R + r;
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    const float v = wave_sum(acc[r][m]);
                    acc[r][m] = 0.f;
                    if (row < a.n && m0 + m < a.m) {
                        if constexpr (kArgmax) {
                            if (v > best_val[m]) {                    // rows ascend: lowest index wins ties
                                best_val[m] = v;
                                best_idx[m] = row;
                            }
                        } else if (lane == 0) {
                            a.y[(int64_t)(m0 + m) * a.ldy + row] = f32_to_bf16_rne(v);
                        }
                    }
                }
            }
        }
    };

    Item<R> buf_a, buf_b;
    Pos load{(int)blockIdx.x * 4 + wave, 0};
    Pos cur = load;
    if (valid(load))
        issue(load, buf_a);
    advance(load);
    while (valid(cur)) {
        Pos next = load;
        if (valid(load))
            issue(load, buf_b);
        advance(load);
        compute(cur, buf_a);
        cur = next;
        if (!valid(cur))
            break;
        next = load;
        if (valid(load))
            issue(load, buf_a);
        advance(load);
        compute(cur, buf_b);
        cur = next;
    }

    if constexpr (kArgmax) {
        // combine the 4 waves of the workgroup, then publish one partial winner per row
        __syncthreads();
        float* wv = reinterpret_cast<float*>(smem);
        int* wi = reinterpret_cast<int*>(smem) + 4 * MT;
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
            for (int w = 1; w < 4; ++w) {
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

__global__ __launch_bounds__(256) void argmax_finish_kernel(const float* __restrict__ part_val,
                                                            const int32_t* __restrict__ part_idx,
                                                            int parts, int parts_used,
                                                            int32_t* __restrict__ argmax_out,
                                                            float* __restrict__ max_out)
{
    __shared__ float sv[256];
    __shared__ int si[256];
    const int m = blockIdx.x, tid = threadIdx.x;
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int p = tid; p < parts_used; p += 256) {
        const float v = part_val[(int64_t)m * parts + p];
        const int i = part_idx[(int64_t)m * parts + p];
        if (v > bv || (v == bv && i < bi)) {
            bv = v;
            bi = i;
        }
    }
    sv[tid] = bv;
    si[tid] = bi;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) {
            const float v = sv[tid + off];
            const int i = si[tid + off];
            if (v > sv[tid] || (v == sv[tid] && i < si[tid])) {
                sv[tid] = v;
                si[tid] = i;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        // every accumulator -inf or NaN: report index 0 rather than the sentinel
        argmax_out[m] = si[0] == 0x7FFFFFFF ? 0 : si[0];
        if (max_out)
            max_out[m] = sv[0];
    }
}

int gemv_max_parts(const DeviceInfo& dev) { return dev.cus * 8; }

namespace {

template <int MT, int R, int kDecode, bool kTail, bool kArgmax>
hipError_t launch_one(const GemmArgs& a, int m0, int blocks, size_t lds, int max_lds, hipStream_t stream)
{
    auto kern = gemv_kernel<MT, R, kDecode, kTail, kArgmax>;
    static bool attr_set = false;                   // per instantiation; racing writers set the same value
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (e != hipSuccess)
            return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, stream, a, m0);
    return hipGetLastError();
}

template <int MT, int kDecode, bool kArgmax>
hipError_t launch_mt(const GemmArgs& a, int m0, bool tail, int blocks, size_t lds, int max_lds,
                     hipStream_t stream)
{
    constexpr int R = 4;
    if (tail)
        return launch_one<MT, R, kDecode, true, kArgmax>(a, m0, blocks, lds, max_lds, stream);
    return launch_one<MT, R, kDecode, false, kArgmax>(a, m0, blocks, lds, max_lds, stream);
}

template <int kDecode, bool kArgmax>
hipError_t launch_decode(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    constexpr int R = 4;
    const int nblk = a.k / 32;
    const bool tail = (nblk % 64) != 0;
    const size_t extra = kDecode == kLut ? (size_t)kLutBytes : 0;
    // two activation rows per pass when their LDS copy fits, else one
    const bool two_fit = (size_t)2 * a.k * 2 + extra <= (size_t)dev.lds_bytes;
    const int n_groups = (a.n + R - 1) / R;
    int blocks_per_cu = 4;
    int blocks = (n_groups + 3) / 4;
    if (blocks > dev.cus * blocks_per_cu)
        blocks = dev.cus * blocks_per_cu;
    if (parts_used)
        *parts_used = blocks;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        hipError_t e;
        if (left >= 2 && two_fit) {
            e = launch_mt<2, kDecode, kArgmax>(a, m0, tail, blocks, (size_t)2 * a.k * 2 + extra,
                                                dev.lds_bytes, stream);
            m0 += 2;
        } else {
            e = launch_mt<1, kDecode, kArgmax>(a, m0, tail, blocks, (size_t)a.k * 2 + extra, dev.lds_bytes,
                                                stream);
            m0 += 1;
        }
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

}  // namespace

hipError_t launch_gemv(const GemmArgs& a, int decode, bool argmax, const DeviceInfo& dev, int* parts_used,
                       hipStream_t stream)
{
    switch (decode) {
    case kBits:
        return argmax ? launch_decode<kBits, true>(a, dev, parts_used, stream)
                      : launch_decode<kBits, false>(a, dev, parts_used, stream);
    case kCvt:
        return argmax ? launch_decode<kCvt, true>(a, dev, parts_used, stream)
                      : launch_decode<kCvt, false>(a, dev, parts_used, stream);
    case kLut:
        return argmax ? launch_decode<kLut, true>(a, dev, parts_used, stream)
                      : launch_decode<kLut, false>(a, dev, parts_used, stream);
    default:
        return hipErrorInvalidValue;
    }
}

hipError_t launch_argmax_finish(const float* part_val, const int32_t* part_idx, int parts, int parts_used,
                                int m, int32_t* argmax_out, float* max_out, hipStream_t stream)
{
    hipLaunchKernelGGL(argmax_finish_kernel, dim3(m), dim3(256), 0, stream, part_val, part_idx, parts,
                       parts_used, argmax_out, max_out);
    return hipGetLastError();
}

}  // namespace mxfp4
