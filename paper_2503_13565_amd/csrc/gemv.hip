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
#include <stdio.h>
#include <stdlib.h>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

enum { kBits = MXFP4_PATH_VALU_BITS, kCvt = MXFP4_PATH_VALU_CVT, kLut = MXFP4_PATH_VALU_LUT };

constexpr int kLutBytes = 256 * 32 * 4;   // 256 byte values x 32 banks x one dword

template <int R, bool kScaleDword>
struct Item {
    u32x4_t q[R];                   // packed nibbles of this lane's block, one per row of the group
    uint32_t s[kScaleDword ? 1 : R];  // scale bytes: this lane's own (one per row), or, in the dword
                                    // scheme, four consecutive scales of row (lane / 16) % R
};

struct Pos {
    int g;              // row group
    int t;              // step along K (64 blocks per step)
};

constexpr int kXRegChunks = 4;    // activation chunks a thread can hold while the weights start

// MT activation rows per pass, R weight rows per group, D register buffers of one step each
// (D-1 steps of loads stay in flight while one is computed), NW waves per workgroup.
// kEpi: the fused form (bias, gate, residual applied at the flush; `epi` is not read otherwise).
// The gate needs R even: a group then holds whole (gate, up) row pairs in neighbouring lanes.
template <int MT, int R, int D, int NW, int kDecode, bool kScaleDword, bool kEpi>
__global__ __launch_bounds__(NW * 64) void gemv_kernel(GemmArgs a, int m0, Epilogue epi)
{
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                  // [MT][4][nblk] chunks
    uint32_t* lut = reinterpret_cast<uint32_t*>(smem + (size_t)MT * a.k * 2);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform, kept scalar
    const int nblk = a.k >> 5;
    const int steps = (nblk + 63) >> 6;
    const int tail_blocks = nblk - (steps - 1) * 64;                 // blocks in the last step (1..64)
    const int n_groups = (a.n + R - 1) / R;
    const int total_waves = gridDim.x * NW;
    const int first_group = (int)blockIdx.x * NW + wave;
    const int q_row_bytes = a.k >> 1;
    const bool argmax = a.part_val != nullptr;

    // Buffer descriptors: all addressing is a scalar offset (row, step) plus lane * 16.
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.q), 0, a.n * q_row_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.s), 0, a.n * nblk, 0x00020000);

    auto valid = [&](const Pos& p) { return p.g < n_groups; };
    auto advance = [&](Pos& p) {
        if (++p.t == steps) {
            p.t = 0;
            p.g += total_waves;
        }
    };
    // the lane's block within step t; lanes past the end of a ragged last step re-read its last block
    auto lane_block = [&](int t) { return (t == steps - 1 && lane >= tail_blocks) ? tail_blocks - 1 : lane; };
    // Always the same number of loads, so that the hardware's in-order load counter can be
    // waited on precisely.  Past the wave's last position the lane offset is pushed beyond the
    // descriptor's range: such loads touch no memory and return zero.
    //
    // Scales.  Byte scheme: one byte load per row, the lane's own block.  Dword scheme (needs
    // K % 128 == 0 so that every dword is aligned and inside its row): the 64 scale bytes of a
    // step are 16 dwords per row; lane l loads dword (l % 16) of row (l / 16) % R, so ONE load
    // brings all R rows' scales of the step, and compute() fetches each row's byte from the lane
    // that holds it with ds_bpermute.
    const int srow = (lane >> 4) % R;
    auto issue = [&](const Pos& p, Item<R, kScaleDword>& it) {
        const bool live = valid(p);
        const int lb = lane_block(p.t);
        const int voff_q = live ? lb * 16 : 0x7FFFFFF0;
        const int g = live ? p.g : 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = min(g * R + r, a.n - 1);                  // ragged N: re-read the last row
            it.q[r] = __builtin_amdgcn_raw_buffer_load_b128(rq, voff_q, row * q_row_bytes + p.t * 1024, 2);
            if constexpr (!kScaleDword) {
                const int voff_s = live ? lb : 0x7FFFFFF0;
                it.s[r] = __builtin_amdgcn_raw_buffer_load_b8(rs, voff_s, row * nblk + p.t * 64, 2);
            }
        }
        if constexpr (kScaleDword) {
            const int row = min(g * R + srow, a.n - 1);
            const int voff_s = live ? row * nblk + (lane & 15) * 4 : 0x7FFFFFF0;
            it.s[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff_s, p.t * 64, 0);   // a row's scale line serves all its steps: cached
        }
    };

    // Prologue.  The activation loads go out first and the first D steps of weight loads right
    // behind them; only the activations are waited for before the LDS copy, so the weights stay
    // in flight across the barrier.  Chunk c (8 elements) of row m goes to [m][c & 3][c >> 2].
    Item<R, kScaleDword> buf[D];
    Pos pos[D];
    Pos load{first_group, 0};
    {
        const int chunks = a.k >> 3;
        constexpr int T = NW * 64;
        u32x4_t xr[MT][kXRegChunks];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const int msrc = min(m0 + m, a.m - 1);                   // ragged M: repeat the last row
            const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
#pragma unroll
            for (int i = 0; i < kXRegChunks; ++i)
                xr[m][i] = xp[min(tid + i * T, chunks - 1)];
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            pos[d] = load;
            issue(load, buf[d]);
            advance(load);
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int i = 0; i < kXRegChunks; ++i) {
                const int c = min(tid + i * T, chunks - 1);          // clamped duplicates rewrite the same data
                xs[(m * 4 + (c & 3)) * nblk + (c >> 2)] = xr[m][i];
            }
            if (chunks > kXRegChunks * T) {                          // long rows: the rest, the slow way
                const int msrc = min(m0 + m, a.m - 1);
                const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
                for (int c = tid + kXRegChunks * T; c < chunks; c += T)
                    xs[(m * 4 + (c & 3)) * nblk + (c >> 2)] = xp[c];
            }
        }
        if constexpr (kDecode == kLut) {
            for (int e = tid; e < 256 * 32; e += NW * 64) {
                const uint32_t byte = (uint32_t)e >> 5;
                const uint32_t lo = __float_as_uint(e2m1_to_f32(byte & 0xFu)) >> 16;
                const uint32_t hi = __float_as_uint(e2m1_to_f32(byte >> 4)) >> 16;
                lut[e] = lo | (hi << 16);
            }
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
    int slots = 0;               // outputs held in res[]
    int flushed_groups = 0;      // row groups of this wave already written
    float acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MT; ++m)
            acc[r][m] = 0.f;

    // Write the held outputs: lane i owns the i-th row finished since the last flush.  Stores
    // and loads share one completion counter but complete out of order with respect to each
    // other, so the counter is drained here; the main loop then only ever sees loads in flight.
    auto flush = [&]() {
        const int j = lane / R, r = lane - j * R;
        const int row = (first_group + (flushed_groups + j) * total_waves) * R + r;
        if constexpr (!kEpi) {
            if (lane < slots && row < a.n) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    if (m0 + m < a.m)
                        a.y[(int64_t)(m0 + m) * a.ldy + row] = f32_to_bf16_rne(res[m]);
            }
        } else {
            const bool gated = epi.act == MXFP4_ACT_SWIGLU;
            const bool own = lane < slots && row < a.n;
            const bool writer = own && !(gated && (lane & 1));        // even lanes hold the gate rows
            const int col = gated ? row >> 1 : row;
            float bv = 0.f, rv[MT];
            if (epi.bias && own)
                bv = bf16_bits_to_f32(epi.bias[row]);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                rv[m] = 0.f;
                if (epi.residual && writer && m0 + m < a.m)
                    rv[m] = bf16_bits_to_f32(epi.residual[(int64_t)(m0 + m) * epi.ldr + col]);
            }
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float v = res[m] + bv;
                const float up = __shfl_down(v, 1);
                if (gated)
                    v = silu_gate(v, up);
                if (writer && m0 + m < a.m)
                    a.y[(int64_t)(m0 + m) * a.ldy + col] = f32_to_bf16_rne(v + rv[m]);
            }
        }
        flushed_groups += slots / R;
        slots = 0;
        drain_vmem();
    };

    auto compute = [&](const Pos& p, Item<R, kScaleDword>& it) {
        const int lb = lane_block(p.t);
        const int bc = p.t * 64 + lb;
        u32x4_t xv[MT][4];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xv[m][j] = xs[(m * 4 + j) * nblk + bc];
        if (p.t == steps - 1 && lane >= tail_blocks) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                it.q[r] = u32x4_t{0, 0, 0, 0};                        // all nibbles +0
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            uint32_t sbyte;
            if constexpr (kScaleDword) {
                // the dword with this lane's scale of row r sits in lane r*16 + lb/4, byte lb%4
                const uint32_t dw = (uint32_t)__builtin_amdgcn_ds_bpermute((r * 16 + (lb >> 2)) * 4, (int)it.s[0]);
                sbyte = (dw >> ((lb & 3) * 8)) & 0xFFu;
            } else {
                sbyte = it.s[r];
            }
            // The scaled convert reads only the exponent field of its scale operand and treats it
            // as E8M0 (0 is 2^-127, 255 is NaN), so byte << 23 is the whole conversion there.
            const float sc = kDecode == kCvt ? __uint_as_float(sbyte << 23) : e8m0_to_f32(sbyte);
            float part[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m)
                part[m] = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t qd = it.q[r][j];
                uint32_t xd[MT][4];
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    xd[m][0] = xv[m][j][0];
                    xd[m][1] = xv[m][j][1];
                    xd[m][2] = xv[m][j][2];
                    xd[m][3] = xv[m][j][3];
                }
                if constexpr (kDecode == kCvt) {
                    bf16x2_t w[4];
                    w[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 0);
                    w[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 1);
                    w[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 2);
                    w[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 3);
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
                        const uint32_t byte = (qd >> (8 * p4)) & 0xFFu;
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
                        const uint32_t byte = (qd >> (8 * p4)) & 0xFFu;
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
            // end of the row group: sum the lanes' partials, then hold or compare the totals
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

    // Positions only grow, so the walk ends when buffer 0 runs dry.  Every trip issues the same
    // loads whether or not the later buffers still had work: every path into the loop head then
    // carries the same queue of outstanding loads and the compiler's counter waits stay exact
    // (an exit path that rejoins the back edge with a shorter queue makes it wait for everything).
    while (valid(pos[0])) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
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
        // combine the waves of the workgroup, then publish one partial winner per row
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

// Second stage of the fused argmax: one wave per activation row reduces the partial winners in
// (value descending, index ascending) order.  No LDS and no barrier: the kernel is all latency.
__global__ __launch_bounds__(64) void argmax_finish_kernel(const float* __restrict__ part_val,
                                                           const int32_t* __restrict__ part_idx,
                                                           int parts, int parts_used,
                                                           int32_t* __restrict__ argmax_out,
                                                           float* __restrict__ max_out)
{
    const int m = blockIdx.x, lane = threadIdx.x;
    const float* pv = part_val + (int64_t)m * parts;
    const int32_t* pi = part_idx + (int64_t)m * parts;
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int p0 = lane; p0 < parts_used; p0 += 64 * 8) {
        float v[8];
        int i[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {                   // eight independent loads in flight
            const int p = p0 + 64 * u;
            v[u] = p < parts_used ? pv[p] : -INFINITY;
            i[u] = p < parts_used ? pi[p] : 0x7FFFFFFF;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (v[u] > bv || (v[u] == bv && i[u] < bi)) {
                bv = v[u];
                bi = i[u];
            }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float v = __shfl_xor(bv, off);
        const int i = __shfl_xor(bi, off);
        if (v > bv || (v == bv && i < bi)) {
            bv = v;
            bi = i;
        }
    }
    if (lane == 0) {
        // every accumulator -inf or NaN: report index 0 rather than the sentinel
        argmax_out[m] = bi == 0x7FFFFFFF ? 0 : bi;
        if (max_out)
            max_out[m] = bv;
    }
}

// The argmax's second stage with the draft verification fused behind it (arXiv 2503.13565,
// section 3.1: the draft tokens after the first mismatch with the target's own picks are
// dropped).  One workgroup: wave w reduces the partial winners of rows w, w + 16, ...; the picks
// meet in LDS; then accept[0] = G, the number of leading draft tokens that equal the picks, and
// accept[1] = the pick at position G (the extra token the verification pass yields).  M - 1
// draft tokens for M rows; M <= kVerifyMaxRows.
__global__ __launch_bounds__(1024) void verify_finish_kernel(const float* __restrict__ part_val,
                                                             const int32_t* __restrict__ part_idx, int parts,
                                                             int parts_used, int m_rows,
                                                             const int32_t* __restrict__ draft,
                                                             int32_t* __restrict__ argmax_out,
                                                             float* __restrict__ max_out,
                                                             int32_t* __restrict__ accept)
{
    __shared__ int tok[kVerifyMaxRows];
    __shared__ int first;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0)
        first = m_rows - 1;
    for (int m = wave; m < m_rows; m += 16) {
        const float* pv = part_val + (int64_t)m * parts;
        const int32_t* pi = part_idx + (int64_t)m * parts;
        float bv = -INFINITY;
        int bi = 0x7FFFFFFF;
        for (int p0 = lane; p0 < parts_used; p0 += 64 * 8) {
            float v[8];
            int i[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + 64 * u;
                v[u] = p < parts_used ? pv[p] : -INFINITY;
                i[u] = p < parts_used ? pi[p] : 0x7FFFFFFF;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (v[u] > bv || (v[u] == bv && i[u] < bi)) {
                    bv = v[u];
                    bi = i[u];
                }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float v = __shfl_xor(bv, off);
            const int i = __shfl_xor(bi, off);
            if (v > bv || (v == bv && i < bi)) {
                bv = v;
                bi = i;
            }
        }
        if (lane == 0) {
            bi = bi == 0x7FFFFFFF ? 0 : bi;
            tok[m] = bi;
            argmax_out[m] = bi;
            if (max_out)
                max_out[m] = bv;
        }
    }
    __syncthreads();
    if (tid < m_rows - 1 && draft[tid] != tok[tid])
        atomicMin(&first, tid);                         // LDS atomic: the first mismatch
    __syncthreads();
    if (tid == 0) {
        accept[0] = first;
        accept[1] = tok[first];
    }
}

int gemv_max_parts(const DeviceInfo& dev) { return dev.cus * 8; }

namespace {

// Launch shape: rows per group, register buffers, waves per workgroup, workgroups per CU.
struct Tune {
    int r, d, nw, wgs_per_cu;
    bool byte_scales;       // force the byte scale loads even when K allows the dword scheme
};

// Rows per group: two (measured 5 % faster than four over the 7B decode linears: more, shorter
// row groups balance the tail better), one when the matrix is so short that SIMDs would idle.
Tune default_tune(int n_rows, int cus)
{
    const int want_groups = cus * 16;
    int r = 2;
    while (r > 1 && (n_rows + r - 1) / r < want_groups)
        r >>= 1;
    return Tune{r, 2, 4, 4, false};
}

// MXFP4_GEMV_TUNE="R,D,NW,WGS[,B]" overrides the launch shape (measurement only; R = 0 keeps
// the default rows per group, B = 1 forces byte scale loads).
bool env_tune(Tune* out)
{
    static Tune t;
    static const bool have = [] {
        if (const char* e = knob("MXFP4_GEMV_TUNE")) {
            int r, d, nw, w, b = 0;
            if (sscanf(e, "%d,%d,%d,%d,%d", &r, &d, &nw, &w, &b) >= 4) {
                t = Tune{r, d, nw, w, b != 0};
                return true;
            }
        }
        return false;
    }();
    if (have)
        *out = t;
    return have;
}

template <int MT, int R, int D, int NW, int kDecode, bool kScaleDword, bool kEpi>
hipError_t launch_one(const GemmArgs& a, int m0, int blocks, size_t lds, int max_lds, hipStream_t stream,
                      const Epilogue& epi)
{
    auto kern = gemv_kernel<MT, R, D, NW, kDecode, kScaleDword, kEpi>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), max_lds); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, stream, a, m0, epi);
    return hipGetLastError();
}

// The fused form exists for the convert decode only (the one AUTO uses).
template <int MT, int R, int D, int NW, int kDecode, bool kScaleDword>
hipError_t launch_either(const GemmArgs& a, int m0, int blocks, size_t lds, int max_lds, hipStream_t stream,
                         const Epilogue* epi)
{
    if (!epi)
        return launch_one<MT, R, D, NW, kDecode, kScaleDword, false>(a, m0, blocks, lds, max_lds, stream, Epilogue{});
    if constexpr (kDecode == kCvt)
        return launch_one<MT, R, D, NW, kDecode, kScaleDword, true>(a, m0, blocks, lds, max_lds, stream, *epi);
    return hipErrorInvalidValue;
}

template <int MT, int kDecode>
hipError_t launch_shape(const GemmArgs& a, int m0, const Tune& t, int blocks, size_t lds, int max_lds,
                        hipStream_t stream, const Epilogue* epi)
{
    const bool sd = (a.k % 128 == 0) && !t.byte_scales;
#define MXFP4_CASE(R_, D_, NW_)                                                                            \
    if (t.r == R_ && t.d == D_ && t.nw == NW_)                                                             \
        return sd ? launch_either<MT, R_, D_, NW_, kDecode, true>(a, m0, blocks, lds, max_lds, stream, epi)  \
                  : launch_either<MT, R_, D_, NW_, kDecode, false>(a, m0, blocks, lds, max_lds, stream, epi);
    MXFP4_CASE(4, 2, 4)
    MXFP4_CASE(2, 2, 4)
    MXFP4_CASE(1, 2, 4)
    if constexpr (kDecode == kCvt) {
        MXFP4_CASE(4, 3, 4)
        MXFP4_CASE(2, 3, 4)
        MXFP4_CASE(2, 4, 4)
        MXFP4_CASE(1, 3, 4)
        MXFP4_CASE(1, 4, 4)
        MXFP4_CASE(4, 2, 8)
        MXFP4_CASE(2, 2, 8)
        MXFP4_CASE(2, 4, 8)
        MXFP4_CASE(1, 4, 8)
    }
#undef MXFP4_CASE
    return hipErrorInvalidValue;
}

template <int kDecode>
hipError_t launch_decode(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream,
                         const Epilogue* epi)
{
    Tune t = default_tune(a.n, dev.cus);
    if constexpr (kDecode == kCvt) {
        Tune e;
        if (env_tune(&e)) {
            if (e.r == 0)
                e.r = t.r;
            t = e;
        }
    }
    if (epi && epi->act == MXFP4_ACT_SWIGLU && t.r == 1)
        t.r = 2;                                    // a group must hold whole (gate, up) pairs
    const size_t extra = kDecode == kLut ? (size_t)kLutBytes : 0;
    // two activation rows per pass when their LDS copy fits, else one
    const bool two_fit = (size_t)2 * a.k * 2 + extra <= (size_t)dev.lds_bytes;
    const int n_groups = (a.n + t.r - 1) / t.r;
    int blocks = (n_groups + t.nw - 1) / t.nw;
    if (blocks > dev.cus * t.wgs_per_cu)
        blocks = dev.cus * t.wgs_per_cu;
    if (blocks > gemv_max_parts(dev))
        blocks = gemv_max_parts(dev);
    if (parts_used)
        *parts_used = blocks;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        hipError_t e;
        if (left >= 2 && two_fit) {
            e = launch_shape<2, kDecode>(a, m0, t, blocks, (size_t)2 * a.k * 2 + extra, dev.lds_bytes, stream, epi);
            m0 += 2;
        } else {
            e = launch_shape<1, kDecode>(a, m0, t, blocks, (size_t)a.k * 2 + extra, dev.lds_bytes, stream, epi);
            m0 += 1;
        }
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

}  // namespace

hipError_t launch_gemv(const GemmArgs& a, int decode, bool argmax, const DeviceInfo& dev, int* parts_used,
                       hipStream_t stream, const Epilogue* epi)
{
    (void)argmax;                                   // the kernels look at a.part_val
    switch (decode) {
    case kBits:
        return launch_decode<kBits>(a, dev, parts_used, stream, epi);
    case kCvt:
        return launch_decode<kCvt>(a, dev, parts_used, stream, epi);
    case kLut:
        return launch_decode<kLut>(a, dev, parts_used, stream, epi);
    default:
        return hipErrorInvalidValue;
    }
}

hipError_t launch_argmax_finish(const float* part_val, const int32_t* part_idx, int parts, int parts_used,
                                int m, int32_t* argmax_out, float* max_out, hipStream_t stream)
{
    hipLaunchKernelGGL(argmax_finish_kernel, dim3(m), dim3(64), 0, stream, part_val, part_idx, parts,
                       parts_used, argmax_out, max_out);
    return hipGetLastError();
}

hipError_t launch_verify_finish(const float* part_val, const int32_t* part_idx, int parts, int parts_used,
                                int m, const int32_t* draft, int32_t* argmax_out, float* max_out,
                                int32_t* accept_out, hipStream_t stream)
{
    if (m < 1 || m > kVerifyMaxRows)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(verify_finish_kernel, dim3(1), dim3(1024), 0, stream, part_val, part_idx, parts,
                       parts_used, m, draft, argmax_out, max_out, accept_out);
    return hipGetLastError();
}

}  // namespace mxfp4
