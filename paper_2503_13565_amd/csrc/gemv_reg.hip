// The decode-step form of the skinny product y = x * dequant(W)^T (arXiv 2503.13565, section
// 3.4.3 and Eq. 2; section 4.4: the product with one token must run at memory speed): one or
// two activation rows, reduction lengths up to 12288, activations held in registers.
//
// What differs from the general kernel in gemv.hip:
//   - A lane always works on the same scale blocks of a row (block t*64 + lane in step t), so
//     its 32 activations per step never change.  They are staged through LDS once (one global
//     read per workgroup) and then live in registers: the streaming loop has no LDS reads.
//   - One workgroup per compute unit, 8, 12 or 16 waves.  The rows of a workgroup are handed to its
//     waves through an LDS counter, one row at a time: the memory system serves the waves of a
//     compute unit very unevenly (the first data reaches them 2 to 6 us after the launch), and
//     with a fixed share per wave the slowest wave set the kernel time.
//   - One weight row per wave step (1 KiB per load instruction), two steps in flight per wave:
//     32 KiB in flight per compute unit, which is where a plain read stream peaks here.
// Decode and multiply-add are as in gemv.hip: the scaled FP4->BF16 convert with the block scale,
// then v_dot2_f32_bf16 with FP32 accumulation (Eq. 2: scaling a power of two commutes with the
// sum of the block).
#include <stdlib.h>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

namespace {

// The kernel arguments are 15 dwords of plain scalars so that they can be preloaded into scalar
// registers when the wave starts (the build passes -amdgpu-kernarg-preload-count=16): every wave
// needs them before it can send its first load.  Measured per launch: a second 64-byte line of
// arguments costs 0.4 us, fetching one line instead of having it preloaded 0.15 us.
struct RegArgs {
    const uint16_t* x;
    const uint8_t* q;
    const uint8_t* s;
    void* out;           // y (BF16 [M, N]), or in the argmax form the partial winners: float
                         // [M, parts] followed by int32 [M, parts]
    int n, k, m, m0;
    int ldx, ldy;
    int parts;           // > 0: argmax form
};

// MT activation rows, STEPS (even) steps of 64 blocks cover K (the last ones may be ragged or
// empty), D step buffers, NW waves per workgroup.  kRagged: K is not STEPS * 2048.
// R weight rows per wave step (a group); group i of workgroup b's sequence is i * gridDim.x + b.
// Epi: NoEpilogue, or Epilogue for the fused form (bias, gate, residual at the flush).  The gate
// needs a pair of rows 2c, 2c + 1 in neighbouring lanes of the held outputs: with R = 2 a group is
// a pair; with R = 1 the counter deals pairs and a wave takes the pair's rows in two trips.
// kBits: 4 (E2M1 nibbles, 16 bytes per block) or 6 (E2M3 codes, 24 bytes per block; one
// v_cvt_scalef32_pk32_bf16_fp6 decodes the whole block).  A wave step of the 6-bit form is 1536
// bytes of a row.  Loading a lane's own 24 bytes directly (16 + 8 at a stride of 24) leaves every
// wave instruction with misaligned, gapped accesses and costs 16 to 21 % of the kernel's time;
// instead the wave loads the 1536 bytes lane-contiguous (16 bytes per lane, then 8), passes them
// through 1536 bytes of LDS of its own and reads back bytes [24 lane, 24 lane + 24).
// Format codes 22 and 24 are the second element formats of those widths (E3M2, E5M2): the same frame
// with the other convert instruction.  Format code 2: the 2-bit ternary codes (8 bytes per block, one
// 64-bit load per lane and step, bit-move decode, late scaling by X / 2).
// kBits 8 (E4M3 bytes, 32 bytes per block, 2048 bytes per wave step): loaded lane-contiguous too
// (16 bytes per lane, twice), and no exchange is needed: a lane keeps what it loaded, two half
// blocks -- elements [16 lane, 16 lane + 16) of the step, block lane / 2, and the same 1024
// elements further, block 32 + lane / 2 -- each with its own scale, and holds the activations of
// exactly those elements (four 16-byte chunks per step, as in the other forms).
typedef __attribute__((ext_vector_type(32))) __bf16 bf16x32_t;
typedef __attribute__((ext_vector_type(6))) unsigned int u32x6_t;
typedef __attribute__((ext_vector_type(16))) unsigned int u32x16_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;

template <int MT, int R, int STEPS, int D, int NW, bool kRagged, class Epi, int kFmt = 4>
__device__ __forceinline__ void gemv_reg_body(const RegArgs& a, const Epi& epi)
{
    // kFmt: the element width, + 16 for the second element format of that width (22: E3M2 in place of
    // E2M3, 24: E5M2 in place of E4M3): same loads and lane mapping, the other convert instruction
    constexpr bool kAlt = kFmt > 16;
    constexpr int kBits = kAlt ? kFmt - 16 : kFmt;
    static_assert(kBits == 4 || kBits == 6 || kBits == 8 || kBits == 2, "element width");
    static_assert(!kAlt || (kBits != 4 && kBits != 2), "the 4-bit and 2-bit formats have one element format");
    // kBits 2: the 2-bit ternary codes, 8 bytes per block, 512 bytes of a row per wave step (one 64-bit load
    // per lane); the activations in registers are what this frame gives the format: in the general
    // kernel a block's 8 bytes of weights pull 64 bytes of activations out of the LDS.
    constexpr int kBlkBytes = kBits == 8 ? 32 : (kBits == 6 ? 24 : (kBits == 2 ? 8 : 16));
    constexpr bool kEpi = !__is_same(Epi, NoEpilogue);
    const int m0 = a.m0;
    static_assert(STEPS % D == 0, "the buffer of a step must be known at compile time");
    constexpr int T = NW * 64;
    constexpr int XPR = (STEPS * 256 + T - 1) / T;          // 16-byte activation chunks per thread and row
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int chunks = a.k >> 3;

    // The activation loads go out before anything else is computed.  Every wave sends its weight
    // loads right behind its own activation loads, and a compute unit serves its loads in order:
    // an activation load that leaves late queues behind the weights of the waves that started
    // earlier and holds the whole workgroup at the barrier below (measured: 50 instructions of
    // address arithmetic in front of it cost 1 us per launch).
    u32x4_t xl[MT][XPR];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int msrc = min(m0 + m, a.m - 1);                       // ragged M: repeat the last row
        const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
#pragma unroll
        for (int i = 0; i < XPR; ++i)
            xl[m][i] = xp[min(tid + i * T, chunks - 1)];
    }

    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);         // [MT][4][nblk] chunks
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nblk = a.k >> 5;
    // Activations that stay in LDS (see below) use rows of STEPS * 64 chunks, zero beyond K: the
    // loop then reads them without a check and every address is a constant away from one base.
    constexpr bool kXLds = MT * STEPS >= 6;
    const int xrow = kXLds ? STEPS * 64 : nblk;              // chunks per (activation row, j)
    int* ctr = reinterpret_cast<int*>(smem + (size_t)MT * 4 * xrow * 16);
    // 6-bit form: R * 1536 bytes per wave behind the counter's 64
    uint8_t* stage = smem + (size_t)MT * 4 * xrow * 16 + 64 + (size_t)wave * (R * 1536);
    const int q_row_bytes = (a.k >> 5) * kBlkBytes;
    const bool argmax = a.parts > 0;
    const int G = gridDim.x, b = blockIdx.x;
    bool gated = false;
    if constexpr (kEpi)
        gated = epi.act == MXFP4_ACT_SWIGLU;
    const bool pair_trips = kEpi && R == 1 && gated;                 // a dealt index is a pair of rows
    const int per_index = pair_trips ? 2 : 1;
    auto row_of = [&](int i) { return (i * G + b) * per_index; };

    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.q), 0, a.n * q_row_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.s), 0, a.n * nblk, 0x00020000);

    if (tid == 0)
        *ctr = NW;                                                   // indices 0..NW-1 are the waves' first rows

    // Fused form: a row's bias and residual are fetched when its trip starts (one broadcast load
    // each, behind descriptors that cover nothing when the operand is absent) and kept with its
    // slot, so the flush has nothing to wait for.
    Epilogue ep{nullptr, nullptr, 0, 0};
    if constexpr (kEpi)
        ep = epi;
    float bias_s = 0.f, res_s[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
        res_s[m] = 0.f;
    const __amdgpu_buffer_rsrc_t rb =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(ep.bias), 0, ep.bias ? a.n * 2 : 0, 0x00020000);
    auto residual_row = [&](int m) {
        return __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(ep.residual + (int64_t)min(a.m0 + m, a.m - 1) * ep.ldr), 0,
            ep.residual ? (gated ? a.n >> 1 : a.n) * 2 : 0, 0x00020000);
    };
    const __amdgpu_buffer_rsrc_t rr0 = residual_row(0), rr1 = residual_row(MT - 1);

    u32x4_t bq[D][R];
    u32x2_t bq2[D][kBits == 6 || kBits == 2 ? R : 1];   // bytes 16..23 of a 6-bit block; the 8 bytes of a 2-bit one
    u32x4_t bqb[D][kBits == 8 ? R : 1];             // 8-bit form: the lane's second 16 bytes
    uint32_t bs[D];
    const int n_groups = (a.n + R - 1) / R;
    const int srow = (lane >> 4) % R;
    // A step always issues the same loads so that the in-order load counter can be waited on
    // exactly; past the end (of the groups, or of a ragged K) the lane offset is pushed out of the
    // descriptor's range: such loads touch no memory and return zero.
    // (nb: the blocks per row again, for the 6-bit form, which hands in a copy the compiler cannot
    // see through once per trip: two lane masks per step kept in registers across the whole row
    // loop made every long-K instance spill)
    auto issue = [&](int grp, int t, int d, int nb) {
        const bool live = grp < n_groups;
        const bool vb = !kRagged || t * 64 + lane < nblk;
        const int g0 = live ? grp * R : 0;
        // 6-bit form: the step's valid bytes are 24 per block left in the row (a multiple of 96)
        const int valid6 = kRagged ? 24 * max(0, min(64, nb - t * 64)) : 1536;
        const int valid8 = kRagged ? 32 * max(0, min(64, nb - t * 64)) : 2048;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = min(g0 + r, a.n - 1);                    // odd N: the last row twice
            if constexpr (kBits == 6) {
                bq[d][r] = __builtin_amdgcn_raw_buffer_load_b128(
                    rq, (live && lane * 16 < valid6) ? lane * 16 : 0x7FFFFFF0, row * q_row_bytes + t * 1536, 2);
                bq2[d][r] = __builtin_amdgcn_raw_buffer_load_b64(
                    rq, (live && 1024 + lane * 8 < valid6) ? 1024 + lane * 8 : 0x7FFFFFF0,
                    row * q_row_bytes + t * 1536, 2);
            } else if constexpr (kBits == 8) {
                bq[d][r] = __builtin_amdgcn_raw_buffer_load_b128(
                    rq, (live && lane * 16 < valid8) ? lane * 16 : 0x7FFFFFF0, row * q_row_bytes + t * 2048, 2);
                bqb[d][r] = __builtin_amdgcn_raw_buffer_load_b128(
                    rq, (live && 1024 + lane * 16 < valid8) ? 1024 + lane * 16 : 0x7FFFFFF0,
                    row * q_row_bytes + t * 2048, 2);
            } else if constexpr (kBits == 2) {
                bq2[d][r] = __builtin_amdgcn_raw_buffer_load_b64(rq, (live && vb) ? lane * kBlkBytes : 0x7FFFFFF0,
                                                                 row * q_row_bytes + t * (64 * kBlkBytes), 2);
            } else {
                bq[d][r] = __builtin_amdgcn_raw_buffer_load_b128(rq, (live && vb) ? lane * kBlkBytes : 0x7FFFFFF0,
                                                                 row * q_row_bytes + t * (64 * kBlkBytes), 2);
            }
        }
        // scale bytes of the step: 16 dwords per row; lane l loads dword l % 16 of row (l / 16) % R
        const int row = min(g0 + srow, a.n - 1);
        bs[d] = __builtin_amdgcn_raw_buffer_load_b32(rs, live ? row * nblk + (lane & 15) * 4 : 0x7FFFFFF0,
                                                     t * 64, 0);
    };
    int grp = row_of(wave);
#pragma unroll
    for (int d = 0; d < D; ++d)
        issue(grp, d, d, nblk);

#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < XPR; ++i) {
            const int c = min(tid + i * T, chunks - 1);              // clamped duplicates rewrite the same data
            xs[(m * 4 + (c & 3)) * xrow + (c >> 2)] = xl[m][i];
        }
    if constexpr (kXLds) {
        const int pad = xrow - nblk;
        for (int e = tid; e < MT * 4 * pad; e += T)
            xs[(e / pad) * xrow + nblk + e % pad] = u32x4_t{0, 0, 0, 0};
    }
    lds_barrier();
    // Up to 64 registers of activations per lane (four steps of one row, two steps of two rows);
    // beyond that they stay in the LDS copy and every step reads its 64 bytes per row from there.
    // (one base per activation row: every read of a row is then within the 64 KB that the LDS
    // instruction's offset field reaches, and no address has to be kept in a register)
    // 8-bit form: chunk j of the lane is chunk 2 (lane % 2) + j % 2 of block lane / 2 + 32 (j / 2)
    const u32x4_t* xrow0 = kBits == 8 ? xs + 2 * (lane & 1) * xrow + (lane >> 1) : xs + lane;
    const u32x4_t* xrow1 = xrow0 + (MT - 1) * 4 * STEPS * 64;
    auto x_of = [&](int m, int t, int j) {
        if constexpr (kBits == 8) {
            if constexpr (kXLds) {
                return (m == 0 ? xrow0 : xrow1)[((j & 1) * STEPS + t) * 64 + 32 * (j >> 1)];
            } else {
                const int blk = t * 64 + (lane >> 1) + 32 * (j >> 1);
                return (!kRagged || blk < nblk) ? xs[(m * 4 + 2 * (lane & 1) + (j & 1)) * nblk + blk]
                                                : u32x4_t{0, 0, 0, 0};
            }
        } else if constexpr (kXLds) {
            return (m == 0 ? xrow0 : xrow1)[(j * STEPS + t) * 64];
        } else {
            return (!kRagged || t * 64 + lane < nblk) ? xs[(m * 4 + j) * nblk + t * 64 + lane] : u32x4_t{0, 0, 0, 0};
        }
    };
    u32x4_t xr[kXLds ? 1 : MT][kXLds ? 1 : STEPS][4];
    if constexpr (!kXLds) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int t = 0; t < STEPS; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    xr[m][t][j] = x_of(m, t, j);
    }

    float best_val[MT];
    int best_idx[MT];
    float res[MT];                  // finished outputs, one per lane
    float acc[R][MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        best_val[m] = -INFINITY;
        best_idx[m] = 0x7FFFFFFF;
        res[m] = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r)
            acc[r][m] = 0.f;
    }
    int rowv = 0;                   // the row whose outputs this lane holds
    int slots = 0;

    // Stores and loads share one completion counter but complete out of order with respect to
    // each other, so the counter is drained here; the loop only ever sees loads in flight.
    auto flush = [&]() {
        if constexpr (!kEpi) {
            if (lane < slots && rowv < a.n) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    if (m0 + m < a.m)
                        static_cast<uint16_t*>(a.out)[(int64_t)(m0 + m) * a.ldy + rowv] = f32_to_bf16_rne(res[m]);
            }
        } else {
            // even lanes hold the gate rows, their right neighbours the up rows (slots fill in pairs)
            const bool own = lane < slots && rowv < a.n;
            const bool writer = own && !(gated && (lane & 1));
            const int col = gated ? rowv >> 1 : rowv;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float v = res[m] + bias_s;
                const float up = __shfl_down(v, 1);
                if (gated)
                    v = silu_gate(v, up);
                if (writer && m0 + m < a.m)
                    static_cast<uint16_t*>(a.out)[(int64_t)(m0 + m) * a.ldy + col] = f32_to_bf16_rne(v + res_s[m]);
            }
        }
        slots = 0;
        drain_vmem();
    };
    auto fetch = [&]() {
        int v = 0;
        if (lane == 0)
            v = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return __builtin_amdgcn_readfirstlane(v);
    };

    const int sh_top = (3 - (lane & 3)) * 8;        // brings this lane's scale byte to bits 31:24
    int i_next = fetch();
    bool second = false;                            // pair_trips: this trip takes the pair's second row
    while (grp < n_groups) {
        int grp_n, i_next2;
        if (pair_trips && !second) {
            grp_n = grp + 1;
            i_next2 = i_next;
        } else {
            grp_n = row_of(i_next);
            i_next2 = fetch();                      // consumed one trip later: its latency is hidden
        }
        second = !second;
        int nb = nblk;
        if constexpr (kBits != 4)
            asm volatile("" : "+s"(nb));
        uint32_t bias_l[R], res_l[R][MT];
        if constexpr (kEpi) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = grp * R + r;                // past N: outside the descriptors, reads zero
                bias_l[r] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rb, row * 2, 0, 0);
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    res_l[r][m] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(
                        m == 0 ? rr0 : rr1, (gated ? row >> 1 : row) * 2, 0, 0);
            }
        }
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            const int d = t % D;
            u32x4_t xq[MT][4];
            if constexpr (kXLds)
                __builtin_amdgcn_sched_barrier(0);  // step by step: across steps the scheduler piles up registers
#pragma unroll
            for (int j = 0; j < 4; ++j)             // in the order of use: chunk j of every activation row
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    if constexpr (kXLds)
                        xq[m][j] = x_of(m, t, j);
                    else
                        xq[m][j] = xr[m][t][j];
                }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if constexpr (kBits == 8) {
                    // scale bytes of blocks lane / 2 and 32 + lane / 2: dwords lane / 8 and 8 + lane / 8
                    // of the row's 16, byte (lane / 2) % 4 of either
                    const int src = (r * 16 + (lane >> 3)) * 4;
                    const int sh8 = (3 - ((lane >> 1) & 3)) * 8;
                    const uint32_t dwa = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)bs[d]);
                    const uint32_t dwb = (uint32_t)__builtin_amdgcn_ds_bpermute(src + 32, (int)bs[d]);
                    float sc2[2] = {__uint_as_float((dwa << sh8) >> 1), __uint_as_float((dwb << sh8) >> 1)};
                    if (kRagged) {
                        const int blk = t * 64 + (lane >> 1);
                        sc2[0] = blk < nblk ? sc2[0] : 1.0f;
                        sc2[1] = blk + 32 < nblk ? sc2[1] : 1.0f;
                    }
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        const u32x4_t piece = p ? bqb[d][r] : bq[d][r];
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj) {
                            const uint32_t qd0 = piece[2 * jj], qd1 = piece[2 * jj + 1];
                            bf16x2_t w[4];
                            if constexpr (kAlt) {
                                w[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(qd0, sc2[p], false);
                                w[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(qd0, sc2[p], true);
                                w[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(qd1, sc2[p], false);
                                w[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(qd1, sc2[p], true);
                            } else {
                                w[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(qd0, sc2[p], false);
                                w[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(qd0, sc2[p], true);
                                w[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(qd1, sc2[p], false);
                                w[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(qd1, sc2[p], true);
                            }
#pragma unroll
                            for (int m = 0; m < MT; ++m) {
                                const u32x4_t xv = xq[m][2 * p + jj];
                                const uint32_t x0 = xv[0], x1 = xv[1], x2 = xv[2], x3 = xv[3];
                                float c = acc[r][m];
                                c = __builtin_amdgcn_fdot2_f32_bf16(w[0], __builtin_bit_cast(bf16x2_t, x0), c, false);
                                c = __builtin_amdgcn_fdot2_f32_bf16(w[1], __builtin_bit_cast(bf16x2_t, x1), c, false);
                                c = __builtin_amdgcn_fdot2_f32_bf16(w[2], __builtin_bit_cast(bf16x2_t, x2), c, false);
                                c = __builtin_amdgcn_fdot2_f32_bf16(w[3], __builtin_bit_cast(bf16x2_t, x3), c, false);
                                acc[r][m] = c;
                            }
                        }
                    }
                    continue;
                }
                // the dword with this lane's scale byte of row r sits in lane r * 16 + lane / 4.
                // The scaled convert reads only the exponent field of its scale operand (as E8M0),
                // so the byte goes to bits 30:23 and whatever lands below is ignored.
                const uint32_t dw = (uint32_t)__builtin_amdgcn_ds_bpermute((r * 16 + (lane >> 2)) * 4, (int)bs[d]);
                float sc = __uint_as_float((dw << sh_top) >> 1);
                if (kRagged)
                    sc = (t * 64 + lane < nblk) ? sc : 1.0f;         // no NaN from a neighbour's scale byte
                if constexpr (kBits == 2) {
                    // codes -> BF16 +-2.0 / +-0 by bit moves, the block's sum scaled by X / 2 = 2^(byte - 128)
                    // afterwards (Eq. 2); bytes 0 and 1 give FP32 subnormals, 0xFF gives NaN
                    const uint32_t sb = (dw << sh_top) >> 24;
                    uint32_t bits = sb >= 2u ? (sb - 1u) << 23 : 0x00200000u << sb;
                    bits = sb == 0xFFu ? 0x7FC00000u : bits;
                    float late = __uint_as_float(bits);
                    if (kRagged)
                        late = (t * 64 + lane < nblk) ? late : 0.f;
                    uint32_t wv[16];
                    decode_t2(bq2[d][r][0], wv);
                    decode_t2(bq2[d][r][1], wv + 8);
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        float v = 0.f;
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const uint32_t xd = xq[m][i >> 2][i & 3];
                            v = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, wv[i]),
                                                                __builtin_bit_cast(bf16x2_t, xd), v, false);
                        }
                        acc[r][m] = __builtin_fmaf(v, late, acc[r][m]);
                    }
                    continue;
                }
                u32x16_t w6 = {};
                if constexpr (kBits == 6) {
                    // lane-contiguous bytes -> the lane's own block.  The buffer is the wave's alone
                    // and a wave's LDS instructions execute in order: no barrier, only the compiler
                    // must keep the order.
                    uint8_t* st = stage + r * 1536;
                    reinterpret_cast<u32x4_t*>(st)[lane] = bq[d][r];
                    reinterpret_cast<u32x2_t*>(st + 1024)[lane] = bq2[d][r];
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    const u32x2_t* rd = reinterpret_cast<const u32x2_t*>(st + lane * 24);
                    const u32x2_t p0 = rd[0], p1 = rd[1], p2 = rd[2];
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    const u32x6_t packed = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1]};
                    if constexpr (kAlt)
                        w6 = __builtin_bit_cast(u32x16_t, __builtin_amdgcn_cvt_scalef32_pk32_bf16_bf6(packed, sc));
                    else
                        w6 = __builtin_bit_cast(u32x16_t, __builtin_amdgcn_cvt_scalef32_pk32_bf16_fp6(packed, sc));
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bf16x2_t w[4];
                    if constexpr (kBits == 6) {
                        const uint32_t w0 = w6[4 * j], w1 = w6[4 * j + 1], w2 = w6[4 * j + 2], w3 = w6[4 * j + 3];
                        w[0] = __builtin_bit_cast(bf16x2_t, w0);
                        w[1] = __builtin_bit_cast(bf16x2_t, w1);
                        w[2] = __builtin_bit_cast(bf16x2_t, w2);
                        w[3] = __builtin_bit_cast(bf16x2_t, w3);
                    } else {
                        const uint32_t qd = bq[d][r][j];
                        w[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 0);
                        w[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 1);
                        w[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 2);
                        w[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 3);
                    }
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        // through scalars: a bit cast applied directly to a vector element reads element 0
                        const uint32_t x0 = xq[m][j][0], x1 = xq[m][j][1], x2 = xq[m][j][2], x3 = xq[m][j][3];
                        float c = acc[r][m];
                        c = __builtin_amdgcn_fdot2_f32_bf16(w[0], __builtin_bit_cast(bf16x2_t, x0), c, false);
                        c = __builtin_amdgcn_fdot2_f32_bf16(w[1], __builtin_bit_cast(bf16x2_t, x1), c, false);
                        c = __builtin_amdgcn_fdot2_f32_bf16(w[2], __builtin_bit_cast(bf16x2_t, x2), c, false);
                        c = __builtin_amdgcn_fdot2_f32_bf16(w[3], __builtin_bit_cast(bf16x2_t, x3), c, false);
                        acc[r][m] = c;
                    }
                }
            }
            const int tn = t + D;
            if (tn < STEPS)
                issue(grp, tn, d, nb);
            else
                issue(grp_n, tn - STEPS, d, nb);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = grp * R + r;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const float v = wave_sum(acc[r][m]);
                acc[r][m] = 0.f;
                if (argmax) {
                    // rows arrive in any order: the lower index wins among equal values
                    if (row < a.n && (v > best_val[m] || (v == best_val[m] && row < best_idx[m]))) {
                        best_val[m] = v;
                        best_idx[m] = row;
                    }
                } else {
                    res[m] = (lane == slots + r) ? v : res[m];
                }
            }
            if (!argmax)
                rowv = (lane == slots + r) ? row : rowv;
            if constexpr (kEpi) {
                bias_s = (lane == slots + r) ? bf16_bits_to_f32(bias_l[r]) : bias_s;
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    res_s[m] = (lane == slots + r) ? bf16_bits_to_f32(res_l[r][m]) : res_s[m];
            }
        }
        if (!argmax) {
            slots += R;
            if (slots + R > 64)
                flush();
        }
        grp = grp_n;
        i_next = i_next2;
    }
    if (!argmax && slots > 0)
        flush();

    if (argmax) {
        // combine the waves of the workgroup, then publish one partial winner per activation row
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
            float* part_val = static_cast<float*>(a.out);
            int32_t* part_idx = reinterpret_cast<int32_t*>(part_val + (int64_t)a.m * a.parts);
            part_val[(int64_t)(m0 + tid) * a.parts + b] = bv;
            part_idx[(int64_t)(m0 + tid) * a.parts + b] = bi;
        }
    }
}

template <int MT, int R, int STEPS, int D, int NW, bool kRagged>
__global__ __launch_bounds__(NW * 64) void gemv_reg_kernel(const uint16_t* x, const uint8_t* q, const uint8_t* s,
                                                           void* out, int n, int k, int m, int m0, int ldx,
                                                           int ldy, int parts)
{
    gemv_reg_body<MT, R, STEPS, D, NW, kRagged>(RegArgs{x, q, s, out, n, k, m, m0, ldx, ldy, parts}, NoEpilogue{});
}

// The fused form: `act` decides which rows a wave starts with, so it takes the last preloaded
// slot; the other epilogue arguments come behind and are first needed when the first trip starts.
template <int MT, int R, int STEPS, int D, int NW, bool kRagged>
__global__ __launch_bounds__(NW * 64) void gemv_reg_fused_kernel(const uint16_t* x, const uint8_t* q,
                                                                 const uint8_t* s, void* out, int n, int k, int m,
                                                                 int m0, int ldx, int ldy, int parts, int act,
                                                                 const uint16_t* bias, const uint16_t* residual,
                                                                 int ldr)
{
    gemv_reg_body<MT, R, STEPS, D, NW, kRagged>(RegArgs{x, q, s, out, n, k, m, m0, ldx, ldy, parts},
                                                Epilogue{bias, residual, ldr, act});
}

// The 6-bit format (q = q6, 24 bytes per block) and the 8-bit format (q = q8, 32 bytes per block).
template <int MT, int R, int STEPS, int D, int NW, bool kRagged, int kBits>
__global__ __launch_bounds__(NW * 64) void gemv_reg6_kernel(const uint16_t* x, const uint8_t* q, const uint8_t* s,
                                                            void* out, int n, int k, int m, int m0, int ldx,
                                                            int ldy, int parts)
{
    gemv_reg_body<MT, R, STEPS, D, NW, kRagged, NoEpilogue, kBits>(
        RegArgs{x, q, s, out, n, k, m, m0, ldx, ldy, parts}, NoEpilogue{});
}

template <int MT, int R, int STEPS, int D, int NW, bool kRagged, int kBits>
hipError_t launch_one6(const GemmArgs& g, int m0, int blocks, size_t lds, hipStream_t stream)
{
    const bool argmax = g.part_val != nullptr;
    if (MT * STEPS >= 6)
        lds = (size_t)MT * STEPS * 4096 + 64;       // padded activation rows
    if ((kBits & 15) == 6)
        lds += (size_t)NW * R * 1536;               // the waves' buffers for the lane exchange
    static LdsLimit lds_limit;                      // of this kernel instance
    if (lds > 64 * 1024)
        if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(gemv_reg6_kernel<MT, R, STEPS, D, NW, kRagged, kBits>),
                                           160 * 1024);
            e != hipSuccess)
            return e;
    hipLaunchKernelGGL((gemv_reg6_kernel<MT, R, STEPS, D, NW, kRagged, kBits>), dim3(blocks), dim3(NW * 64), lds, stream,
                       g.x, g.q, g.s, argmax ? static_cast<void*>(g.part_val) : static_cast<void*>(g.y), g.n, g.k,
                       g.m, m0, (int)g.ldx, (int)g.ldy, argmax ? g.parts : 0);
    return hipGetLastError();
}

template <int MT, int R, int STEPS, int D, int NW, bool kRagged>
hipError_t launch_one(const GemmArgs& g, int m0, int blocks, size_t lds, hipStream_t stream, const Epilogue* epi)
{
    const bool argmax = g.part_val != nullptr;
    if (MT * STEPS >= 6)
        lds = (size_t)MT * STEPS * 4096 + 64;       // padded activation rows
    static LdsLimit lds_limit, lds_limit_fused;     // of these kernel instances
    if (lds > 64 * 1024) {
        hipError_t e = lds_limit_fused.raise(
            reinterpret_cast<const void*>(gemv_reg_fused_kernel<MT, R, STEPS, D, NW, kRagged>), 160 * 1024);
        if (e == hipSuccess)
            e = lds_limit.raise(reinterpret_cast<const void*>(gemv_reg_kernel<MT, R, STEPS, D, NW, kRagged>), 160 * 1024);
        if (e != hipSuccess)
            return e;
    }
    if (epi)
        hipLaunchKernelGGL((gemv_reg_fused_kernel<MT, R, STEPS, D, NW, kRagged>), dim3(blocks), dim3(NW * 64), lds,
                           stream, g.x, g.q, g.s, static_cast<void*>(g.y), g.n, g.k, g.m, m0, (int)g.ldx,
                           (int)g.ldy, 0, epi->act, epi->bias, epi->residual, epi->ldr);
    else
        hipLaunchKernelGGL((gemv_reg_kernel<MT, R, STEPS, D, NW, kRagged>), dim3(blocks), dim3(NW * 64), lds,
                           stream, g.x, g.q, g.s,
                           argmax ? static_cast<void*>(g.part_val) : static_cast<void*>(g.y), g.n, g.k, g.m, m0,
                           (int)g.ldx, (int)g.ldy, argmax ? g.parts : 0);
    return hipGetLastError();
}

template <int MT>
hipError_t launch_steps(const GemmArgs& a, int m0, int steps2, bool ragged, int blocks, size_t lds,
                        hipStream_t stream, const Epilogue* epi, int nw)
{
    // 16 waves hold at most 128 registers each: enough for four steps of one activation row.
    // From six steps on (K > 8192) the activations stay in the LDS copy: registers are free
    // again, so 16 waves with one weight row per step here too; the instances cover 6, 8, 12, 14
    // and 16 steps and a shorter K leaves the last ones partly or wholly empty.  (Six steps in
    // registers need 8 waves of two rows, three steps in flight: 7.4 us against 6.6 on the 7B
    // down projection.  Two activation rows from LDS were tried too: the compiler spills in
    // every such instance.)
    switch (steps2) {
    case 2:
        // (`nw` is waves_for's answer: 12 waves where a compute unit has at most 40 rows, beyond that two
        // workgroups of 8 per unit, or one of 16 when the call also has passes of two rows)
        if constexpr (MT == 1) {
            if (nw == 8)
                return ragged ? launch_one<MT, 1, 2, 2, 8, true>(a, m0, blocks, lds, stream, epi)
                              : launch_one<MT, 1, 2, 2, 8, false>(a, m0, blocks, lds, stream, epi);
            if (nw == 12)
                return ragged ? launch_one<MT, 1, 2, 2, 12, true>(a, m0, blocks, lds, stream, epi)
                              : launch_one<MT, 1, 2, 2, 12, false>(a, m0, blocks, lds, stream, epi);
            return ragged ? launch_one<MT, 1, 2, 2, 16, true>(a, m0, blocks, lds, stream, epi)
                          : launch_one<MT, 1, 2, 2, 16, false>(a, m0, blocks, lds, stream, epi);
        } else {                                      // two activation rows need more registers: 12 waves (or 8, twice)
            if (nw == 8)
                return ragged ? launch_one<MT, 1, 2, 2, 8, true>(a, m0, blocks, lds, stream, epi)
                              : launch_one<MT, 1, 2, 2, 8, false>(a, m0, blocks, lds, stream, epi);
            return ragged ? launch_one<MT, 1, 2, 2, 12, true>(a, m0, blocks, lds, stream, epi)
                          : launch_one<MT, 1, 2, 2, 12, false>(a, m0, blocks, lds, stream, epi);
        }
    case 4:
        if constexpr (MT == 1)
            return ragged ? launch_one<MT, 1, 4, 2, 12, true>(a, m0, blocks, lds, stream, epi)
                          : launch_one<MT, 1, 4, 2, 12, false>(a, m0, blocks, lds, stream, epi);
        break;
    case 6:
        // 8 waves with three steps in flight (24 KiB per unit): a 7B down projection has one row per wave
        // of the 16-wave form, whose six steps then pass two at a time.  Measured 6.32 against 6.75 us
        // (4096 x 11008), 6.86 / 6.96 (4096 x 12288), 10.31 / 10.56 (8192 x 11008); six in flight, or two
        // rows per step, are slower.  The same choice loses at 4 steps (K = 8192) and at 14 (K = 28672).
        if constexpr (MT == 1)
            return launch_one<MT, 1, 6, 3, 8, true>(a, m0, blocks, lds, stream, epi);
        break;
    case 8:
        if constexpr (MT == 1)
            return launch_one<MT, 1, 8, 2, 16, true>(a, m0, blocks, lds, stream, epi);
        break;
    case 10:
    case 12:
        if constexpr (MT == 1)
            return launch_one<MT, 1, 12, 2, 16, true>(a, m0, blocks, lds, stream, epi);
        break;
    case 14:
        if constexpr (MT == 1)
            return launch_one<MT, 1, 14, 2, 16, true>(a, m0, blocks, lds, stream, epi);
        break;
    case 16:
        if constexpr (MT == 1)
            return launch_one<MT, 1, 16, 2, 16, true>(a, m0, blocks, lds, stream, epi);
        break;
    }
    return hipErrorInvalidValue;
}

// The 6-bit and 8-bit formats: the same instances (all of them ready for a ragged K), no fused form.
template <int MT, int kBits>
hipError_t launch_steps6(const GemmArgs& a, int m0, int steps2, int blocks, size_t lds, hipStream_t stream)
{
    switch (steps2) {
    case 2:
        if constexpr (MT == 1)
            return launch_one6<MT, 1, 2, 2, 12, true, kBits>(a, m0, blocks, lds, stream);
        else
            return launch_one6<MT, 2, 2, 2, 8, true, kBits>(a, m0, blocks, lds, stream);
    case 4:
        if constexpr (MT == 1)
            return launch_one6<MT, 1, 4, 2, 12, true, kBits>(a, m0, blocks, lds, stream);
        break;
    case 6:
        if constexpr (MT == 1)
            return launch_one6<MT, 1, 6, 2, 16, true, kBits>(a, m0, blocks, lds, stream);
        break;
    case 8:
        if constexpr (MT == 1)
            return launch_one6<MT, 1, 8, 2, 16, true, kBits>(a, m0, blocks, lds, stream);
        break;
    case 10:
    case 12:
        if constexpr (MT == 1)
            return launch_one6<MT, 1, 12, 2, 16, true, kBits>(a, m0, blocks, lds, stream);
        break;
    case 14:
        if constexpr (MT == 1)
            return launch_one6<MT, 1, 14, 2, 16, true, kBits>(a, m0, blocks, lds, stream);
        break;
    case 16:
        if constexpr (MT == 1)
            return launch_one6<MT, 1, 16, 2, 16, true, kBits>(a, m0, blocks, lds, stream);
        break;
    }
    return hipErrorInvalidValue;
}

// ---- several independent products in one launch ----------------------------------------------
//
// One token, MXFP4 weights, the same K (up to 8192: activations in registers) and up to kMultiMax
// products that do not read each other's outputs.  The weight rows of all of them form one list
// (product p owns the virtual rows [first, first + n)); the list is dealt exactly as in the single
// product, and a wave that crosses from one product to the next only swaps its buffer descriptors
// and its activation registers: every product's activation row is staged in LDS when the kernel
// starts, so there is no barrier, no refill of the load pipeline and no launch between products.
// The outputs a wave holds (one per lane, each with its own address) are written when 64 have
// gathered or the list ends, not at the crossing: a store drains the wave's loads in flight.
struct MultiProb {
    const uint16_t* x;
    const uint8_t* q;
    const uint8_t* s;
    void* out;           // y (BF16 [N]), or the partial winners (float [parts], int32 [parts])
    int n, first, parts, k;
};
struct MultiArgs {
    int count, k, total, pad;
    MultiProb p[kMultiMax];      // unused entries: x of entry 0 (it is loaded), n = 0, first = total
};

template <int STEPS, bool kRagged>
__global__ __launch_bounds__(1024) void gemv_multi_kernel(const MultiArgs a)
{
    constexpr int NW = 16, D = 2, T = NW * 64;
    static_assert(STEPS % D == 0 && STEPS * 256 <= T, "one 16-byte activation chunk per thread and product");
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int nblk = a.k >> 5, chunks = a.k >> 3, q_row_bytes = nblk * 16;

    u32x4_t xl[kMultiMax];
#pragma unroll
    for (int p = 0; p < kMultiMax; ++p)
        xl[p] = reinterpret_cast<const u32x4_t*>(a.p[p].x)[min(tid, chunks - 1)];

    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                     // [count][4][nblk] chunks
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int* ctr = reinterpret_cast<int*>(smem + (size_t)a.count * a.k * 2);
    float* wv = reinterpret_cast<float*>(ctr + 16);                      // the waves' argmax winners
    int* wi = reinterpret_cast<int*>(wv + NW);
    const int G = gridDim.x, b = blockIdx.x;
    auto row_of = [&](int i) { return i * G + b; };
    if (tid == 0)
        *ctr = NW;

    struct Set {
        __amdgpu_buffer_rsrc_t rq, rs;
        void* out;
        int first, n, parts, idx;
    };
    // the product that owns virtual row v, looking from product `from` on (v only ever grows)
    auto set_for = [&](int v, int from) {
        int idx = from;
        while (idx < a.count - 1 && v >= a.p[idx].first + a.p[idx].n)
            ++idx;
        const MultiProb& pr = a.p[idx];
        Set st;
        st.rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(pr.q), 0, pr.n * q_row_bytes, 0x00020000);
        st.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(pr.s), 0, pr.n * nblk, 0x00020000);
        st.out = pr.out;
        st.first = pr.first;
        st.n = pr.n;
        st.parts = pr.parts;
        st.idx = idx;
        return st;
    };

    u32x4_t bq[D];
    uint32_t bs[D];
    // as in the single product: a step always issues the same loads; past the end of the list (or
    // of a ragged K) the lane offset leaves the descriptor's range and the load returns zero
    auto issue = [&](const Set& st, int v, int t, int d) {
        const bool live = v < a.total;
        const bool vb = !kRagged || t * 64 + lane < nblk;
        const int row = live ? v - st.first : 0;
        bq[d] = __builtin_amdgcn_raw_buffer_load_b128(st.rq, (live && vb) ? lane * 16 : 0x7FFFFFF0,
                                                      row * q_row_bytes + t * 1024, 2);
        bs[d] = __builtin_amdgcn_raw_buffer_load_b32(st.rs, live ? row * nblk + (lane & 15) * 4 : 0x7FFFFFF0, t * 64,
                                                     0);
    };
    int grp = row_of(wave);
    Set cur = set_for(grp, 0);
#pragma unroll
    for (int d = 0; d < D; ++d)
        issue(cur, grp, d, d);

    {
        const int c = min(tid, chunks - 1);                 // clamped duplicates rewrite the same data
#pragma unroll
        for (int p = 0; p < kMultiMax; ++p)
            if (p < a.count)
                xs[(p * 4 + (c & 3)) * nblk + (c >> 2)] = xl[p];
    }
    lds_barrier();

    u32x4_t xr[STEPS][4];
    auto load_x = [&](int idx) {
#pragma unroll
        for (int t = 0; t < STEPS; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xr[t][j] = (!kRagged || t * 64 + lane < nblk) ? xs[(idx * 4 + j) * nblk + t * 64 + lane]
                                                              : u32x4_t{0, 0, 0, 0};
    };
    load_x(cur.idx);

    float best_val = -INFINITY;         // at most one product of a launch takes the argmax form
    int best_idx = 0x7FFFFFFF;
    float res = 0.f, acc = 0.f;
    uint16_t* dst = nullptr;            // where the output held by this lane goes (any product's y)
    int slots = 0;
    auto flush = [&]() {
        if (lane < slots)
            *dst = f32_to_bf16_rne(res);
        slots = 0;
        drain_vmem();                   // stores and loads share a counter: the loop sees only loads
    };
    auto fetch = [&]() {
        int v = 0;
        if (lane == 0)
            v = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return __builtin_amdgcn_readfirstlane(v);
    };

    const int sh_top = (3 - (lane & 3)) * 8;
    int i_next = fetch();
    while (grp < a.total) {
        const int grp_n = row_of(i_next);
        const int i_next2 = fetch();
        Set nxt = cur;
        if (grp_n < a.total && grp_n >= cur.first + cur.n)
            nxt = set_for(grp_n, cur.idx);
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            const int d = t % D;
            const uint32_t dw = (uint32_t)__builtin_amdgcn_ds_bpermute((lane >> 2) * 4, (int)bs[d]);
            float sc = __uint_as_float((dw << sh_top) >> 1);
            if (kRagged)
                sc = (t * 64 + lane < nblk) ? sc : 1.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t qd = bq[d][j];
                const bf16x2_t w0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 0);
                const bf16x2_t w1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 1);
                const bf16x2_t w2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 2);
                const bf16x2_t w3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 3);
                const uint32_t x0 = xr[t][j][0], x1 = xr[t][j][1], x2 = xr[t][j][2], x3 = xr[t][j][3];
                acc = __builtin_amdgcn_fdot2_f32_bf16(w0, __builtin_bit_cast(bf16x2_t, x0), acc, false);
                acc = __builtin_amdgcn_fdot2_f32_bf16(w1, __builtin_bit_cast(bf16x2_t, x1), acc, false);
                acc = __builtin_amdgcn_fdot2_f32_bf16(w2, __builtin_bit_cast(bf16x2_t, x2), acc, false);
                acc = __builtin_amdgcn_fdot2_f32_bf16(w3, __builtin_bit_cast(bf16x2_t, x3), acc, false);
            }
            const int tn = t + D;
            if (tn < STEPS)
                issue(cur, grp, tn, d);
            else
                issue(nxt, grp_n, tn - STEPS, d);
        }
        const float v = wave_sum(acc);
        acc = 0.f;
        const int row = grp - cur.first;
        if (cur.parts > 0) {
            if (v > best_val || (v == best_val && row < best_idx)) {
                best_val = v;
                best_idx = row;
            }
        } else {
            res = (lane == slots) ? v : res;
            dst = (lane == slots) ? static_cast<uint16_t*>(cur.out) + row : dst;
            if (++slots == 64)
                flush();
        }
        if (nxt.idx != cur.idx) {                           // the next row belongs to another product
            cur = nxt;
            load_x(cur.idx);
        }
        grp = grp_n;
        i_next = i_next2;
    }
    if (slots > 0)
        flush();

    // the argmax product, if there is one: combine the waves, publish the workgroup's winner
    int am = -1;
#pragma unroll
    for (int p = 0; p < kMultiMax; ++p)
        am = (p < a.count && a.p[p].parts > 0) ? p : am;
    if (am >= 0) {
        if (lane == 0) {
            wv[wave] = best_val;
            wi[wave] = best_idx;
        }
        __syncthreads();
        if (tid == 0) {
            float bv = wv[0];
            int bi = wi[0];
            for (int w = 1; w < NW; ++w)
                if (wv[w] > bv || (wv[w] == bv && wi[w] < bi)) {
                    bv = wv[w];
                    bi = wi[w];
                }
            float* part_val = static_cast<float*>(a.p[am].out);
            int32_t* part_idx = reinterpret_cast<int32_t*>(part_val + a.p[am].parts);
            part_val[b] = bv;
            part_idx[b] = bi;
        }
    }
}

template <int STEPS, bool kRagged>
hipError_t launch_multi_one(const MultiArgs& ma, int blocks, size_t lds, hipStream_t stream)
{
    static LdsLimit lds_limit;                      // of this kernel instance
    if (lds > 64 * 1024)
        if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(gemv_multi_kernel<STEPS, kRagged>), 160 * 1024);
            e != hipSuccess)
            return e;
    hipLaunchKernelGGL((gemv_multi_kernel<STEPS, kRagged>), dim3(blocks), dim3(1024), lds, stream, ma);
    return hipGetLastError();
}

// The same for products of different K (each up to 32768): the activation rows stay in LDS, padded
// with zeros to a whole (even) number of steps as in the single product's long-K form, and a step
// reads its 64 bytes per lane from there; the step count of a row is the product's own.
__global__ __launch_bounds__(1024) void gemv_multi_lds_kernel(const MultiArgs a)
{
    constexpr int NW = 16, D = 2, T = NW * 64;
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    auto steps_of = [](int k) { return ((((k >> 5) + 63) >> 6) + 1) & ~1; };

    // every product's first 1024 chunks of 16 bytes go out before anything else
    u32x4_t xl[kMultiMax];
#pragma unroll
    for (int p = 0; p < kMultiMax; ++p)
        xl[p] = reinterpret_cast<const u32x4_t*>(a.p[p].x)[min(tid, (a.p[p].k >> 3) - 1)];

    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);         // per product [4][steps * 64] chunks
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int x_chunks = 0;
#pragma unroll
    for (int p = 0; p < kMultiMax; ++p)
        x_chunks += p < a.count ? steps_of(a.p[p].k) * 256 : 0;
    int* ctr = reinterpret_cast<int*>(xs + x_chunks);
    float* wv = reinterpret_cast<float*>(ctr + 16);
    int* wi = reinterpret_cast<int*>(wv + NW);
    const int G = gridDim.x, b = blockIdx.x;
    auto row_of = [&](int i) { return i * G + b; };
    if (tid == 0)
        *ctr = NW;

    struct Set {
        __amdgpu_buffer_rsrc_t rq, rs;
        void* out;
        int first, n, parts, idx, nblk, steps, xoff;
        int fill[3];    // the struct without padding: copying it then moves registers only
    };
    auto set_for = [&](Set& st, int v, int from, int from_xoff) __attribute__((always_inline)) {
        int idx = from, xoff = from_xoff;
        while (idx < a.count - 1 && v >= a.p[idx].first + a.p[idx].n) {
            xoff += steps_of(a.p[idx].k) * 256;
            ++idx;
        }
        const MultiProb& pr = a.p[idx];
        st.nblk = pr.k >> 5;
        st.steps = steps_of(pr.k);
        st.xoff = xoff;
        st.rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(pr.q), 0, pr.n * st.nblk * 16, 0x00020000);
        st.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(pr.s), 0, pr.n * st.nblk, 0x00020000);
        st.out = pr.out;
        st.first = pr.first;
        st.n = pr.n;
        st.parts = pr.parts;
        st.idx = idx;
        st.fill[0] = st.fill[1] = st.fill[2] = 0;
    };

    u32x4_t bq[D];
    uint32_t bs[D];
    auto issue = [&](const Set& st, int v, int t, int d) {
        const bool live = v < a.total;
        const bool vb = t * 64 + lane < st.nblk;
        const int row = live ? v - st.first : 0;
        bq[d] = __builtin_amdgcn_raw_buffer_load_b128(st.rq, (live && vb) ? lane * 16 : 0x7FFFFFF0,
                                                      row * (st.nblk * 16) + t * 1024, 2);
        bs[d] = __builtin_amdgcn_raw_buffer_load_b32(st.rs, live ? row * st.nblk + (lane & 15) * 4 : 0x7FFFFFF0, t * 64,
                                                     0);
    };
    int grp = row_of(wave);
    Set cur;
    set_for(cur, grp, 0, 0);
#pragma unroll
    for (int d = 0; d < D; ++d)
        issue(cur, grp, d, d);

    // stage the activation rows: chunk c of a row goes to [c % 4][c / 4]; zeros behind the row's end
    {
        int xoff = 0;
#pragma unroll
        for (int p = 0; p < kMultiMax; ++p) {
            if (p < a.count) {
                const int chunks = a.p[p].k >> 3, nblk = a.p[p].k >> 5, row = steps_of(a.p[p].k) * 64;
                if (tid < chunks)
                    xs[xoff + (tid & 3) * row + (tid >> 2)] = xl[p];
                const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.p[p].x);
                for (int c = tid + T; c < chunks; c += T)        // K > 8192 only
                    xs[xoff + (c & 3) * row + (c >> 2)] = xp[c];
                const int pad = row - nblk;
                for (int e = tid; e < 4 * pad; e += T)
                    xs[xoff + (e / pad) * row + nblk + e % pad] = u32x4_t{0, 0, 0, 0};
                xoff += 4 * row;
            }
        }
    }
    lds_barrier();

    float best_val = -INFINITY;
    int best_idx = 0x7FFFFFFF;
    float res = 0.f, acc = 0.f;
    uint16_t* dst = nullptr;
    int slots = 0;
    auto flush = [&]() {
        if (lane < slots)
            *dst = f32_to_bf16_rne(res);
        slots = 0;
        drain_vmem();
    };
    auto fetch = [&]() {
        int v = 0;
        if (lane == 0)
            v = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return __builtin_amdgcn_readfirstlane(v);
    };

    const int sh_top = (3 - (lane & 3)) * 8;
    int i_next = fetch();
    while (grp < a.total) {
        const int grp_n = row_of(i_next);
        const int i_next2 = fetch();
        Set nxt = cur;
        if (grp_n < a.total && grp_n >= cur.first + cur.n)
            set_for(nxt, grp_n, cur.idx, cur.xoff);
        const u32x4_t* xb = xs + cur.xoff + lane;
        for (int t = 0; t < cur.steps; t += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int tt = t + d;
                __builtin_amdgcn_sched_barrier(0);      // step by step: a step's loads go out when it ends
                const uint32_t dw = (uint32_t)__builtin_amdgcn_ds_bpermute((lane >> 2) * 4, (int)bs[d]);
                float sc = __uint_as_float((dw << sh_top) >> 1);
                sc = (tt * 64 + lane < cur.nblk) ? sc : 1.0f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u32x4_t xv = xb[(j * cur.steps + tt) * 64];
                    const uint32_t qd = bq[d][j];
                    const bf16x2_t w0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 0);
                    const bf16x2_t w1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 1);
                    const bf16x2_t w2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 2);
                    const bf16x2_t w3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 3);
                    const uint32_t x0 = xv[0], x1 = xv[1], x2 = xv[2], x3 = xv[3];
                    acc = __builtin_amdgcn_fdot2_f32_bf16(w0, __builtin_bit_cast(bf16x2_t, x0), acc, false);
                    acc = __builtin_amdgcn_fdot2_f32_bf16(w1, __builtin_bit_cast(bf16x2_t, x1), acc, false);
                    acc = __builtin_amdgcn_fdot2_f32_bf16(w2, __builtin_bit_cast(bf16x2_t, x2), acc, false);
                    acc = __builtin_amdgcn_fdot2_f32_bf16(w3, __builtin_bit_cast(bf16x2_t, x3), acc, false);
                }
                // the step two ahead: of this row, or of the next one (perhaps another product's);
                // chosen with selects, not branches, so that the loads in flight stay countable
                const int tn = tt + D;
                const bool same = tn < cur.steps;
                Set pick;
                pick.rq = same ? cur.rq : nxt.rq;
                pick.rs = same ? cur.rs : nxt.rs;
                pick.first = same ? cur.first : nxt.first;
                pick.nblk = same ? cur.nblk : nxt.nblk;
                issue(pick, same ? grp : grp_n, same ? tn : tn - cur.steps, d);
            }
        }
        const float v = wave_sum(acc);
        acc = 0.f;
        const int row = grp - cur.first;
        if (cur.parts > 0) {
            if (v > best_val || (v == best_val && row < best_idx)) {
                best_val = v;
                best_idx = row;
            }
        } else {
            res = (lane == slots) ? v : res;
            dst = (lane == slots) ? static_cast<uint16_t*>(cur.out) + row : dst;
            if (++slots == 64)
                flush();
        }
        cur = nxt;
        grp = grp_n;
        i_next = i_next2;
    }
    if (slots > 0)
        flush();

    int am = -1;
#pragma unroll
    for (int p = 0; p < kMultiMax; ++p)
        am = (p < a.count && a.p[p].parts > 0) ? p : am;
    if (am >= 0) {
        if (lane == 0) {
            wv[wave] = best_val;
            wi[wave] = best_idx;
        }
        __syncthreads();
        if (tid == 0) {
            float bv = wv[0];
            int bi = wi[0];
            for (int w = 1; w < NW; ++w)
                if (wv[w] > bv || (wv[w] == bv && wi[w] < bi)) {
                    bv = wv[w];
                    bi = wi[w];
                }
            float* part_val = static_cast<float*>(a.p[am].out);
            int32_t* part_idx = reinterpret_cast<int32_t*>(part_val + a.p[am].parts);
            part_val[b] = bv;
            part_idx[b] = bi;
        }
    }
}

int even_steps(int k) { return ((((k >> 5) + 63) >> 6) + 1) & ~1; }
// two activation rows in the 6- and 8-bit forms: two weight rows per wave step, 8 waves
bool wide_group(int steps2, int mt, int bits) { return mt == 2 && steps2 == 2 && bits != 4; }
// Waves per workgroup of the instance that launch_steps picks.  The 4-bit form at one activation row,
// from a sweep of 4 to 16 waves per step count (us per launch, 16 waves -> the choice): two steps
// (K <= 4096) 12 waves while a compute unit has at most 40 rows -- N = 2048: 3.81 -> 3.53, 4096: 4.52 ->
// 3.84, 8192: 5.71 -> 5.52, 10240: 6.21 -> 5.98, but 12288: 7.07 -> 7.20 and no gain beyond; four steps
// (K <= 8192) 12 waves at any N -- 8192 x 8192 8.14 -> 7.65, 10240 x 8192 9.43 -> 9.27, 57344 x 8192
// 39.9 -> 38.9; six steps 8 waves (see launch_steps); from eight steps on 16.
// `alone`: every pass of the call has this many rows (a call of one row, or of exactly two), so no
// other pass has to share the grid.
bool two_workgroups(int steps2, int mt, int bits, int n, int cus, bool alone)
{
    // the same for a call of exactly two rows: 12288 x 4096 7.91 -> 7.64 us, 22016 x 4096 11.17 -> 11.01,
    // 32000 x 4096 14.68 -> 14.37 against one workgroup of 12 waves
    if (alone && bits == 4 && mt == 2 && steps2 == 2 && n > 40 * cus)
        return true;
    // K <= 4096, one row, more than 40 rows per unit: two workgroups of 8 waves per compute unit against
    // one of 16 -- qkv 7.10 -> 6.89 us, gate+up 10.19 -> 9.96, LM head 13.30 -> 13.06 (two of 12: 7.10,
    // 9.92, 13.04; two or three of 6: slower)
    return alone && bits == 4 && mt == 1 && steps2 == 2 && n > 40 * cus;
}
int waves_for(int steps2, int mt, int bits, int n, int cus, bool alone)
{
    if (two_workgroups(steps2, mt, bits, n, cus, alone))
        return 8;
    if (wide_group(steps2, mt, bits))
        return 8;
    // two activation rows, 4-bit: 12 waves of one weight row against the 8 waves of two rows it ran before --
    // 4096 x 4096 4.70 -> 4.31 us, 12288 x 4096 8.16 -> 7.81, 22016 x 4096 11.80 -> 11.13, 32000 x 4096 15.63 -> 14.71
    if (bits == 4 && mt == 2)
        return 12;
    if (bits == 4 && mt == 1) {
        if (steps2 == 2)
            return n <= 40 * cus ? 12 : 16;
        if (steps2 == 4)
            return 12;
        if (steps2 == 6)
            return 8;
    }
    // the 6- and 8-bit forms: 12 waves up to four steps at any N (E5M2 / E3M2, 16 -> 12 waves: 4096 x 4096
    // 5.50 -> 5.24 / 4.85 -> 4.63 us, 22016 x 4096 16.8 -> 16.6 / 13.4 -> 13.3, 8192 x 8192 13.0 -> 12.9 / 10.8 -> 10.6)
    if (bits != 4 && mt == 1 && steps2 <= 4)
        return 12;
    return 16;
}
int rows_per_step(int steps2, int mt, int bits) { return wide_group(steps2, mt, bits) ? 2 : 1; }

}  // namespace

// K % 128 == 0 (dword scale loads), K <= 32768 (16 steps), and enough weight rows to give every
// compute unit a workgroup's worth.  Activation rows go two per pass up to K = 4096 and one per
// pass beyond: more rows than that are better served by the general kernel (one pass for two
// rows at any K) or the MFMA tiles.
bool gemv_reg_can_run(const GemmArgs& a, const DeviceInfo& dev)
{
    if (a.k % 128 != 0 || a.m < 1 || even_steps(a.k) > 16)
        return false;
    if (a.ldx > 0x7FFFFFFF || a.ldy > 0x7FFFFFFF)           // 32-bit leading dimensions in the kernel
        return false;
    if (a.part_val && a.part_idx != reinterpret_cast<int32_t*>(a.part_val + (size_t)a.m * a.parts))
        return false;                                       // the kernel derives the index array's place
    if ((size_t)2 * a.k * 2 + 64 > (size_t)dev.lds_bytes)
        return false;
    return a.n >= dev.cus * 8;
}

// One launch for `count` products of one token: every one must be a shape the single product takes
// in registers (K <= 8192), all with the same K, their activation rows together within the LDS.
// One K of at most four steps: the register form (the rows themselves in LDS); else the padded rows.
static bool multi_in_registers(const GemmArgs* items, int count)
{
    for (int i = 1; i < count; ++i)
        if (items[i].k != items[0].k)
            return false;
    return even_steps(items[0].k) <= 4;
}

static size_t multi_lds_bytes(const GemmArgs* items, int count)
{
    size_t x = 0;
    for (int i = 0; i < count; ++i)
        x += multi_in_registers(items, count) ? (size_t)items[i].k * 2 : (size_t)even_steps(items[i].k) * 4096;
    return x + 64 + 128;
}

bool gemv_multi_can_run(const GemmArgs* items, int count, const DeviceInfo& dev)
{
    if (count < 2 || count > kMultiMax)
        return false;
    int64_t total = 0;
    int argmaxes = 0;
    for (int i = 0; i < count; ++i) {
        const GemmArgs& a = items[i];
        if (a.m != 1 || !gemv_reg_can_run(a, dev))
            return false;
        argmaxes += a.part_val != nullptr;
        total += a.n;
    }
    return argmaxes <= 1 && total < 0x7FFFFFFF - 64 * 1024 && multi_lds_bytes(items, count) <= (size_t)dev.lds_bytes;
}

hipError_t launch_gemv_multi(const GemmArgs* items, int count, const DeviceInfo& dev, int* parts_used,
                             hipStream_t stream)
{
    if (!gemv_multi_can_run(items, count, dev))
        return hipErrorInvalidValue;
    MultiArgs ma{};
    ma.count = count;
    ma.k = items[0].k;
    int first = 0;
    for (int i = 0; i < count; ++i) {
        const GemmArgs& a = items[i];
        const bool argmax = a.part_val != nullptr;
        ma.p[i] = MultiProb{a.x, a.q, a.s, argmax ? static_cast<void*>(a.part_val) : static_cast<void*>(a.y), a.n, first,
                            argmax ? a.parts : 0, a.k};
        first += a.n;
    }
    ma.total = first;
    for (int i = count; i < kMultiMax; ++i)
        ma.p[i] = MultiProb{items[0].x, nullptr, nullptr, nullptr, 0, first, 0, items[0].k};
    const int blocks = min(dev.cus, (first + 15) / 16);     // every product has at least 8 rows per CU
    if (parts_used)
        *parts_used = blocks;
    const int steps2 = even_steps(ma.k);
    const bool ragged = ma.k != steps2 * 2048;
    const size_t lds = multi_lds_bytes(items, count);
    if (!multi_in_registers(items, count)) {
        static LdsLimit lds_limit;                  // of this kernel
        if (lds > 64 * 1024)
            if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(gemv_multi_lds_kernel), 160 * 1024);
                e != hipSuccess)
                return e;
        hipLaunchKernelGGL(gemv_multi_lds_kernel, dim3(blocks), dim3(1024), lds, stream, ma);
        return hipGetLastError();
    }
    if (steps2 == 2)
        return ragged ? launch_multi_one<2, true>(ma, blocks, lds, stream) : launch_multi_one<2, false>(ma, blocks, lds, stream);
    return ragged ? launch_multi_one<4, true>(ma, blocks, lds, stream) : launch_multi_one<4, false>(ma, blocks, lds, stream);
}

bool gemv_reg_single_pass(const GemmArgs& a) { return a.m == 1 || (a.m == 2 && even_steps(a.k) <= 2); }

hipError_t launch_gemv_reg(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream,
                           const Epilogue* epi, int bits)
{
    if (bits != 4 && ((bits != 6 && bits != 8 && bits != 22 && bits != 24 && bits != 2) || epi))
        return hipErrorInvalidValue;
    const int steps2 = even_steps(a.k);
    const bool ragged = a.k != steps2 * 2048;
    // one workgroup per compute unit; the argmax form writes one partial winner per workgroup, so
    // every pass must use the same number of workgroups: the count of the narrowest pass
    const bool pairs = a.m >= 2 && steps2 <= 2;
    // every pass alike: one row per pass (no pairs), or the call is one pass of two rows
    auto alone = [&](int mt) { return mt == 2 ? pairs && a.m == 2 : !pairs; };
    auto blocks_for = [&](int mt) {
        const int r = rows_per_step(steps2, mt, bits), nw = waves_for(steps2, mt, bits, a.n, dev.cus, alone(mt));
        const int n_groups = (a.n + r - 1) / r;
        return min(dev.cus * (two_workgroups(steps2, mt, bits, a.n, dev.cus, alone(mt)) ? 2 : 1), (n_groups + nw - 1) / nw);
    };
    const int blocks = !pairs ? blocks_for(1) : (a.m == 2 ? blocks_for(2) : min(blocks_for(1), blocks_for(2)));
    if (parts_used)
        *parts_used = blocks;
    for (int m0 = 0; m0 < a.m;) {
        hipError_t e;
        if (a.m - m0 >= 2 && steps2 <= 2) {
            e = bits == 6    ? launch_steps6<2, 6>(a, m0, steps2, blocks, (size_t)2 * a.k * 2 + 64, stream)
                : bits == 8  ? launch_steps6<2, 8>(a, m0, steps2, blocks, (size_t)2 * a.k * 2 + 64, stream)
                : bits == 22 ? launch_steps6<2, 22>(a, m0, steps2, blocks, (size_t)2 * a.k * 2 + 64, stream)
                : bits == 24 ? launch_steps6<2, 24>(a, m0, steps2, blocks, (size_t)2 * a.k * 2 + 64, stream)
                : bits == 2  ? launch_steps6<2, 2>(a, m0, steps2, blocks, (size_t)2 * a.k * 2 + 64, stream)
                            : launch_steps<2>(a, m0, steps2, ragged, blocks, (size_t)2 * a.k * 2 + 64, stream, epi,
                                              waves_for(steps2, 2, bits, a.n, dev.cus, alone(2)));
            m0 += 2;
        } else {
            e = bits == 6    ? launch_steps6<1, 6>(a, m0, steps2, blocks, (size_t)a.k * 2 + 64, stream)
                : bits == 8  ? launch_steps6<1, 8>(a, m0, steps2, blocks, (size_t)a.k * 2 + 64, stream)
                : bits == 22 ? launch_steps6<1, 22>(a, m0, steps2, blocks, (size_t)a.k * 2 + 64, stream)
                : bits == 24 ? launch_steps6<1, 24>(a, m0, steps2, blocks, (size_t)a.k * 2 + 64, stream)
                : bits == 2  ? launch_steps6<1, 2>(a, m0, steps2, blocks, (size_t)a.k * 2 + 64, stream)
                            : launch_steps<1>(a, m0, steps2, ragged, blocks, (size_t)a.k * 2 + 64, stream, epi,
                                              waves_for(steps2, 1, bits, a.n, dev.cus, alone(1)));
            m0 += 1;
        }
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

}  // namespace mxfp4
