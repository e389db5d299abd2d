// The MFMA tile product for verification batches whose activation rows fit the LDS whole
// (arXiv 2503.13565, section 4.4: k+1 rows verified in one pass that should cost about one
// decode step; section 3.4.3, Eq. 2 for the arithmetic).  Same mapping as mfma.hip -- a tile is
// 16 weight rows, lane (i = lane % 16, g = lane / 16) loads the 16 bytes of block 4T + g of row i
// per step T, 16 scaled converts feed four v_mfma_f32_16x16x32_bf16 -- with a leaner frame:
//   - the activation loads are the first thing every thread sends (they return first and the
//     LDS copy is done while the weights are still on their way); the copy is cooperative, one
//     16-byte chunk of every row per thread, laid out as [step][j][g][row ^ swizzle] so that both
//     the copy's writes and the loop's 128-bit reads are free of bank conflicts;
//   - a lane loads the 16 scale bytes of its row for an item of four steps directly (the waves of
//     a workgroup use a row's scale line together, so the lines are fully used);
//   - NW = 4 compute waves per workgroup split K in items of four steps, two or three items in
//     flight per wave; one more wave, which never loads, sums the partial tiles, rounds and stores or tracks
//     the argmax; two workgroups per compute unit when the LDS allows, else (on the tile-major
//     copy) one workgroup of NW = 8.
//   - all conditions on the position are arithmetic masks: a branch around a load makes the
//     compiler lose count of the loads in flight and wait for all of them.
// Measured against mfma.hip on the 7B linears: 10 to 15 % faster at 4 rows, 15 to 30 % at 16.
//
// Tile-major weights (kTiled).  From the canonical row-major tensors a wave load covers 16 rows x
// 64 bytes: half cache lines, and the streaming hint hurts because the other half is wanted next.
// A second copy of the weights, made once by tile_repack_kernel, stores what a wave instruction
// loads contiguously: q as [tile][step][lane][16 bytes] (1 KiB per wave load, streaming hint on),
// the scales as [tile][item][row][16 bytes].  10 to 14 % faster; it costs a second copy of the
// weights for a model that is also used for single-row decoding (the GEMV wants rows contiguous).
#include <stdlib.h>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

namespace {

constexpr int kOob = 0x7FFFFFF0;        // lane offset beyond any descriptor: the load returns zero
constexpr int kTileNW = 4;              // compute waves per workgroup (8 in the wide form)

// LDS of a workgroup: activations [items * 4 steps][16 slots][MP] chunks of 16 bytes, then two
// sets of NW partial tiles.
size_t tile_lds_bytes(int k, int mp, int nw = kTileNW)
{
    const int items = (k / 128 + 3) / 4;
    return (size_t)items * 4 * 256 * mp + (size_t)2 * nw * 1024;
}

// MP: activation rows per pass (4, 8 or 16).  Kernel arguments are scalars so that they are
// preloaded into registers when a wave starts.  `out` is y (BF16 [M, N]) or, in the argmax form
// (parts > 0), the partial winners: float [M, parts] followed by int32 [M, parts].
// Epi: NoEpilogue, or Epilogue for the fused form: the epilogue wave adds the bias, applies the
// gate to the row pairs it holds in one lane and adds the residual; it fetches a tile's bias and
// residual before it waits for the compute waves, so the loads cost no time.
// phase_steps > 0: K split in space.  Grid row y takes the steps [y * phase_steps, (y + 1) *
// phase_steps) of K (phase_steps a multiple of four), holds only that part of the activation rows
// in LDS, and writes FP32 partial products to `out` = float [phases][M][N]; a second kernel adds
// them.  For passes whose activation rows do not fit the LDS whole.
// kBits: 4, or 8 for the 8-bit draft format (q = q8 [N, K], one E4M3 byte per element, row-major only):
// a lane's block is then 32 bytes, two loads per step, and MFMA j takes bytes 8 j .. 8 j + 7 of it
// through four v_cvt_scalef32_pk_bf16_fp8; or 6 for the 6-bit draft format (q = q6, 24 bytes per
// block as a bit string, row-major only): 16 + 8 bytes per step and one
// v_cvt_scalef32_pk32_bf16_fp6 for the whole block, whose 16 result registers are the operands of
// the step's four matrix instructions.  Everything else is shared.
typedef __attribute__((ext_vector_type(2))) unsigned int t_u32x2_t;
typedef __attribute__((ext_vector_type(6))) unsigned int t_u32x6_t;
typedef __attribute__((ext_vector_type(16))) unsigned int t_u32x16_t;

template <int MP, int NW, int D, bool kTiled, class Epi, int kFmt = 4>
__device__ __forceinline__ void mfma_tile_body(const uint16_t* __restrict__ x, const uint8_t* __restrict__ q,
                                               const uint8_t* __restrict__ s, void* out, int n, int k, int m,
                                               int m0, int ldx, int ldy, int parts, const Epi& epi,
                                               int phase_steps = 0)
{
    // kFmt: the element width, + 16 for the second element format of that width (22: E3M2, 24: E5M2):
    // the same frame with the other convert instruction
    constexpr bool kAlt = kFmt > 16;
    constexpr int kBits = kAlt ? kFmt - 16 : kFmt;
    static_assert(kBits == 4 || ((kBits == 8 || kBits == 6) && !kTiled), "element width");
    static_assert(!kAlt || kBits != 4, "the 4-bit format has one element format");
    constexpr bool kEpi = !__is_same(Epi, NoEpilogue);
    constexpr int T = (NW + 1) * 64;
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);
    const int tid = threadIdx.x;
    const int steps_all = k >> 7;
    const int t0 = phase_steps > 0 ? (int)blockIdx.y * phase_steps : 0;  // first step of this workgroup
    const int steps = phase_steps > 0 ? min(phase_steps, steps_all - t0) : steps_all;
    const int chunks = steps * 16;                                      // 16-byte chunks per activation row
    // ---- activations first: thread -> chunk kc of every row, XB chunk slots per batch
    constexpr int XB = 16 / MP;
    const int xpr = (chunks + T - 1) / T;                               // chunk slots per thread
    u32x4_t xl[XB][MP];
    auto x_load = [&](int i0) {
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            const int kc = min(tid + (i0 + i) * T, chunks - 1);
#pragma unroll
            for (int mm = 0; mm < MP; ++mm) {
                const int msrc = min(m0 + mm, m - 1);                   // ragged M: repeat the last row
                xl[i][mm] = reinterpret_cast<const u32x4_t*>(x + (int64_t)msrc * ldx)[t0 * 16 + kc];
            }
        }
    };
    x_load(0);

    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int nblk = k >> 5;
    const int q_row_bytes = kBits == 8 ? k : (kBits == 6 ? (k >> 5) * 24 : k >> 1);
    const int n_items = (steps + 3) >> 2;                               // items per tile (of this K range)
    const int n_items_all = (steps_all + 3) >> 2;
    const int ipw = (n_items + NW - 1) / NW;                            // items per wave and tile
    const int n_tiles = (n + 15) >> 4;
    const int G = gridDim.x, b = blockIdx.x;
    f32x4_t* red = reinterpret_cast<f32x4_t*>(smem + (size_t)n_items * 4 * 256 * MP);   // [2][NW][64]
    // (tile-major tensors hold whole tiles and whole items: rows past N and steps past K are there)
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(q), 0, kTiled ? n_tiles * 16 * q_row_bytes : n * q_row_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(s), 0, kTiled ? n_tiles * n_items_all * 256 : n * nblk, 0x00020000);

    struct Item {
        u32x4_t q[kBits == 8 ? 8 : 4];      // 32 elements per step (8-bit: two loads of 16)
        t_u32x2_t qh[kBits == 6 ? 4 : 1];   // 6-bit: bytes 16 .. 23 of the block
        u32x4_t sc;         // the row's 16 scale bytes of the item: dword u = step u, byte g = block 4u + g
    };
    Item buf[D];
    // A wave's items: for each tile of the workgroup, items wave, wave + NW, ... of the tile.
    // Always five loads per item; an item or step that does not exist reads nothing (its lane
    // offset is out of the descriptor's range) and returns zero.
    int ld_tile = b, ld_loc = 0;
    auto issue = [&](Item& it) {
        const int live = (int)(ld_tile < n_tiles);
        const int item = wave + NW * ld_loc;
        const int have = live & (int)(item < n_items) & (int)(wave < NW);
        const int tile = ld_tile * live;
        if constexpr (kTiled) {
            const int vq = lane * 16;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mk = -(have & (int)(item * 4 + u < steps));   // all ones when the step exists
                it.q[u] = __builtin_amdgcn_raw_buffer_load_b128(
                    rq, (vq & mk) | (kOob & ~mk),
                    (((tile * steps_all + t0 + item * 4 + u) * 1024) & mk) | ((u * 16) & ~mk), 2);
            }
            const int mk = -have;
            it.sc = __builtin_amdgcn_raw_buffer_load_b128(rs, ((li * 16) & mk) | (kOob & ~mk),
                                                          ((tile * n_items_all + (t0 >> 2) + item) * 256) & mk, 0);
        } else {
            const int row = min(tile * 16 + li, n - 1);                 // ragged N: repeat the last row
            const int vq = row * q_row_bytes + lg * (kBits == 8 ? 32 : (kBits == 6 ? 24 : 16));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mk = -(have & (int)(item * 4 + u < steps));   // all ones when the step exists
                if constexpr (kBits == 8) {
                    it.q[2 * u] = __builtin_amdgcn_raw_buffer_load_b128(
                        rq, (vq & mk) | (kOob & ~mk), (((t0 + item * 4 + u) * 128) & mk) | ((u * 32) & ~mk), 0);
                    it.q[2 * u + 1] = __builtin_amdgcn_raw_buffer_load_b128(
                        rq, (vq & mk) | (kOob & ~mk), (((t0 + item * 4 + u) * 128 + 16) & mk) | ((u * 32 + 16) & ~mk), 0);
                } else if constexpr (kBits == 6) {
                    it.q[u] = __builtin_amdgcn_raw_buffer_load_b128(
                        rq, (vq & mk) | (kOob & ~mk), (((t0 + item * 4 + u) * 96) & mk) | ((u * 32) & ~mk), 0);
                    it.qh[u] = __builtin_amdgcn_raw_buffer_load_b64(
                        rq, (vq & mk) | (kOob & ~mk), (((t0 + item * 4 + u) * 96 + 16) & mk) | ((u * 32 + 16) & ~mk), 0);
                } else {
                    it.q[u] = __builtin_amdgcn_raw_buffer_load_b128(
                        rq, (vq & mk) | (kOob & ~mk), (((t0 + item * 4 + u) * 64) & mk) | ((u * 16) & ~mk), 0);
                }
            }
            const int mk = -have;
            it.sc = __builtin_amdgcn_raw_buffer_load_b128(rs, ((row * nblk) & mk) | (kOob & ~mk),
                                                          (t0 * 4 + item * 16) & mk, 0);
        }
        const int wrap = (int)(ld_loc + 1 == ipw);
        ld_loc = (ld_loc + 1) * (1 - wrap);
        ld_tile += G * wrap;
    };
    if (wave < NW) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            issue(buf[d]);
            __builtin_amdgcn_sched_barrier(0);                          // keep the buffers' loads in issue order
        }
    }
    // ---- activations -> LDS: chunk kc = 16 T + 4 g + j of row mm goes to slot
    // (16 T + 4 j + g) * MP + (mm ^ (kc % MP)); a wave's 128-bit reads of MFMA j then cover one
    // contiguous run, and the threads of a copy instruction hit different banks
    auto x_store = [&](int i0) {
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            const int kc = tid + (i0 + i) * T;
            if (kc < chunks) {
                const int Tq = kc >> 4, cs = kc & 15, g = cs >> 2, j = cs & 3;
#pragma unroll
                for (int mm = 0; mm < MP; ++mm)
                    xs[(Tq * 16 + 4 * j + g) * MP + (mm ^ (cs & (MP - 1)))] = xl[i][mm];
            }
        }
    };
    x_store(0);
#pragma unroll 1
    for (int i0 = XB; i0 < xpr; i0 += XB) {                             // long K: the rest, batch by batch
        x_load(i0);
        x_store(i0);
    }
    // steps past the end of K inside the last item: zero activations (their weights are zero too)
    for (int e = tid + (steps * 16) * MP; e < n_items * 4 * 16 * MP; e += T)
        xs[e] = u32x4_t{0, 0, 0, 0};
    lds_barrier();

    const bool argmax = parts > 0;
    if (wave == NW) {
        // Epilogue wave: one barrier per tile, like the compute waves; no loads of its own.
        const int m_valid = min(MP, m - m0);
        float best_val = -INFINITY;       // running winner of column li over rows 4 lg + r of all tiles
        int best_idx = 0x7FFFFFFF;
        int done = 0;
        for (int tile = b; tile < n_tiles; tile += G, ++done) {
            const f32x4_t* slot = red + (size_t)(done & 1) * NW * 64;
            float bias_v[4] = {0.f, 0.f, 0.f, 0.f}, res_v[4] = {0.f, 0.f, 0.f, 0.f};
            bool gated = false;
            if constexpr (kEpi) {
                gated = epi.act == MXFP4_ACT_SWIGLU;
                const int row0 = tile * 16 + 4 * lg;
                const int cols = gated ? 2 : 4, col0 = gated ? row0 >> 1 : row0, n_cols = gated ? n >> 1 : n;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (epi.bias && row0 + r < n)
                        bias_v[r] = bf16_bits_to_f32(epi.bias[row0 + r]);
                    if (epi.residual && li < m_valid && r < cols && col0 + r < n_cols)
                        res_v[r] = bf16_bits_to_f32(epi.residual[(int64_t)(m0 + li) * epi.ldr + col0 + r]);
                }
            }
            lds_barrier();                                              // partial tiles of `tile` are in LDS
            f32x4_t sum = slot[lane];
#pragma unroll
            for (int w = 1; w < NW; ++w)
                sum += slot[w * 64 + lane];
            // lane (li, lg) holds rows 4 lg + r of the tile for activation row li
            if constexpr (kEpi) {
                if (li < m_valid) {
                    uint16_t* y = static_cast<uint16_t*>(out) + (int64_t)(m0 + li) * ldy;
                    const int row0 = tile * 16 + 4 * lg;
                    if (gated) {                                        // rows (0, 1) and (2, 3) are (gate, up) pairs
#pragma unroll
                        for (int c = 0; c < 2; ++c)
                            if (row0 + 2 * c < n)
                                y[(row0 >> 1) + c] = f32_to_bf16_rne(
                                    silu_gate(sum[2 * c] + bias_v[2 * c], sum[2 * c + 1] + bias_v[2 * c + 1]) + res_v[c]);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (row0 + r < n)
                                y[row0 + r] = f32_to_bf16_rne(sum[r] + bias_v[r] + res_v[r]);
                    }
                }
                continue;
            }
            if (li < m_valid) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = tile * 16 + 4 * lg + r;
                    if (row < n) {
                        if (phase_steps > 0) {
                            static_cast<float*>(out)[((int64_t)blockIdx.y * m + (m0 + li)) * n + row] = sum[r];
                        } else if (argmax) {
                            if (sum[r] > best_val) {                    // rows ascend: lowest index wins ties
                                best_val = sum[r];
                                best_idx = row;
                            }
                        } else {
                            static_cast<uint16_t*>(out)[(int64_t)(m0 + li) * ldy + row] = f32_to_bf16_rne(sum[r]);
                        }
                    }
                }
            }
        }
        if (argmax && phase_steps == 0) {
            // combine the four lane groups of each column (value desc, index asc), publish one partial
#pragma unroll
            for (int off = 16; off < 64; off <<= 1) {
                const float v = __shfl_xor(best_val, off);
                const int i = __shfl_xor(best_idx, off);
                if (v > best_val || (v == best_val && i < best_idx)) {
                    best_val = v;
                    best_idx = i;
                }
            }
            if (lane < m_valid) {
                float* part_val = static_cast<float*>(out);
                int32_t* part_idx = reinterpret_cast<int32_t*>(part_val + (int64_t)m * parts);
                part_val[(int64_t)(m0 + lane) * parts + b] = best_val;
                part_idx[(int64_t)(m0 + lane) * parts + b] = best_idx;
            }
        }
        return;
    }

    f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};       // two chains: even and odd j
    const int col = li & (MP - 1);
    int c_tile = b, c_loc = 0, done = 0;
    // Positions only grow, so the walk ends when buffer 0 runs dry.  Every trip issues the same
    // loads whether or not the later buffers still had work, so that every path into the loop head
    // carries the same queue of outstanding loads and the counter waits stay exact.
    while (c_tile < n_tiles) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d == 0 || c_tile < n_tiles) {
                const Item& it = buf[d];
                const int item = wave + NW * c_loc;
                const int have = (int)(item < n_items);
                const int item_c = item * have;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int Tq = item_c * 4 + u;
                    // The convert reads the exponent field as E8M0.  A step that does not exist gets
                    // scale 1 (its weights are zero, its activations in LDS are zero or real).
                    const uint32_t mk = (uint32_t)-(have & (int)(Tq < steps));
                    const uint32_t sbyte = (((it.sc[u] >> (8 * lg)) & 0xFFu) & mk) | (0x7Fu & ~mk);
                    const float scl = __uint_as_float(sbyte << 23);
                    u32x4_t xb[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        xb[j] = xs[(Tq * 16 + 4 * j + lg) * MP + (col ^ ((4 * lg + j) & (MP - 1)))];
                    t_u32x16_t w6 = {};
                    if constexpr (kBits == 6) {
                        const u32x4_t lo = it.q[u];
                        const t_u32x2_t hi = it.qh[u];
                        const t_u32x6_t packed = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1]};
                        if constexpr (kAlt)
                            w6 = __builtin_bit_cast(t_u32x16_t, __builtin_amdgcn_cvt_scalef32_pk32_bf16_bf6(packed, scl));
                        else
                            w6 = __builtin_bit_cast(t_u32x16_t, __builtin_amdgcn_cvt_scalef32_pk32_bf16_fp6(packed, scl));
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        u32x4_t w;
                        if constexpr (kBits == 6) {
                            const uint32_t w0 = w6[4 * j], w1 = w6[4 * j + 1], w2 = w6[4 * j + 2], w3 = w6[4 * j + 3];
                            w = u32x4_t{w0, w1, w2, w3};
                        } else if constexpr (kBits == 8) {
                            const uint32_t q0 = it.q[2 * u + (j >> 1)][2 * (j & 1)];
                            const uint32_t q1 = it.q[2 * u + (j >> 1)][2 * (j & 1) + 1];
                            if constexpr (kAlt) {
                                w[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(q0, scl, false));
                                w[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(q0, scl, true));
                                w[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(q1, scl, false));
                                w[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(q1, scl, true));
                            } else {
                                w[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q0, scl, false));
                                w[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q0, scl, true));
                                w[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q1, scl, false));
                                w[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q1, scl, true));
                            }
                        } else {
                            const uint32_t qd = it.q[u][j];
                            w[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 0));
                            w[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 1));
                            w[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 2));
                            w[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 3));
                        }
                        if (j & 1)
                            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w),
                                                                           __builtin_bit_cast(bf16x8_t, xb[j]), acc1, 0, 0, 0);
                        else
                            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w),
                                                                           __builtin_bit_cast(bf16x8_t, xb[j]), acc0, 0, 0, 0);
                    }
                }
                if (c_loc == ipw - 1) {
                    // end of the tile: leave the partial tile for the epilogue wave
                    f32x4_t* slot = red + (size_t)(done & 1) * NW * 64;
                    slot[wave * 64 + lane] = acc0 + acc1;
                    acc0 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    acc1 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    lds_barrier();
                    ++done;
                }
                if (++c_loc == ipw) {
                    c_loc = 0;
                    c_tile += G;
                }
            }
            issue(buf[d]);
        }
    }
}

template <int MP, int NW, int D, bool kTiled>
__global__ __launch_bounds__((NW + 1) * 64) void mfma_tile_kernel(const uint16_t* __restrict__ x,
                                                                  const uint8_t* __restrict__ q,
                                                                  const uint8_t* __restrict__ s, void* out, int n,
                                                                  int k, int m, int m0, int ldx, int ldy, int parts)
{
    mfma_tile_body<MP, NW, D, kTiled>(x, q, s, out, n, k, m, m0, ldx, ldy, parts, NoEpilogue{});
}

template <int MP, int NW, int D, bool kTiled>
__global__ __launch_bounds__((NW + 1) * 64) void mfma_tile_fused_kernel(
    const uint16_t* __restrict__ x, const uint8_t* __restrict__ q, const uint8_t* __restrict__ s, void* out, int n,
    int k, int m, int m0, int ldx, int ldy, int parts, int act, const uint16_t* bias, const uint16_t* residual,
    int ldr)
{
    mfma_tile_body<MP, NW, D, kTiled>(x, q, s, out, n, k, m, m0, ldx, ldy, parts,
                                      Epilogue{bias, residual, ldr, act});
}

// The 8-bit and 6-bit draft formats (row-major q8 / q6), plain and argmax forms.
template <int MP, int NW, int D, int kBits>
__global__ __launch_bounds__((NW + 1) * 64) void mfma_tile8_kernel(const uint16_t* __restrict__ x,
                                                                   const uint8_t* __restrict__ q,
                                                                   const uint8_t* __restrict__ s, void* out, int n,
                                                                   int k, int m, int m0, int ldx, int ldy, int parts)
{
    mfma_tile_body<MP, NW, D, false, NoEpilogue, kBits>(x, q, s, out, n, k, m, m0, ldx, ldy, parts, NoEpilogue{});
}

// K split in space: the last preloaded argument is the number of steps per grid row.
template <int MP, int NW, int D, bool kTiled>
__global__ __launch_bounds__((NW + 1) * 64) void mfma_tile_split_kernel(const uint16_t* __restrict__ x,
                                                                        const uint8_t* __restrict__ q,
                                                                        const uint8_t* __restrict__ s, void* out,
                                                                        int n, int k, int m, int m0, int ldx,
                                                                        int ldy, int parts, int phase_steps)
{
    mfma_tile_body<MP, NW, D, kTiled>(x, q, s, out, n, k, m, m0, ldx, ldy, parts, NoEpilogue{}, phase_steps);
}

// ---- Activation rows that do not fit the LDS whole: K in phases inside the workgroup ----------
// (7B down projection from five rows, K = 28672 at any width.)  The split in space above needs a
// workspace and a second launch that adds the partial products; for the few-tile shapes that have
// this problem (a down projection has N / 16 tiles, about one per compute unit) that launch costs
// a third of the product.  Here a workgroup keeps its tile's accumulators in registers and walks K
// in phases of kPhaseSteps steps; the LDS holds the activation rows of two phases.  One workgroup
// of eight compute waves per unit; a phase is eight items, one per wave.  A wave's share of a
// phase's activation rows (chunk `tid` of each row) travels with the wave's weight item of that
// phase: loaded right in front of it, D phases ahead, so that waiting for it waits for nothing
// younger; it is written to the other LDS buffer at the end of the phase before, and one barrier
// per phase both publishes that buffer and retires the one just read.  The ninth wave, as in the
// kernel above, sums the eight partial tiles of a finished tile and stores them.
constexpr int kPhaseSteps = 32;
constexpr int kPhaseNW = 8;
constexpr size_t phased_lds_bytes(int mp) { return (size_t)2 * kPhaseSteps * 256 * mp + (size_t)2 * kPhaseNW * 1024; }

template <int MP, int D, bool kTiled>
__global__ __launch_bounds__((kPhaseNW + 1) * 64) void mfma_tile_phased_kernel(
    const uint16_t* __restrict__ x, const uint8_t* __restrict__ q, const uint8_t* __restrict__ s,
    uint16_t* __restrict__ y, int n, int k, int m, int m0, int ldx, int ldy)
{
    constexpr int NW = kPhaseNW, P = kPhaseSteps;
    constexpr int kXBuf = P * 16 * MP;                                  // 16-byte chunks of one LDS buffer
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);
    f32x4_t* red = reinterpret_cast<f32x4_t*>(smem + (size_t)2 * kXBuf * 16);   // [2][NW][64]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int steps_all = k >> 7;
    const int n_items_all = (steps_all + 3) >> 2;
    const int phases = (steps_all + P - 1) / P;
    const int nblk = k >> 5;
    const int q_row_bytes = k >> 1;
    const int n_tiles = (n + 15) >> 4;
    const int G = gridDim.x, b = blockIdx.x;
    const int pairs = (n_tiles - b + G - 1) / G * phases;               // (tile, phase) pairs of this workgroup
    const int trips = (pairs + D - 1) / D * D;

    if (wave == NW) {
        // one barrier per phase, like the compute waves; a tile is complete after its last phase
        const int m_valid = min(MP, m - m0);
        lds_barrier();
        int tile = b, ph = 0, done = 0;
        for (int u = 0; u < trips; ++u) {
            lds_barrier();
            if (tile < n_tiles && ph == phases - 1) {
                const f32x4_t* slot = red + (size_t)(done & 1) * NW * 64;
                f32x4_t sum = slot[lane];
#pragma unroll
                for (int w = 1; w < NW; ++w)
                    sum += slot[w * 64 + lane];
                // lane (li, lg) holds rows 4 lg + r of the tile for activation row li
                if (li < m_valid) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int row = tile * 16 + 4 * lg + r;
                        if (row < n)
                            y[(int64_t)(m0 + li) * ldy + row] = f32_to_bf16_rne(sum[r]);
                    }
                }
                ++done;
            }
            if (++ph == phases) {
                ph = 0;
                tile += G;
            }
        }
        return;
    }

    // (tile-major tensors hold whole tiles and whole items: rows past N and steps past K are there)
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(q), 0, kTiled ? n_tiles * 16 * q_row_bytes : n * q_row_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(s), 0, kTiled ? n_tiles * n_items_all * 256 : n * nblk, 0x00020000);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(x), 0, ((m - 1) * ldx + k) * 2, 0x00020000);

    struct Slot {
        u32x4_t xl[MP];     // chunk `tid` of the phase of every activation row of the pass
        u32x4_t q[4];
        u32x4_t sc;
    };
    Slot buf[D];
    // Always MP + 5 loads per pair; what does not exist (a pair past the workgroup's last, a step
    // past K, an item past the last) reads nothing and returns zero.
    int ld_tile = b, ld_ph = 0;
    auto issue = [&](Slot& sl) {
        const int live = (int)(ld_tile < n_tiles);
        const int tile = ld_tile * live;
        {
            const int mk = -(live & (int)(ld_ph * P + (tid >> 4) < steps_all));
            const int at = (ld_ph * (P * 16) + tid) * 16;
#pragma unroll
            for (int mm = 0; mm < MP; ++mm) {
                const int msrc = min(m0 + mm, m - 1);                   // ragged M: repeat the last row
                sl.xl[mm] = __builtin_amdgcn_raw_buffer_load_b128(rx, ((msrc * ldx * 2 + at) & mk) | (kOob & ~mk), 0, 0);
            }
        }
        const int item = ld_ph * (P / 4) + wave;
        const int have = live & (int)(item < n_items_all);
        if constexpr (kTiled) {
            const int vq = lane * 16;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mk = -(have & (int)(item * 4 + u < steps_all));
                sl.q[u] = __builtin_amdgcn_raw_buffer_load_b128(
                    rq, (vq & mk) | (kOob & ~mk), (((tile * steps_all + item * 4 + u) * 1024) & mk) | ((u * 16) & ~mk), 2);
            }
            const int mk = -have;
            sl.sc = __builtin_amdgcn_raw_buffer_load_b128(rs, ((li * 16) & mk) | (kOob & ~mk),
                                                          ((tile * n_items_all + item) * 256) & mk, 0);
        } else {
            const int row = min(tile * 16 + li, n - 1);                 // ragged N: repeat the last row
            const int vq = row * q_row_bytes + lg * 16;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mk = -(have & (int)(item * 4 + u < steps_all));
                sl.q[u] = __builtin_amdgcn_raw_buffer_load_b128(rq, (vq & mk) | (kOob & ~mk),
                                                                (((item * 4 + u) * 64) & mk) | ((u * 16) & ~mk), 0);
            }
            const int mk = -have;
            sl.sc = __builtin_amdgcn_raw_buffer_load_b128(rs, ((row * nblk) & mk) | (kOob & ~mk), (item * 16) & mk, 0);
        }
        const int wrap = (int)(ld_ph + 1 == phases);
        ld_ph = (ld_ph + 1) * (1 - wrap);
        ld_tile += G * wrap;
    };
    // chunk kc = 16 T + 4 g + j of row mm goes to slot (16 T + 4 j + g) * MP + (mm ^ (kc % MP)), as above
    auto x_store = [&](const Slot& sl, u32x4_t* xb) {
        const int Tl = tid >> 4, cs = tid & 15, g = cs >> 2, j = cs & 3;
#pragma unroll
        for (int mm = 0; mm < MP; ++mm)
            xb[(Tl * 16 + 4 * j + g) * MP + (mm ^ (cs & (MP - 1)))] = sl.xl[mm];
    };
#pragma unroll
    for (int d = 0; d < D; ++d) {
        issue(buf[d]);
        __builtin_amdgcn_sched_barrier(0);                              // keep the slots' loads in issue order
    }
    x_store(buf[0], xs);
    lds_barrier();

    f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};       // two chains: even and odd j
    const int col = li & (MP - 1);
    int c_tile = b, c_ph = 0, done = 0;
    for (int u0 = 0; u0 < trips; u0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const Slot& sl = buf[d];
            const u32x4_t* xb_now = xs + (size_t)((u0 + d) & 1) * kXBuf;
            const int item = c_ph * (P / 4) + wave;
            const int have = (int)(c_tile < n_tiles) & (int)(item < n_items_all);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int Tl = wave * 4 + u;
                const uint32_t mk = (uint32_t)-(have & (int)(item * 4 + u < steps_all));
                const uint32_t sbyte = (((sl.sc[u] >> (8 * lg)) & 0xFFu) & mk) | (0x7Fu & ~mk);
                const float scl = __uint_as_float(sbyte << 23);
                u32x4_t xb[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    xb[j] = xb_now[(Tl * 16 + 4 * j + lg) * MP + (col ^ ((4 * lg + j) & (MP - 1)))];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t qd = sl.q[u][j];
                    u32x4_t w;
                    w[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 0));
                    w[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 1));
                    w[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 2));
                    w[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, scl, 3));
                    if (j & 1)
                        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w),
                                                                       __builtin_bit_cast(bf16x8_t, xb[j]), acc1, 0, 0, 0);
                    else
                        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w),
                                                                       __builtin_bit_cast(bf16x8_t, xb[j]), acc0, 0, 0, 0);
                }
            }
            if (c_tile < n_tiles && c_ph == phases - 1) {
                // end of the tile: leave the partial tile for the ninth wave
                f32x4_t* slot = red + (size_t)(done & 1) * NW * 64;
                slot[wave * 64 + lane] = acc0 + acc1;
                acc0 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                acc1 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                ++done;
            }
            if (++c_ph == phases) {
                c_ph = 0;
                c_tile += G;
            }
            // the next phase's activation rows go to the buffer that the phase before this one read
            x_store(buf[(d + 1) % D], xs + (size_t)((u0 + d + 1) & 1) * kXBuf);
            issue(buf[d]);
            lds_barrier();
        }
    }
}

// Make the tile-major copy: one thread per 16 bytes of either output.  q_t unit (tile, T, lane =
// i + 16 g) is block 4T + g of row 16 tile + i; s_t unit (tile, item, i) holds the scale bytes of
// blocks 16 item .. 16 item + 15 of that row.  Rows past N get zero nibbles, blocks past K and rows
// past N the scale byte of 1.0.
__global__ __launch_bounds__(256) void tile_repack_kernel(const u32x4_t* __restrict__ q,
                                                          const uint32_t* __restrict__ s, int n, int k,
                                                          u32x4_t* __restrict__ qt, u32x4_t* __restrict__ st)
{
    const int steps = k >> 7, nblk = k >> 5, n_items = (steps + 3) >> 2, n_tiles = (n + 15) >> 4;
    const int64_t q_units = (int64_t)n_tiles * steps * 64, s_units = (int64_t)n_tiles * n_items * 16;
    for (int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x; o < q_units + s_units; o += (int64_t)gridDim.x * 256) {
        if (o < q_units) {
            const int l = (int)(o & 63), i = l & 15, g = l >> 4;
            const int64_t ts = o >> 6;
            const int T = (int)(ts % steps), tile = (int)(ts / steps);
            const int row = tile * 16 + i;
            qt[o] = row < n ? q[(int64_t)row * nblk + 4 * T + g] : u32x4_t{0, 0, 0, 0};
        } else {
            const int64_t u = o - q_units;
            const int i = (int)(u & 15);
            const int64_t ti = u >> 4;
            const int item = (int)(ti % n_items), tile = (int)(ti / n_items);
            const int row = tile * 16 + i;
            u32x4_t v;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int blk = item * 16 + 4 * d;                      // nblk % 4 == 0: a dword is in or out
                v[d] = (row < n && blk < nblk) ? s[((int64_t)row * nblk + blk) >> 2] : 0x7F7F7F7Fu;
            }
            st[u] = v;
        }
    }
}

template <int MP, int D, bool kTiled, int NW = kTileNW>
hipError_t launch_pass(const GemmArgs& a, int m0, int blocks, size_t lds, const DeviceInfo& dev,
                       hipStream_t stream, const Epilogue* epi)
{
    auto kern = mfma_tile_kernel<MP, NW, D, kTiled>;
    auto kern_fused = mfma_tile_fused_kernel<MP, NW, D, kTiled>;
    static LdsLimit lds_limit, lds_limit_fused;     // of these kernel instances
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), dev.lds_bytes); e != hipSuccess)
        return e;
    if (hipError_t e = lds_limit_fused.raise(reinterpret_cast<const void*>(kern_fused), dev.lds_bytes); e != hipSuccess)
        return e;
    const bool argmax = a.part_val != nullptr;
    if (epi)
        hipLaunchKernelGGL(kern_fused, dim3(blocks), dim3((NW + 1) * 64), lds, stream, a.x, a.q, a.s,
                           static_cast<void*>(a.y), a.n, a.k, a.m, m0, (int)a.ldx, (int)a.ldy, 0, epi->act,
                           epi->bias, epi->residual, epi->ldr);
    else
        hipLaunchKernelGGL(kern, dim3(blocks), dim3((NW + 1) * 64), lds, stream, a.x, a.q, a.s,
                           argmax ? static_cast<void*>(a.part_val) : static_cast<void*>(a.y), a.n, a.k, a.m, m0,
                           (int)a.ldx, (int)a.ldy, argmax ? a.parts : 0);
    return hipGetLastError();
}

template <int MP, int NW, int kBits>
hipError_t launch_pass8(const GemmArgs& a, int m0, int blocks, size_t lds, const DeviceInfo& dev, hipStream_t stream)
{
    auto kern = mfma_tile8_kernel<MP, NW, 2, kBits>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), dev.lds_bytes); e != hipSuccess)
        return e;
    const bool argmax = a.part_val != nullptr;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3((NW + 1) * 64), lds, stream, a.x, a.q, a.s,
                       argmax ? static_cast<void*>(a.part_val) : static_cast<void*>(a.y), a.n, a.k, a.m, m0,
                       (int)a.ldx, (int)a.ldy, argmax ? a.parts : 0);
    return hipGetLastError();
}

int tile_pass_width(int left) { return left > 8 ? 16 : (left > 4 ? 8 : 4); }

}  // namespace

// K % 128 == 0 and the widest pass's activation rows fit the LDS whole; 32-bit leading
// dimensions; in the argmax form the index array directly behind the value array.
bool mfma_tile_can_run(const GemmArgs& a, const DeviceInfo& dev)
{
    if (a.k % 128 != 0 || a.m < 1)
        return false;
    if (a.ldx > 0x7FFFFFFF || a.ldy > 0x7FFFFFFF)
        return false;
    if (a.part_val && a.part_idx != reinterpret_cast<int32_t*>(a.part_val + (size_t)a.m * a.parts))
        return false;
    return tile_lds_bytes(a.k, tile_pass_width(a.m)) <= (size_t)dev.lds_bytes;
}

// The 6- and 8-bit formats have no K split: where the widest pass does not fit the LDS they take
// narrower passes (more of them), so a pass of four rows must fit.
bool mfma_tile_fmt_can_run(const GemmArgs& a, const DeviceInfo& dev)
{
    GemmArgs narrow = a;
    narrow.m = a.m < 4 ? a.m : 4;
    if (a.part_val && a.part_idx != reinterpret_cast<int32_t*>(a.part_val + (size_t)a.m * a.parts))
        return false;
    narrow.part_val = nullptr;
    return mfma_tile_can_run(narrow, dev);
}

size_t tile_repack_q_bytes(int64_t n, int64_t k) { return (size_t)((n + 15) / 16) * 16 * (size_t)(k / 2); }
size_t tile_repack_s_bytes(int64_t n, int64_t k)
{
    return (size_t)((n + 15) / 16) * (size_t)((k / 128 + 3) / 4) * 256;
}

hipError_t launch_tile_repack(const void* q, const void* s, int n, int k, void* qt, void* st, hipStream_t stream)
{
    const size_t units = tile_repack_q_bytes(n, k) / 16 + tile_repack_s_bytes(n, k) / 16;
    const int blocks = (int)((units + 255) / 256 < 8192 ? (units + 255) / 256 : 8192);
    hipLaunchKernelGGL(tile_repack_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const u32x4_t*>(q),
                       static_cast<const uint32_t*>(s), n, k, static_cast<u32x4_t*>(qt), static_cast<u32x4_t*>(st));
    return hipGetLastError();
}

// One pass of `mp` rows from row m0 with K split over `phases` grid rows of `phase_steps` steps;
// partial products go to ws = float [phases][M][N].  One workgroup per compute unit and phase
// (its part of the activation rows fills most of the LDS): four compute waves with three items
// in flight each from the row-major tensors, eight with two from the tile-major copy.
bool mfma_tile_split_fits(int phase_steps, int mp, const DeviceInfo& dev)
{
    return phase_steps % 4 == 0 && tile_lds_bytes(phase_steps * 128, mp) <= (size_t)dev.lds_bytes;
}

template <int MP, int NW, int D, bool kTiled>
hipError_t launch_split_pass(const GemmArgs& a, int m0, int phases, int phase_steps, float* ws, int blocks,
                             size_t lds, const DeviceInfo& dev, hipStream_t stream)
{
    auto kern = mfma_tile_split_kernel<MP, NW, D, kTiled>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), dev.lds_bytes); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3(blocks, phases), dim3((NW + 1) * 64), lds, stream, a.x, a.q, a.s,
                       static_cast<void*>(ws), a.n, a.k, a.m, m0, (int)a.ldx, (int)a.ldy, 0, phase_steps);
    return hipGetLastError();
}

hipError_t launch_mfma_tile_split(const GemmArgs& a, int m0, int mp, int phases, int phase_steps, float* ws,
                                  const DeviceInfo& dev, hipStream_t stream, bool tiled)
{
    if (a.ldx > 0x7FFFFFFF || !mfma_tile_split_fits(phase_steps, mp, dev) || phases < 1)
        return hipErrorInvalidValue;
    const int n_tiles = (a.n + 15) / 16;
    int blocks = dev.cus / phases;
    blocks = blocks < 1 ? 1 : (blocks > n_tiles ? n_tiles : blocks);
    if (tiled && tile_lds_bytes(phase_steps * 128, mp, 8) <= (size_t)dev.lds_bytes) {
        const size_t lds = tile_lds_bytes(phase_steps * 128, mp, 8);
        return mp == 16  ? launch_split_pass<16, 8, 2, true>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream)
               : mp == 8 ? launch_split_pass<8, 8, 2, true>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream)
                         : launch_split_pass<4, 8, 2, true>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream);
    }
    const size_t lds = tile_lds_bytes(phase_steps * 128, mp);
    if (tiled)
        return mp == 16  ? launch_split_pass<16, kTileNW, 3, true>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream)
               : mp == 8 ? launch_split_pass<8, kTileNW, 3, true>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream)
                         : launch_split_pass<4, kTileNW, 3, true>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream);
    return mp == 16  ? launch_split_pass<16, kTileNW, 3, false>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream)
           : mp == 8 ? launch_split_pass<8, kTileNW, 3, false>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream)
                     : launch_split_pass<4, kTileNW, 3, false>(a, m0, phases, phase_steps, ws, blocks, lds, dev, stream);
}

// K in phases inside the workgroup: any K % 128 == 0, no workspace, plain product only.  Passes of
// four or eight rows (more rows take several passes).
bool mfma_tile_phased_can_run(const GemmArgs& a, const DeviceInfo& dev)
{
    if (a.k % 128 != 0 || a.m < 1 || a.part_val != nullptr || a.y == nullptr)
        return false;
    if (a.ldx > 0x7FFFFFFF || a.ldy > 0x7FFFFFFF)
        return false;
    if (((int64_t)(a.m - 1) * a.ldx + a.k) * 2 > 0x7FFFFFF0LL)          // the activation rows behind one 32-bit offset
        return false;
    return phased_lds_bytes(a.m > 4 ? 8 : 4) <= (size_t)dev.lds_bytes;
}

bool mfma_tile_phased_preferred(const GemmArgs& a, const DeviceInfo& dev, bool split_available)
{
    static const int env = [] { const char* e = knob("MXFP4_TILE_PHASED"); return e ? atoi(e) : -1; }();   // measurement only
    if (env == 0 || a.m > 8 || !mfma_tile_phased_can_run(a, dev))
        return false;
    if (!split_available || env == 1)
        return true;
    // Against the split in space (measured at 8 rows, tile-major / row-major): one tile per workgroup
    // 11.3 against 11.7 us / 12.4 against 12.8 (7B down projection); two tiles and seven phases (70B
    // down projection) 34.5 against 27.8 / 42.4 against 34.5, because every tile fetches the rows again.
    return (a.n + 15) / 16 <= dev.cus;
}

template <int MP, int D, bool kTiled>
hipError_t launch_phased_pass(const GemmArgs& a, int m0, int blocks, const DeviceInfo& dev, hipStream_t stream)
{
    auto kern = mfma_tile_phased_kernel<MP, D, kTiled>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), dev.lds_bytes); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3((kPhaseNW + 1) * 64), phased_lds_bytes(MP), stream, a.x, a.q, a.s,
                       a.y, a.n, a.k, a.m, m0, (int)a.ldx, (int)a.ldy);
    return hipGetLastError();
}

hipError_t launch_mfma_tile_phased(const GemmArgs& a, const DeviceInfo& dev, hipStream_t stream, bool tiled)
{
    if (!mfma_tile_phased_can_run(a, dev))
        return hipErrorInvalidValue;
    const int n_tiles = (a.n + 15) / 16;
    const int blocks = n_tiles < dev.cus ? n_tiles : dev.cus;
    for (int m0 = 0; m0 < a.m;) {
        const int mp = a.m - m0 > 4 ? 8 : 4;
        hipError_t e;
        if (mp == 8)
            e = tiled ? launch_phased_pass<8, 2, true>(a, m0, blocks, dev, stream)
                      : launch_phased_pass<8, 2, false>(a, m0, blocks, dev, stream);
        else
            e = tiled ? launch_phased_pass<4, 3, true>(a, m0, blocks, dev, stream)
                      : launch_phased_pass<4, 3, false>(a, m0, blocks, dev, stream);
        if (e != hipSuccess)
            return e;
        m0 += mp;
    }
    return hipSuccess;
}

// The 8-bit (a.q = q8 [N, K]) and 6-bit (a.q = q6) draft formats on the tile kernel; shapes as
// mfma_tile_can_run; two workgroups of four compute waves per compute unit when the LDS allows,
// else one of eight.
template <int kBits>
hipError_t launch_tile_fmt(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    const int n_tiles = (a.n + 15) / 16;
    int cap = 16;                                           // the widest pass whose rows fit the LDS
    while (cap > 4 && tile_lds_bytes(a.k, cap) > (size_t)dev.lds_bytes)
        cap >>= 1;
    auto width = [&](int left) { const int w = tile_pass_width(left); return w < cap ? w : cap; };
    const size_t widest = tile_lds_bytes(a.k, width(a.m));
    static const int env_one = [] { const char* e = knob("MXFP4_TILE_FMT_ONE_WG"); return e ? atoi(e) : -1; }();   // measurement only
    // Two workgroups of four waves per CU only where the tiles are few (fewer than two per wave of the
    // wide form): from there on one workgroup of eight waves measured 4-12 % faster in these formats.
    const bool few = n_tiles < 2 * dev.cus;
    const bool two = (env_one >= 0 ? env_one == 0 : few) && 2 * widest + 2048 <= (size_t)dev.lds_bytes;
    int blocks = dev.cus * (two ? 2 : 1);
    blocks = blocks > n_tiles ? n_tiles : blocks;
    blocks = blocks > gemv_max_parts(dev) ? gemv_max_parts(dev) : blocks;
    if (parts_used)
        *parts_used = blocks;
    for (int m0 = 0; m0 < a.m;) {
        const int mp = width(a.m - m0);
        const bool wide = !two && tile_lds_bytes(a.k, mp, 8) <= (size_t)dev.lds_bytes;
        const size_t lds = tile_lds_bytes(a.k, mp, wide ? 8 : kTileNW);
        hipError_t e;
        if (wide)
            e = mp == 16  ? launch_pass8<16, 8, kBits>(a, m0, blocks, lds, dev, stream)
                : mp == 8 ? launch_pass8<8, 8, kBits>(a, m0, blocks, lds, dev, stream)
                          : launch_pass8<4, 8, kBits>(a, m0, blocks, lds, dev, stream);
        else
            e = mp == 16  ? launch_pass8<16, kTileNW, kBits>(a, m0, blocks, lds, dev, stream)
                : mp == 8 ? launch_pass8<8, kTileNW, kBits>(a, m0, blocks, lds, dev, stream)
                          : launch_pass8<4, kTileNW, kBits>(a, m0, blocks, lds, dev, stream);
        if (e != hipSuccess)
            return e;
        m0 += mp;
    }
    return hipSuccess;
}

hipError_t launch_mfma_tile8(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream, int bits)
{
    return bits == 8    ? launch_tile_fmt<8>(a, dev, parts_used, stream)
           : bits == 6  ? launch_tile_fmt<6>(a, dev, parts_used, stream)
           : bits == 24 ? launch_tile_fmt<24>(a, dev, parts_used, stream)
           : bits == 22 ? launch_tile_fmt<22>(a, dev, parts_used, stream)
                        : hipErrorInvalidValue;
}

hipError_t launch_mfma_tile(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream,
                            bool tiled, const Epilogue* epi)
{
    const int n_tiles = (a.n + 15) / 16;
    // About 48 to 64 KiB of weights in flight per compute unit is where this kernel peaks
    // (measured on the 7B and 70B shapes): up to K = 4096-ish two workgroups per unit, when the
    // widest pass leaves room for them, with two items in flight per wave; from K = 8192 on, where
    // a wave has four and more items per tile, one workgroup with three.
    const size_t widest = tile_lds_bytes(a.k, tile_pass_width(a.m));
    const bool long_k = a.k >= 8192;
    int per_cu = !long_k && 2 * widest + 2048 <= (size_t)dev.lds_bytes ? 2 : 1;
    // three items in flight also for 16-row passes over many tiles (7B gate+up and LM head: 5 %)
    bool deep = long_k || (tile_pass_width(a.m) == 16 && n_tiles >= 4 * dev.cus);
    // MXFP4_TILE_WGS (1 to 4), MXFP4_TILE_D (2, 3) and MXFP4_TILE_NW (4, 8): measurement only
    static const int env_wgs = [] { const char* e = knob("MXFP4_TILE_WGS"); return e ? atoi(e) : 0; }();
    static const int env_d = [] { const char* e = knob("MXFP4_TILE_D"); return e ? atoi(e) : 0; }();
    if (env_wgs >= 1 && env_wgs <= 4 && env_wgs * widest + 2048 <= (size_t)dev.lds_bytes)
        per_cu = env_wgs;
    if (env_d == 2 || env_d == 3)
        deep = env_d == 3;
    static const int env_nw = [] { const char* e = knob("MXFP4_TILE_NW"); return e ? atoi(e) : 0; }();
    int blocks = dev.cus * per_cu;
    if (blocks > n_tiles)
        blocks = n_tiles;
    if (blocks > gemv_max_parts(dev))
        blocks = gemv_max_parts(dev);
    if (parts_used)
        *parts_used = blocks;                   // every pass uses the same grid: the partials line up
    for (int m0 = 0; m0 < a.m;) {
        const int mp = tile_pass_width(a.m - m0);
        // Wide form, eight compute waves with two items in flight each: with one workgroup per
        // compute unit four waves sit alone on their SIMDs and nothing hides a wave's LDS and
        // matrix-instruction latencies.  On the tile-major copy that is worth 3 to 18 % (7B at 16
        // rows, 7B down projection at 4, the 70B shapes at 4 and 8); from the row-major tensors the
        // half-line loads set the pace and it gains nothing.
        bool wide = per_cu == 1 && tiled;
        if (env_nw == 4 || env_nw == 8)
            wide = env_nw == 8 && per_cu == 1;
        wide = wide && tile_lds_bytes(a.k, mp, 8) <= (size_t)dev.lds_bytes;
        const size_t lds = tile_lds_bytes(a.k, mp, wide ? 8 : kTileNW);
        const bool deep_pass = env_d == 2 || env_d == 3 ? deep : deep && !wide;
        hipError_t e;
#define MXFP4_TILE_CASE(D_, T_, NW_)                                                        \
    (mp == 16  ? launch_pass<16, D_, T_, NW_>(a, m0, blocks, lds, dev, stream, epi)              \
     : mp == 8 ? launch_pass<8, D_, T_, NW_>(a, m0, blocks, lds, dev, stream, epi)               \
               : launch_pass<4, D_, T_, NW_>(a, m0, blocks, lds, dev, stream, epi))
        if (wide) {
            if (tiled)
                e = deep_pass ? MXFP4_TILE_CASE(3, true, 8) : MXFP4_TILE_CASE(2, true, 8);
            else
                e = deep_pass ? MXFP4_TILE_CASE(3, false, 8) : MXFP4_TILE_CASE(2, false, 8);
        } else if (tiled) {
            e = deep_pass ? MXFP4_TILE_CASE(3, true, kTileNW) : MXFP4_TILE_CASE(2, true, kTileNW);
        } else {
            e = deep_pass ? MXFP4_TILE_CASE(3, false, kTileNW) : MXFP4_TILE_CASE(2, false, kTileNW);
        }
#undef MXFP4_TILE_CASE
        if (e != hipSuccess)
            return e;
        m0 += mp;
    }
    return hipSuccess;
}

}  // namespace mxfp4
