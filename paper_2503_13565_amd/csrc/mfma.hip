// Skinny product y = x * dequant(W)^T on the matrix cores of gfx950, for verification batches
// (arXiv 2503.13565, section 4.4: k+1 rows are verified in one pass and the pass has to cost
// about as much as one decode step; section 3.4.3, Eq. 2 for the arithmetic).
//
// Why matrix cores for so few rows: on the vector ALUs every extra activation row costs half an
// instruction per weight, which exhausts the ALU budget of a memory-speed kernel at 3 to 4 rows.
// Here a weight costs half a vector instruction (the scaled FP4->BF16 convert) whatever the
// number of rows, and v_mfma_f32_16x16x32_bf16 does the multiply-adds for up to 16 rows at once.
// K = 32 of the instruction is one MX scale block per lane group.
//
// Mapping.  A tile is 16 weight rows.  Lane (i = lane % 16, g = lane / 16) loads, per step T,
// the 16 bytes of block 4T + g of row i: 32 weights that feed four MFMAs (dword j = the lane's
// 8 k-slots of MFMA j) after 16 converts; the block's scale goes into the converts.  The
// activation operand of MFMA j for lane (col = lane % 16, g) is x[col][32 (4T + g) + 8 j .. + 8],
// one 128-bit LDS read.  NW compute waves of a workgroup split K; each copies the activations of
// its own K slice into LDS once, as [T][j][g][MP] chunks of 8 elements so that one wave read
// covers one contiguous run, accumulates a 16 x 16 FP32 tile over its slice and leaves it in LDS;
// one more wave, which never loads, sums the partial tiles in a fixed order, rounds and stores
// (or tracks the argmax), so that the compute waves only ever have loads in flight and their load
// counter stays exact.  Workgroups are persistent over tiles; loads run one item (4 steps) ahead
// in a second register buffer.  When M * K outgrows the LDS, K is also cut into phases across
// workgroups (grid dimension y) whose FP32 partial products meet in a workspace.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

namespace {

constexpr int kCh = 4;             // steps (16-byte loads per lane) per pipeline item

// Bytes of the activation copy of a workgroup whose K range is `steps` steps: every one of the NW
// compute waves owns a slice of whole items.
template <int NW>
__host__ __device__ constexpr size_t x_lds_bytes(int steps, int mp)
{
    return (size_t)(((steps + kCh - 1) / kCh + NW - 1) / NW) * NW * kCh * 256 * mp;
}

// Dwords per row of a tile's scale block in LDS: one per step, rounded so that the 16 bytes of an
// item are aligned and, beyond the last wave's slice, readable; plus a skew against bank conflicts.
template <int NW>
__host__ __device__ constexpr int scale_row_dwords_t(int steps)
{
    return ((steps + kCh - 1) / kCh + NW - 1) / NW * NW * kCh + 4;
}
constexpr int kSentinel = 0x7FFFFFF0;   // lane offset beyond any descriptor: the load returns zero

__device__ __forceinline__ void lds_barrier_mfma()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

struct MItem {
    u32x4_t q[kCh];     // 32 nibbles per step
    uint32_t sp;        // this lane's dword of the scale block of the workgroup's NEXT tile
};

struct MPos {
    int tile;
    int c;          // item within the tile
    int ph;         // phase of the in-time K split this workgroup is in (0 when there is none)
};

// MP: activation rows held per pass (4, 8 or 16); NW: compute waves per workgroup (they split K);
// the workgroup has NW + 1 waves, wave 0 is the epilogue wave; D: register buffers.
//
// K split.  When MP rows of all of K do not fit the LDS, K is cut into a.phases runs of
// a.phase_steps steps.  In time (a.splitk_ws == NULL): the workgroup walks the phases one after
// the other over all its tiles; every compute wave re-copies its activation slice when it enters
// a phase, and the epilogue wave keeps each tile's running FP32 sum in LDS until the last phase.
// In space (a.splitk_ws != NULL): grid dimension y is the phase and the partial products go to
// the workspace (for matrices with too many tiles per workgroup to keep their sums in LDS).
// kEpi: the fused form (bias, gate on the row pairs a lane holds, residual; `epi` is not read
// otherwise).
template <int MP, int NW, int D, bool kEpi>
__global__ __launch_bounds__((NW + 1) * 64) void mfma_kernel(GemmArgs a, int m0, Epilogue epi)
{
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                          // [NW][steps_w][4][4][MP] chunks of 8 elements
    f32x4_t* red = reinterpret_cast<f32x4_t*>(smem + x_lds_bytes<NW>(a.phase_steps, MP));   // [2][NW][64] partial tiles
    const int scw = scale_row_dwords_t<NW>(a.phase_steps);
    uint32_t* sc = reinterpret_cast<uint32_t*>(red + 2 * NW * 64);           // [2][16][scw] scale blocks
    f32x4_t* accl = reinterpret_cast<f32x4_t*>(sc + 2 * 16 * scw);           // [tiles of this workgroup][64] running sums
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave - 1;                                      // K slice of a compute wave
    const int li = lane & 15, lg = lane >> 4;
    const int nblk = a.k >> 5;
    const int q_row_bytes = a.k >> 1;
    const int steps_all = a.k >> 7;                               // steps of 4 blocks in all of K
    const bool in_space = a.splitk_ws != nullptr;
    const int n_ph = in_space ? 1 : a.phases;                     // phases this workgroup walks
    __builtin_assume(n_ph >= 1);
    const int ph0 = in_space ? (int)blockIdx.y : 0;
    auto t_begin_of = [&](int ph) { return (ph0 + ph) * a.phase_steps; };
    auto t_total_of = [&](int ph) { return min(steps_all - (ph0 + ph) * a.phase_steps, a.phase_steps); };
    // steps per wave and tile, in whole items of kCh steps (the same in every phase; a shorter last
    // phase leaves steps absent)
    const int items = ((a.phase_steps + kCh - 1) / kCh + NW - 1) / NW;
    const int steps_w = items * kCh;
    const int n_tiles = (a.n + 15) >> 4;
    const bool argmax = a.part_val != nullptr;
    const int m_valid = min(MP, a.m - m0);

    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.q), 0, a.n * q_row_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.s), 0, a.n * nblk, 0x00020000);

    // Activations.  A compute wave only ever multiplies with the K slice it owns, so it copies
    // just that slice into its own region of the LDS: no wave waits for another's copy and no
    // barrier is needed.  Per item (64 chunks of 8 elements, one per lane) the MP rows' loads are
    // all in flight together.  Chunk 4 g + j of step u goes to slot 16 u + 4 j + g: the four lane
    // groups of one MFMA then read four adjacent segments, 1 KiB contiguous per wave read at
    // MP = 16, free of bank conflicts.  Rows past M repeat the last; steps past the end of the
    // phase copy its last step (their weights are zero).
    u32x4_t* xw = xs + (size_t)max(kw, 0) * steps_w * 16 * MP;
    constexpr int kXLoads = MP > 8 ? MP : 8;                      // loads in flight per batch
    constexpr int kXBatch = kXLoads / MP;
    u32x4_t xv[kXLoads];
    auto x_load = [&](int c0, int ph) {
#pragma unroll
        for (int i = 0; i < kXBatch; ++i) {
            const int c = min(c0 + i, items - 1);                 // a batch's surplus repeats the last item
            const int t = min(kw * steps_w + c * kCh + (lane >> 4), t_total_of(ph) - 1);
            const int chunk = (t_begin_of(ph) + t) * 16 + (lane & 15);
#pragma unroll
            for (int m = 0; m < MP; ++m) {
                const int msrc = min(m0 + m, a.m - 1);
                xv[i * MP + m] = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx)[chunk];
            }
        }
    };
    auto x_store = [&](int c0) {
        const int sl = (lane & 48) | ((lane & 3) << 2) | ((lane >> 2) & 3);
#pragma unroll
        for (int i = 0; i < kXBatch; ++i) {
            const int c = min(c0 + i, items - 1);
#pragma unroll
            for (int m = 0; m < MP; ++m)
                xw[(c * 64 + sl) * MP + m] = xv[i * MP + m];
        }
    };

    // The walk: phase by phase, within a phase this workgroup's tiles in ascending order, within
    // a tile this wave's items.
    auto valid = [&](const MPos& p) { return p.ph < n_ph; };
    // (selects and bitwise conditions rather than branches and short-circuits throughout the walk:
    // once the compiler turns a condition on the position into control flow around the loads it
    // can no longer count the loads in flight)
    auto next_tile = [&](int* tile, int* ph) {
        const int t = *tile + (int)gridDim.x;
        const bool wrap = t >= n_tiles;
        *tile = wrap ? (int)blockIdx.x : t;
        *ph += wrap ? 1 : 0;
    };
    auto advance = [&](MPos& p) {
        const bool last = p.c + 1 == items;
        int tile = p.tile, ph = p.ph;
        next_tile(&tile, &ph);
        p.c = last ? 0 : p.c + 1;
        p.tile = last ? tile : p.tile;
        p.ph = last ? ph : p.ph;
    };
    // Step T (relative to its phase) of this wave for slot u of item c, and whether it exists.
    auto step_of = [&](const MPos& p, int u, bool* ok) {
        const int t = kw * steps_w + p.c * kCh + u;
        *ok = (int)valid(p) & (int)(t < t_total_of(p.ph));
        return t;
    };
    // Scales.  A tile's scale block is 16 rows x t_total dwords (a dword holds the four scales of one
    // step).  A lane needs 16 bytes of ONE row per item, which as a load touches 16 cache lines per
    // wave for 256 useful bytes and fills the L1 with lines it uses an eighth of.  Instead the
    // workgroup's waves fetch the block of the NEXT tile of the walk together, one dword per lane
    // and item in row-major order (256 contiguous bytes per wave load), park it in LDS, and every
    // wave reads the 16 bytes it needs from there after the barrier that ends the tile.
    // Dword d = (c * NW + kw) * 64 + lane of the block: its row and step, false past the block.
    // (d / t_total by multiplication: exact for d < 2^14 and t_total <= 2^9, which K <= 65536 keeps;
    // t_total is a.phase_steps except in the last phase of K)
    const int tt_last = steps_all - (a.phases - 1) * a.phase_steps;
    const uint32_t magic_full = __builtin_amdgcn_readfirstlane((1u << 24) / (uint32_t)min(a.phase_steps, steps_all) + 1u);
    const uint32_t magic_last = __builtin_amdgcn_readfirstlane((1u << 24) / (uint32_t)tt_last + 1u);
    auto sp_place = [&](int c, int ph, int* r, int* t) {
        const bool last = ph0 + ph == a.phases - 1;
        const uint32_t tt = (uint32_t)t_total_of(ph);
        const uint32_t d = (uint32_t)((c * NW + kw) * 64 + lane);
        const uint32_t rr = __umulhi(d << 8, last ? magic_last : magic_full);
        *r = (int)rr;
        *t = (int)(d - rr * tt);
        return rr < 16u;
    };
    // the scale block of tile `tile` in phase `ph` (ph == n_ph: there is none, nothing is read)
    auto sp_load = [&](int tile, int ph, int c) {
        const int phc = min(ph, n_ph - 1);
        int r, t;
        const bool ok = (int)sp_place(c, phc, &r, &t) & (int)(ph < n_ph);
        const int row = min(tile * 16 + r, a.n - 1);
        return __builtin_amdgcn_raw_buffer_load_b32(rs, ok ? row * nblk + (t_begin_of(phc) + t) * 4 : kSentinel, 0, 0);
    };
    auto sp_store = [&](int slot, int ph, int c, uint32_t v) {
        int r, t;
        if (sp_place(c, min(ph, n_ph - 1), &r, &t))
            sc[(slot * 16 + r) * scw + t] = v;
    };
    // Always kCh + 1 loads per item (absent steps read nothing and return zero), so that the
    // in-order load counter can be waited on exactly.  The weight loads carry no streaming hint:
    // a wave load covers half a cache line per row and the next step wants the other half.
    auto issue = [&](const MPos& p, MItem& it) {
        const bool live = valid(p);
        const int tile = live ? p.tile : 0;
        const int ph = live ? p.ph : 0;
        const int row = min(tile * 16 + li, a.n - 1);             // ragged N: repeat the last row
        const int vq = row * q_row_bytes + lg * 16;
#pragma unroll
        for (int u = 0; u < kCh; ++u) {
            bool ok;
            const int t = step_of(p, u, &ok);
            // (an absent step's load differs from its neighbours' in the scalar offset, so that the
            // compiler cannot merge them into one and lose count of the loads in flight)
            it.q[u] = __builtin_amdgcn_raw_buffer_load_b128(rq, ok ? vq : kSentinel,
                                                            ok ? (t_begin_of(ph) + t) * 64 : u * 16, 0);
        }
        int ntile = tile, nph = ph;
        next_tile(&ntile, &nph);
        it.sp = sp_load(ntile, live ? nph : n_ph, p.c);
    };

    const int col = li % MP;
    float best_val = -INFINITY;       // wave 0: running winner of column li over rows 4 lg + r of all tiles
    int best_idx = 0x7FFFFFFF;

    if (wave == 0) {
        // Epilogue wave: one barrier per tile and phase, like the compute waves; no loads of its own.
        lds_barrier_mfma();                                       // scales of the first tile are in LDS
        int tp_done = 0;
        for (int ph = 0; ph < n_ph; ++ph) {
            int ti = 0;
            for (int tile = (int)blockIdx.x; tile < n_tiles; tile += gridDim.x, ++ti, ++tp_done) {
                const f32x4_t* slot = red + (size_t)(tp_done & 1) * NW * 64;
                lds_barrier_mfma();                               // partial tiles of (tile, ph) are in LDS
                f32x4_t sum = slot[lane];
#pragma unroll
                for (int w = 1; w < NW; ++w)
                    sum += slot[w * 64 + lane];
                if (n_ph > 1) {                                   // K split in time: phases add up in order
                    if (ph > 0)
                        sum = accl[ti * 64 + lane] + sum;
                    if (ph < n_ph - 1) {
                        accl[ti * 64 + lane] = sum;
                        continue;
                    }
                }
                // lane (li, lg) holds rows 4 lg + r of the tile for activation row li
                if constexpr (kEpi) {
                    // fused form without a split in space (there the finish kernel applies it)
                    if (!in_space) {
                        if (li < m_valid) {
                            const bool gated = epi.act == MXFP4_ACT_SWIGLU;
                            const int row0 = tile * 16 + 4 * lg;
                            const int cols = gated ? 2 : 4, col0 = gated ? row0 >> 1 : row0;
                            const int n_cols = gated ? a.n >> 1 : a.n;
                            float bias_v[4] = {0.f, 0.f, 0.f, 0.f}, res_v[4] = {0.f, 0.f, 0.f, 0.f};
                            uint16_t* y = a.y + (int64_t)(m0 + li) * a.ldy;
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                if (epi.bias && row0 + r < a.n)
                                    bias_v[r] = bf16_bits_to_f32(epi.bias[row0 + r]);
                                if (epi.residual && r < cols && col0 + r < n_cols)
                                    res_v[r] = bf16_bits_to_f32(epi.residual[(int64_t)(m0 + li) * epi.ldr + col0 + r]);
                            }
                            if (gated) {                          // rows (0, 1) and (2, 3) are (gate, up) pairs
#pragma unroll
                                for (int c = 0; c < 2; ++c)
                                    if (col0 + c < n_cols)
                                        y[col0 + c] = f32_to_bf16_rne(silu_gate(sum[2 * c] + bias_v[2 * c],
                                                                                sum[2 * c + 1] + bias_v[2 * c + 1]) +
                                                                      res_v[c]);
                            } else {
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    if (row0 + r < a.n)
                                        y[row0 + r] = f32_to_bf16_rne(sum[r] + bias_v[r] + res_v[r]);
                            }
                        }
                        continue;
                    }
                }
                if (li < m_valid) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int row = tile * 16 + 4 * lg + r;
                        if (row < a.n) {
                            if (in_space) {
                                a.splitk_ws[((int64_t)blockIdx.y * a.m + (m0 + li)) * a.n + row] = sum[r];
                            } else if (argmax) {
                                if (sum[r] > best_val) {          // rows ascend: lowest index wins ties
                                    best_val = sum[r];
                                    best_idx = row;
                                }
                            } else {
                                a.y[(int64_t)(m0 + li) * a.ldy + row] = f32_to_bf16_rne(sum[r]);
                            }
                        }
                    }
                }
            }
        }
    } else {
        MItem buf[D];
        MPos pos[D];
        MPos load{(int)blockIdx.x, 0, 0};
        // The weight loads go out first, with as few instructions in front of them as possible:
        // at three waves per SIMD every hundred instructions of set-up delay them by half a
        // microsecond, and nothing else can start before they are back anyway.
#pragma unroll
        for (int d = 0; d < D; ++d) {
            pos[d] = load;
            issue(load, buf[d]);
            advance(load);
            __builtin_amdgcn_sched_barrier(0);                    // keep the buffers' loads in issue order
        }
        // scale block of the first tile: four items' dwords in flight at a time
        uint32_t sp0[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            sp0[i] = sp_load((int)blockIdx.x, i < items ? 0 : n_ph, i);
        x_load(0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < items)
                sp_store(0, 0, i, sp0[i]);
        x_store(0);
#pragma unroll 1
        for (int c0 = kXBatch; c0 < items; c0 += kXBatch) {       // long K slices: the rest, batch by batch
            x_load(c0, 0);
            x_store(c0);
        }
#pragma unroll 1
        for (int c0 = 4; c0 < items; c0 += 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                sp0[i] = sp_load((int)blockIdx.x, c0 + i < items ? 0 : n_ph, c0 + i);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (c0 + i < items)
                    sp_store(0, 0, c0 + i, sp0[i]);
        }
        lds_barrier_mfma();                                       // scales of the first tile are in LDS

        f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};   // two chains: even and odd j
        int tp_done = 0;              // (tile, phase) pairs finished by this workgroup
        int cur_ph = 0;               // phase whose activations this wave holds in LDS
        auto compute = [&](const MPos& p, const MItem& it) {
            if (p.ph != cur_ph) {
                // entering the next phase of an in-time K split: this wave's slice of its activations
#pragma unroll 1
                for (int c0 = 0; c0 < items; c0 += kXBatch) {
                    x_load(c0, p.ph);
                    x_store(c0);
                }
                cur_ph = p.ph;
            }
            // the four steps' scale dwords of this lane's row; byte lg of dword u is its block's scale
            const u32x4_t sv = *reinterpret_cast<const u32x4_t*>(
                sc + ((tp_done & 1) * 16 + li) * scw + kw * steps_w + p.c * kCh);
            {
                int ntile = p.tile, nph = p.ph;
                next_tile(&ntile, &nph);
                sp_store((tp_done + 1) & 1, nph, p.c, it.sp);
            }
#pragma unroll
            for (int u = 0; u < kCh; ++u) {
                bool ok;
                step_of(p, u, &ok);
                const int local = p.c * kCh + u;                  // absent steps: zero weights, copied x
                u32x4_t xb[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    xb[j] = xw[(16 * local + 4 * j + lg) * MP + col];
                // The convert reads the exponent field as E8M0.  A step past the end of K gets scale
                // 2^-127 (its weights are zero, and what LDS holds there could say NaN).
                const uint32_t sbyte = ok ? ((sv[u] >> (8 * lg)) & 0xFFu) : 0u;
                const float scl = __uint_as_float(sbyte << 23);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t qd = it.q[u][j];
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
            if (p.c == items - 1) {
                // end of the tile: leave the partial tile for the epilogue wave
                f32x4_t* slot = red + (size_t)(tp_done & 1) * NW * 64;
                slot[kw * 64 + lane] = acc0 + acc1;
                acc0 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                acc1 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                lds_barrier_mfma();
                ++tp_done;
            }
        };

        // Positions only grow, so the walk ends when buffer 0 runs dry.  Every trip issues the
        // same loads whether or not the later buffers still had work: every path into the loop head then
        // carries the same queue of outstanding loads and the compiler's counter waits stay exact.
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
    }

    if (argmax && !in_space && wave == 0) {
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
            a.part_val[(int64_t)(m0 + lane) * a.parts + blockIdx.x] = best_val;
            a.part_idx[(int64_t)(m0 + lane) * a.parts + blockIdx.x] = best_idx;
        }
    }
}

// Second kernel of the split-K form: add the phases' partial products in phase order, then round
// and store, or find each workgroup's (max, index) for the argmax's last stage.
// kEpi: the fused form; a thread then takes one output column: one weight row, or with the gate
// the pair of rows 2c, 2c + 1.
template <bool kEpi>
__global__ __launch_bounds__(256) void splitk_finish_kernel(GemmArgs a, Epilogue epi)
{
    __shared__ float sv[4];
    __shared__ int si[4];
    const int tid = threadIdx.x;
    const bool argmax = a.part_val != nullptr;
    if constexpr (kEpi) {
        const bool gated = epi.act == MXFP4_ACT_SWIGLU;
        const int n_cols = gated ? a.n >> 1 : a.n;
        for (int m = blockIdx.y; m < a.m; m += gridDim.y) {
            for (int c = (int)blockIdx.x * 256 + tid; c < n_cols; c += gridDim.x * 256) {
                const int n0 = gated ? 2 * c : c;
                float z0 = 0.f, z1 = 0.f;
                for (int p = 0; p < a.phases; ++p) {
                    const float* w = a.splitk_ws + ((int64_t)p * a.m + m) * a.n + n0;
                    z0 += w[0];
                    if (gated)
                        z1 += w[1];
                }
                if (epi.bias) {
                    z0 += bf16_bits_to_f32(epi.bias[n0]);
                    if (gated)
                        z1 += bf16_bits_to_f32(epi.bias[n0 + 1]);
                }
                float t = gated ? silu_gate(z0, z1) : z0;
                if (epi.residual)
                    t += bf16_bits_to_f32(epi.residual[(int64_t)m * epi.ldr + c]);
                a.y[(int64_t)m * a.ldy + c] = f32_to_bf16_rne(t);
            }
        }
        return;
    }
    for (int m = blockIdx.y; m < a.m; m += gridDim.y) {
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int n = (int)blockIdx.x * 256 + tid; n < a.n; n += gridDim.x * 256) {
        float sum = 0.f;
        for (int p = 0; p < a.phases; ++p)
            sum += a.splitk_ws[((int64_t)p * a.m + m) * a.n + n];
        if (argmax) {
            if (sum > bv) {                                       // n ascends per thread
                bv = sum;
                bi = n;
            }
        } else {
            a.y[(int64_t)m * a.ldy + n] = f32_to_bf16_rne(sum);
        }
    }
    if (argmax) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float v = __shfl_xor(bv, off);
            const int i = __shfl_xor(bi, off);
            if (v > bv || (v == bv && i < bi)) {
                bv = v;
                bi = i;
            }
        }
        if ((tid & 63) == 0) {
            sv[tid >> 6] = bv;
            si[tid >> 6] = bi;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 4; ++w)
                if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) {
                    bv = sv[w];
                    bi = si[w];
                }
            a.part_val[(int64_t)m * a.parts + blockIdx.x] = bv;
            a.part_idx[(int64_t)m * a.parts + blockIdx.x] = bi;
        }
        __syncthreads();                                          // sv, si are reused by the next row
    }
    }
}

// Launch one pass.  The grid is what is resident at once (asked of the runtime: the LDS a
// workgroup may use is less than the nominal size divides into), by default one workgroup per CU
// (measured: eight compute waves per CU with two items in flight each already saturate the memory
// system, and a second workgroup only lengthens the start-up burst), split over grid_y phases
// when K is split in space.  *blocks is the cap on workgroups per phase on entry (0 = none) and
// the count used on return.
template <int MP, int NW, int D, bool kEpi>
hipError_t launch_one(const GemmArgs& a, int m0, int grid_y, size_t lds, const DeviceInfo& dev, int* blocks,
                      hipStream_t stream, const Epilogue& epi)
{
    auto kern = mfma_kernel<MP, NW, D, kEpi>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), dev.lds_bytes); e != hipSuccess)
        return e;
    thread_local size_t occ_lds = ~(size_t)0;
    thread_local int occ = 0;
    if (occ_lds != lds) {
        int nb = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, reinterpret_cast<const void*>(kern),
                                                                   (NW + 1) * 64, lds);
        if (e != hipSuccess)
            return e;
        occ = nb;
        occ_lds = lds;
    }
    static const int max_per_cu = [] {                             // MXFP4_MFMA_WGS: measurement only
        const char* e = knob("MXFP4_MFMA_WGS");
        const int v = e ? atoi(e) : 0;
        return v >= 1 && v <= 4 ? v : 1;
    }();
    const int per_cu = occ < 1 ? 1 : (occ > max_per_cu ? max_per_cu : occ);
    const int n_tiles = (a.n + 15) / 16;
    int nb = dev.cus * per_cu / grid_y;
    nb = nb < 1 ? 1 : (nb > n_tiles ? n_tiles : nb);
    if (nb > gemv_max_parts(dev))
        nb = gemv_max_parts(dev);
    if (*blocks > 0 && nb > *blocks)
        nb = *blocks;
    *blocks = nb;
    hipLaunchKernelGGL(kern, dim3(nb, grid_y), dim3((NW + 1) * 64), lds, stream, a, m0, epi);
    return hipGetLastError();
}

constexpr int kNW = 8;

constexpr size_t kRedBytes = (size_t)2 * kNW * 64 * 16;
constexpr int kGrain = kNW * kCh;      // steps that give every compute wave one item
constexpr size_t kAccCap = 16 * 1024;  // in-time split: running sums of at most 16 tiles per workgroup in LDS

size_t lds_need(int steps, int mp)
{
    return x_lds_bytes<kNW>(steps, mp) + kRedBytes + (size_t)2 * 16 * scale_row_dwords_t<kNW>(steps) * 4;
}

// LDS a workgroup should stay under when K may be split: all of it (one workgroup per CU), so K is
// only cut when the activation rows of a pass cannot be held whole.
size_t lds_target(const DeviceInfo& dev)
{
    static const int env = [] {
        const char* e = knob("MXFP4_MFMA_LDS_TARGET");
        return e ? atoi(e) : 0;
    }();
    return env > 0 ? (size_t)env : (size_t)dev.lds_bytes;
}

// Steps per phase (a multiple of kCh) and number of phases for a pass of `mp` activation rows,
// with `reserve` bytes of LDS kept for other use.
void plan_phases(int k, int mp, const DeviceInfo& dev, bool may_split, size_t reserve, int* phase_steps,
                 int* phases)
{
    const int t_total = k / 128;
    int steps = (t_total + kCh - 1) / kCh * kCh;
    if (may_split) {
        // per step: 256 bytes of activations per row and 2 x 16 scale dwords; 512 more for the skew
        const size_t fixed = kRedBytes + 512 + reserve, per_step = (size_t)256 * mp + 128;
        int fit = lds_target(dev) > fixed ? (int)((lds_target(dev) - fixed) / per_step) / kGrain * kGrain : 0;
        if (fit < kGrain && (size_t)dev.lds_bytes > fixed)
            fit = (int)(((size_t)dev.lds_bytes - fixed) / per_step) / kGrain * kGrain;
        if (fit < kGrain)
            fit = kGrain;                                         // the caller checks that it fits
        if (fit < steps) {
            const int p = (t_total + fit - 1) / fit;
            steps = ((t_total + p - 1) / p + kCh - 1) / kCh * kCh;     // even phases
        }
    }
    *phase_steps = steps;
    *phases = (t_total + steps - 1) / steps;
}

int pass_width(int left) { return left > 8 ? 16 : (left > 4 ? 8 : 4); }

// Workgroups of a pass whose K is split (one per CU: its LDS is more than half full).
int split_blocks(int n, const DeviceInfo& dev)
{
    const int n_tiles = (n + 15) / 16;
    int nb = dev.cus < n_tiles ? dev.cus : n_tiles;
    return nb < gemv_max_parts(dev) ? nb : gemv_max_parts(dev);
}

// How a pass of `mp` rows deals with activations that do not fit the LDS whole.
enum SplitMode { kNoSplit, kInTime, kInSpace, kNarrow };

// In space when the caller gave a workspace (measured faster: the phases run side by side and
// every workgroup copies its activations once; in time every phase change exposes the latency of
// the next copy); else in time when the workgroup's tiles are few enough to keep their running
// sums in LDS beside one phase of activations; else narrower passes.
SplitMode split_mode(int mp, int n, int k, const DeviceInfo& dev, bool have_ws, size_t* acc_bytes)
{
    const int steps_all = (k / 128 + kCh - 1) / kCh * kCh;
    *acc_bytes = 0;
    if (lds_need(steps_all, mp) <= (size_t)dev.lds_bytes)
        return kNoSplit;
    if (have_ws)
        return kInSpace;
    const int nb = split_blocks(n, dev);
    const size_t acc = (size_t)(((n + 15) / 16 + nb - 1) / nb) * 1024;
    if (acc <= kAccCap) {
        int steps, phases;
        plan_phases(k, mp, dev, true, acc, &steps, &phases);
        if (lds_need(steps, mp) + acc <= (size_t)dev.lds_bytes) {
            *acc_bytes = acc;
            return kInTime;
        }
    }
    return kNarrow;
}

}  // namespace

bool mfma_can_run(const GemmArgs& a, const DeviceInfo& dev, bool have_splitk_ws)
{
    if (a.k % 128 != 0)
        return false;
    // four rows must be able to run: whole, split in time, or split in space with a workspace
    size_t acc;
    return split_mode(4, a.n, a.k, dev, have_splitk_ws, &acc) != kNarrow;
}

size_t mfma_splitk_bytes(int m, int n, int k, const DeviceInfo& dev)
{
    if (k % 128 != 0)
        return 0;
    size_t acc;
    const int mp = pass_width(m);                                 // the first pass is the widest
    if (split_mode(mp, n, k, dev, true, &acc) != kInSpace)
        return 0;
    int steps, phases;
    plan_phases(k, mp, dev, true, 0, &steps, &phases);
    return (size_t)phases * m * n * sizeof(float);
}

// The tile-major copy with K split in space: the call has a workspace and a phase of the widest
// pass fits the tile kernel.
bool mfma_tiled_split_can_run(const GemmArgs& a, const DeviceInfo& dev)
{
    if (a.k % 128 != 0 || a.m < 1 || a.ldx > 0x7FFFFFFF)
        return false;
    size_t acc_bytes = 0;
    if (split_mode(pass_width(a.m), a.n, a.k, dev, true, &acc_bytes) != kInSpace)
        return false;
    int steps = 0, phases = 1;
    plan_phases(a.k, pass_width(a.m), dev, true, 0, &steps, &phases);
    return mfma_tile_split_fits(steps, pass_width(a.m), dev);
}

hipError_t launch_mfma(const GemmArgs& a_in, const DeviceInfo& dev, float* splitk_ws, int* parts_used,
                       hipStream_t stream, bool general_only, const Epilogue* epi, bool tiled)
{
    if (tiled && (!splitk_ws || !mfma_tiled_split_can_run(a_in, dev)))
        return hipErrorInvalidValue;
    static const bool legacy = [] {
        const char* e = knob("MXFP4_MFMA_LEGACY");
        return e && atoi(e) != 0;
    }();
    if (!tiled && !legacy && !general_only && mfma_tile_can_run(a_in, dev))
        return launch_mfma_tile(a_in, dev, parts_used, stream, false, epi);
    if (!tiled && !legacy && !general_only && !epi && mfma_tile_phased_preferred(a_in, dev, splitk_ws != nullptr))
        return launch_mfma_tile_phased(a_in, dev, stream, false);
    if (!mfma_can_run(a_in, dev, splitk_ws != nullptr))
        return hipErrorInvalidValue;
    GemmArgs a = a_in;
    // the widest pass decides how the call deals with activations that do not fit the LDS; a split
    // in space uses one plan for all passes (the finish kernel adds the same phases for every row)
    size_t acc_bytes = 0;
    const SplitMode mode = split_mode(pass_width(a.m), a.n, a.k, dev, splitk_ws != nullptr, &acc_bytes);
    int space_steps = 0, space_phases = 1;
    if (mode == kInSpace)
        plan_phases(a.k, pass_width(a.m), dev, true, 0, &space_steps, &space_phases);
    // split in space: the leaner tile kernel takes the passes when a phase's activations fit it
    const bool tile_split = tiled || (mode == kInSpace && !legacy && !general_only && a.ldx <= 0x7FFFFFFF &&
                                      mfma_tile_split_fits(space_steps, pass_width(a.m), dev));
    int first_blocks = 0;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        int mp = pass_width(left);
        if (tile_split) {
            hipError_t e = launch_mfma_tile_split(a, m0, mp, space_phases, space_steps, splitk_ws, dev, stream, tiled);
            if (e != hipSuccess)
                return e;
            m0 += mp;
            continue;
        }
        int steps, phases, grid_y = 1;
        size_t lds;
        int blocks = 0;
        a.splitk_ws = nullptr;
        if (mode == kInSpace) {
            steps = space_steps;
            phases = grid_y = space_phases;
            lds = lds_need(steps, mp);
            a.splitk_ws = splitk_ws;
        } else {
            // the widest pass that runs whole or with K split in time
            SplitMode pm = split_mode(mp, a.n, a.k, dev, false, &acc_bytes);
            while (pm == kNarrow && mp > 4) {
                mp >>= 1;
                pm = split_mode(mp, a.n, a.k, dev, false, &acc_bytes);
            }
            if (pm == kNarrow)
                return hipErrorInvalidValue;
            if (pm == kInTime) {
                plan_phases(a.k, mp, dev, true, acc_bytes, &steps, &phases);
                lds = lds_need(steps, mp) + (phases > 1 ? acc_bytes : 0);
                blocks = split_blocks(a.n, dev);                  // the running sums are sized for this grid
            } else {
                plan_phases(a.k, mp, dev, false, 0, &steps, &phases);
                lds = lds_need(steps, mp);
            }
        }
        if (lds > (size_t)dev.lds_bytes)
            return hipErrorInvalidValue;
        // the argmax partial arrays are indexed by workgroup: no pass may use more than the first
        if (a.part_val != nullptr && mode != kInSpace && first_blocks > 0 && (blocks == 0 || blocks > first_blocks))
            blocks = first_blocks;
        a.phases = phases;
        a.phase_steps = steps;
        static const int depth = [] {                             // MXFP4_MFMA_DEPTH: measurement only
            const char* e = knob("MXFP4_MFMA_DEPTH");
            const int v = e ? atoi(e) : 0;
            return v >= 2 && v <= 4 ? v : 2;
        }();
        hipError_t e;
        // the fused form exists at the default depth only
#define MXFP4_MFMA_CASE(MP_)                                                                       \
    (epi          ? launch_one<MP_, kNW, 2, true>(a, m0, grid_y, lds, dev, &blocks, stream, *epi)    \
     : depth == 4 ? launch_one<MP_, kNW, 4, false>(a, m0, grid_y, lds, dev, &blocks, stream, Epilogue{})  \
     : depth == 3 ? launch_one<MP_, kNW, 3, false>(a, m0, grid_y, lds, dev, &blocks, stream, Epilogue{})  \
                  : launch_one<MP_, kNW, 2, false>(a, m0, grid_y, lds, dev, &blocks, stream, Epilogue{}))
        if (mp == 16)
            e = MXFP4_MFMA_CASE(16);
        else if (mp == 8)
            e = MXFP4_MFMA_CASE(8);
        else
            e = MXFP4_MFMA_CASE(4);
#undef MXFP4_MFMA_CASE
        if (e != hipSuccess)
            return e;
        if (m0 == 0)
            first_blocks = blocks;
        m0 += mp;
    }
    if (mode == kInSpace) {
        // every pass used the widest pass's plan, so every row has all phases written
        a.splitk_ws = splitk_ws;
        a.phases = space_phases;
        int fblocks = (a.n + 255) / 256;
        if (fblocks > gemv_max_parts(dev))
            fblocks = gemv_max_parts(dev);
        if (epi)
            hipLaunchKernelGGL(splitk_finish_kernel<true>, dim3(fblocks, a.m < 1024 ? a.m : 1024), dim3(256), 0,
                               stream, a, *epi);
        else
            hipLaunchKernelGGL(splitk_finish_kernel<false>, dim3(fblocks, a.m < 1024 ? a.m : 1024), dim3(256), 0,
                               stream, a, Epilogue{});
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
        first_blocks = fblocks;
    }
    if (parts_used)
        *parts_used = first_blocks;
    return hipSuccess;
}

}  // namespace mxfp4
