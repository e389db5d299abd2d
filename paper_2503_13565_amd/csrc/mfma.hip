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
// one 128-bit LDS read; activations are staged once per workgroup as [T][j][g][MP] chunks of 8
// elements, so that one wave read covers one contiguous run.  NW compute waves of a workgroup split K, each accumulates
// a 16 x 16 FP32 tile over its K slice and leaves it in LDS; one more wave, which never loads
// weights, sums the partial tiles in a fixed order, rounds and stores (or tracks the argmax), so
// that the compute waves only ever have loads in flight and their load counter stays exact.
// Workgroups are persistent over tiles; loads run one item (4 steps) ahead in a second register
// buffer.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

namespace {

constexpr int kCh = 4;             // steps (16-byte loads per lane) per pipeline item
constexpr int kSentinel = 0x7FFFFFF0;   // lane offset beyond any descriptor: the load returns zero

__device__ __forceinline__ void lds_barrier_mfma()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

struct MItem {
    u32x4_t q[kCh];     // 32 nibbles per step
    u32x4_t s;          // the 16 scale bytes of the row's 16 blocks of this item (4 steps x 4 groups)
};

struct MPos {
    int tile;
    int c;          // item within the tile
};

// MP: activation rows held per pass (4, 8 or 16); NW: compute waves per workgroup (they split K);
// the workgroup has NW + 1 waves, wave 0 is the epilogue wave.
template <int MP, int NW>
__global__ __launch_bounds__((NW + 1) * 64) void mfma_kernel(GemmArgs a, int m0)
{
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                          // [steps][4][4][MP] chunks of 8 elements
    f32x4_t* red = reinterpret_cast<f32x4_t*>(smem + (size_t)a.phase_steps * 256 * MP);  // [2][NW][64] partial tiles
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave - 1;                                      // K slice of a compute wave
    const int li = lane & 15, lg = lane >> 4;
    const int nblk = a.k >> 5;
    const int q_row_bytes = a.k >> 1;
    // this workgroup's K range in steps of 4 blocks: all of K, or one phase of the split-K form
    const int t_begin = (int)blockIdx.y * a.phase_steps;
    const int t_end = min(a.k >> 7, t_begin + a.phase_steps);
    const int t_total = t_end - t_begin;
    // steps per wave and tile, in whole items of kCh steps, so that an item's 16 scale bytes per
    // row are one run that starts at a multiple of 16 blocks
    const int items = ((t_total + kCh - 1) / kCh + NW - 1) / NW;
    const int steps_w = items * kCh;
    const int n_tiles = (a.n + 15) >> 4;
    const bool argmax = a.part_val != nullptr;
    const int m_valid = min(MP, a.m - m0);

    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.q), 0, a.n * q_row_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a.s), 0, a.n * nblk, 0x00020000);

    // Stage the activations (all waves; the compute waves do it after their first weight loads are
    // out).  Chunk c = 16 T + 4 g + j of row m goes to xs[(16 T + 4 j + g) * MP + m]: the four lane
    // groups of one MFMA then read four adjacent segments, 1 KiB contiguous per wave read at
    // MP = 16, which is free of bank conflicts however the hardware groups the lanes.  Rows past M
    // repeat the last.  Consecutive threads read consecutive chunks of a row; four independent
    // loads per thread are in flight at a time.
    auto stage_x = [&]() {
        const int chunks = t_total * 16;                          // of this K range
        constexpr int kBatch = 4;
        constexpr int kThreads = (NW + 1) * 64;
#pragma unroll 1
        for (int m = 0; m < MP; ++m) {
            const int msrc = min(m0 + m, a.m - 1);
            const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx) + t_begin * 16;
            for (int c0 = tid; c0 < chunks; c0 += kBatch * kThreads) {
                u32x4_t v[kBatch];
#pragma unroll
                for (int b = 0; b < kBatch; ++b)
                    v[b] = xp[min(c0 + b * kThreads, chunks - 1)];
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    const int c = min(c0 + b * kThreads, chunks - 1);   // clamped duplicates rewrite the same data
                    const int slot = (c & ~15) | ((c & 3) << 2) | ((c >> 2) & 3);
                    xs[slot * MP + m] = v[b];
                }
            }
        }
    };

    auto valid = [&](const MPos& p) { return p.tile < n_tiles; };
    auto advance = [&](MPos& p) {
        if (++p.c == items) {
            p.c = 0;
            p.tile += gridDim.x;
        }
    };
    // Step T of this wave for slot u of item c, and whether it exists (wave-uniform).
    auto step_of = [&](const MPos& p, int u, bool* ok) {
        const int local = p.c * kCh + u;
        const int t = kw * steps_w + local;                       // relative to t_begin
        *ok = valid(p) && local < steps_w && t < t_total;
        return t;
    };
    // Always kCh + 1 loads per item (absent steps read nothing and return zero), so that the
    // in-order load counter can be waited on exactly.  The weight loads carry no streaming hint:
    // a wave load covers half a cache line per row and the next step wants the other half.  The
    // scales of an item are one 16-byte load per row (the four lanes of a row load the same bytes):
    // 16 cache lines touched per item instead of 64 with a byte load per step.
    auto issue = [&](const MPos& p, MItem& it) {
        const int tile = valid(p) ? p.tile : 0;
        const int row = min(tile * 16 + li, a.n - 1);             // ragged N: repeat the last row
        const int vq = row * q_row_bytes + lg * 16;
#pragma unroll
        for (int u = 0; u < kCh; ++u) {
            bool ok;
            const int t = step_of(p, u, &ok);
            it.q[u] = __builtin_amdgcn_raw_buffer_load_b128(rq, ok ? vq : kSentinel, ok ? (t_begin + t) * 64 : 0, 0);
        }
        bool ok0;
        const int t0 = step_of(p, 0, &ok0);
        it.s = __builtin_amdgcn_raw_buffer_load_b128(rs, ok0 ? row * nblk : kSentinel, ok0 ? (t_begin + t0) * 4 : 0, 0);
    };

    const int col = li % MP;
    float best_val = -INFINITY;       // wave 0: running winner of column li over rows 4 lg + r of all tiles
    int best_idx = 0x7FFFFFFF;

    if (wave == 0) {
        // Epilogue wave: one barrier per tile, like the compute waves; no weight loads of its own.
        stage_x();
        lds_barrier_mfma();                                       // activations staged
        int tiles_done = 0;
        for (int tile = (int)blockIdx.x; tile < n_tiles; tile += gridDim.x, ++tiles_done) {
            const f32x4_t* slot = red + (size_t)(tiles_done & 1) * NW * 64;
            lds_barrier_mfma();                                   // partial tiles of `tile` are in LDS
            f32x4_t sum = slot[lane];
#pragma unroll
            for (int w = 1; w < NW; ++w)
                sum += slot[w * 64 + lane];
            // lane (li, lg) holds rows 4 lg + r of the tile for activation row li
            if (li < m_valid) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = tile * 16 + 4 * lg + r;
                    if (row < a.n) {
                        if (a.splitk_ws) {
                            a.splitk_ws[((int64_t)blockIdx.y * a.m + (m0 + li)) * a.n + row] = sum[r];
                        } else if (argmax) {
                            if (sum[r] > best_val) {              // rows ascend: lowest index wins ties
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
    } else {
        MItem buf[2];
        MPos pos[2];
        MPos load{(int)blockIdx.x, 0};
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            pos[d] = load;
            issue(load, buf[d]);
            advance(load);
            __builtin_amdgcn_sched_barrier(0);                    // keep the buffers' loads in issue order
        }
        stage_x();
        lds_barrier_mfma();                                       // activations staged

        f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};   // two chains: even and odd j
        int tiles_done = 0;
        auto compute = [&](const MPos& p, const MItem& it) {
#pragma unroll
            for (int u = 0; u < kCh; ++u) {
                bool ok;
                const int t = step_of(p, u, &ok);
                const int tc = ok ? t : 0;                        // absent steps: zero weights, any finite x
                u32x4_t xb[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    xb[j] = xs[(16 * tc + 4 * j + lg) * MP + col];
                // byte lg of dword u is this lane's block scale; the convert reads the exponent field
                // as E8M0.  A step past the end of K gets scale 2^-127 (its weights are zero, and
                // bytes read past the row's scales could say NaN).
                const uint32_t sbyte = ok ? ((it.s[u] >> (8 * lg)) & 0xFFu) : 0u;
                const float sc = __uint_as_float(sbyte << 23);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t qd = it.q[u][j];
                    u32x4_t w;
                    w[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 0));
                    w[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 1));
                    w[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 2));
                    w[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(qd, sc, 3));
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
                f32x4_t* slot = red + (size_t)(tiles_done & 1) * NW * 64;
                slot[kw * 64 + lane] = acc0 + acc1;
                acc0 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                acc1 = f32x4_t{0.f, 0.f, 0.f, 0.f};
                lds_barrier_mfma();
                ++tiles_done;
            }
        };

        // Positions only grow, so the walk ends when buffer 0 runs dry.  Every trip issues the
        // same loads whether or not buffer 1 still had work: every path into the loop head then
        // carries the same queue of outstanding loads and the compiler's counter waits stay exact.
        while (valid(pos[0])) {
            compute(pos[0], buf[0]);
            pos[0] = load;
            issue(load, buf[0]);
            advance(load);
            if (valid(pos[1]))
                compute(pos[1], buf[1]);
            pos[1] = load;
            issue(load, buf[1]);
            advance(load);
        }
    }

    if (argmax && !a.splitk_ws && wave == 0) {
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
__global__ __launch_bounds__(256) void splitk_finish_kernel(GemmArgs a)
{
    __shared__ float sv[4];
    __shared__ int si[4];
    const int tid = threadIdx.x;
    const bool argmax = a.part_val != nullptr;
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

template <int MP, int NW>
hipError_t launch_one(const GemmArgs& a, int m0, int blocks, int phases, size_t lds, int max_lds,
                      hipStream_t stream)
{
    auto kern = mfma_kernel<MP, NW>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (e != hipSuccess)
            return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(blocks, phases), dim3((NW + 1) * 64), lds, stream, a, m0);
    return hipGetLastError();
}

constexpr int kNW = 8;

size_t lds_need(int steps, int mp) { return (size_t)steps * 256 * mp + (size_t)2 * kNW * 64 * 16; }

// LDS a workgroup should stay under when K may be split: two workgroups per CU.
size_t lds_target(const DeviceInfo& dev)
{
    static const int env = [] {
        const char* e = getenv("MXFP4_MFMA_LDS_TARGET");
        return e ? atoi(e) : 0;
    }();
    return env > 0 ? (size_t)env : (size_t)dev.lds_bytes / 2;
}

// Steps per phase (a multiple of kCh) and number of phases for a pass of `mp` activation rows.
void plan_phases(int k, int mp, const DeviceInfo& dev, bool may_split, int* phase_steps, int* phases)
{
    const int t_total = k / 128;
    int steps = (t_total + kCh - 1) / kCh * kCh;
    if (may_split) {
        // two workgroups per CU if a phase still gives every compute wave an item, else one
        const size_t red_bytes = (size_t)2 * kNW * 64 * 16;
        int fit = (int)((lds_target(dev) - red_bytes) / ((size_t)256 * mp)) / kCh * kCh;
        if (fit < kNW * kCh)
            fit = (int)(((size_t)dev.lds_bytes - red_bytes) / ((size_t)256 * mp)) / kCh * kCh;
        if (fit < kCh)
            fit = kCh;
        if (fit < steps) {
            const int p = (t_total + fit - 1) / fit;
            steps = ((t_total + p - 1) / p + kCh - 1) / kCh * kCh;     // even phases
        }
    }
    *phase_steps = steps;
    *phases = (t_total + steps - 1) / steps;
}

int pass_width(int left) { return left > 8 ? 16 : (left > 4 ? 8 : 4); }

}  // namespace

bool mfma_can_run(const GemmArgs& a, const DeviceInfo& dev, bool have_splitk_ws)
{
    if (a.k % 128 != 0)
        return false;
    // with room for split-K partial products any K goes; without, four rows of all of K must fit
    return have_splitk_ws || lds_need((a.k / 128 + kCh - 1) / kCh * kCh, 4) <= (size_t)dev.lds_bytes;
}

size_t mfma_splitk_bytes(int m, int n, int k, const DeviceInfo& dev)
{
    if (k % 128 != 0)
        return 0;
    int max_phases = 1;
    for (int m0 = 0; m0 < m;) {
        const int mp = pass_width(m - m0);
        int steps, phases;
        plan_phases(k, mp, dev, true, &steps, &phases);
        max_phases = phases > max_phases ? phases : max_phases;
        m0 += mp;
    }
    return max_phases > 1 ? (size_t)max_phases * m * n * sizeof(float) : 0;
}

hipError_t launch_mfma(const GemmArgs& a_in, const DeviceInfo& dev, float* splitk_ws, int* parts_used,
                       hipStream_t stream)
{
    if (!mfma_can_run(a_in, dev, splitk_ws != nullptr))
        return hipErrorInvalidValue;
    GemmArgs a = a_in;
    const int n_tiles = (a.n + 15) / 16;
    // one plan for the whole call: the widest pass decides the phases (narrower passes fit too)
    bool split = false;
    int split_steps = 0, split_phases = 1;
    if (splitk_ws) {
        plan_phases(a.k, pass_width(a.m), dev, true, &split_steps, &split_phases);
        split = split_phases > 1;
    }
    int first_blocks = 0;
    int max_phases = 1;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        int mp = pass_width(left);
        int steps = split_steps, phases = split_phases;
        if (!split) {
            plan_phases(a.k, mp, dev, false, &steps, &phases);
            // all of K in one pass: the widest pass whose activation copy fits the LDS
            while (mp > 4 && lds_need(steps, mp) > (size_t)dev.lds_bytes)
                mp >>= 1;
        }
        const size_t lds = lds_need(steps, mp);
        int per_cu = (int)((size_t)dev.lds_bytes / lds);
        per_cu = per_cu < 1 ? 1 : (per_cu > 2 ? 2 : per_cu);      // 9 waves each: a third would not fit the SIMDs evenly
        int blocks = dev.cus * per_cu / phases;
        blocks = blocks < 1 ? 1 : (blocks > n_tiles ? n_tiles : blocks);
        if (blocks > gemv_max_parts(dev))
            blocks = gemv_max_parts(dev);
        if (m0 == 0)
            first_blocks = blocks;
        // the argmax partial arrays are indexed by workgroup: keep the grid the same for all passes
        if (a.part_val != nullptr && !split)
            blocks = first_blocks < blocks ? first_blocks : blocks;
        a.splitk_ws = split ? splitk_ws : nullptr;
        a.phases = phases;
        a.phase_steps = steps;
        max_phases = phases > max_phases ? phases : max_phases;
        hipError_t e;
        if (mp == 16)
            e = launch_one<16, kNW>(a, m0, blocks, phases, lds, dev.lds_bytes, stream);
        else if (mp == 8)
            e = launch_one<8, kNW>(a, m0, blocks, phases, lds, dev.lds_bytes, stream);
        else
            e = launch_one<4, kNW>(a, m0, blocks, phases, lds, dev.lds_bytes, stream);
        if (e != hipSuccess)
            return e;
        m0 += mp;
    }
    if (split) {
        // every pass used the widest pass's plan, so every row has all phases written
        a.phases = max_phases;
        int fblocks = (a.n + 255) / 256;
        if (fblocks > gemv_max_parts(dev))
            fblocks = gemv_max_parts(dev);
        hipLaunchKernelGGL(splitk_finish_kernel, dim3(fblocks, a.m < 1024 ? a.m : 1024), dim3(256), 0, stream, a);
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
