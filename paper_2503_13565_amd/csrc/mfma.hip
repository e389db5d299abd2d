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
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                          // [K/8][MP] chunks of 8 elements
    f32x4_t* red = reinterpret_cast<f32x4_t*>(smem + (size_t)a.k * 2 * MP);  // [2][NW][64] partial tiles
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave - 1;                                      // K slice of a compute wave
    const int li = lane & 15, lg = lane >> 4;
    const int nblk = a.k >> 5;
    const int q_row_bytes = a.k >> 1;
    const int t_total = a.k >> 7;                                 // steps of 4 blocks along K
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
        const int chunks = a.k >> 3;
        constexpr int kBatch = 4;
        constexpr int kThreads = (NW + 1) * 64;
#pragma unroll 1
        for (int m = 0; m < MP; ++m) {
            const int msrc = min(m0 + m, a.m - 1);
            const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
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
        const int t = kw * steps_w + local;
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
            it.q[u] = __builtin_amdgcn_raw_buffer_load_b128(rq, ok ? vq : kSentinel, ok ? t * 64 : 0, 0);
        }
        bool ok0;
        const int t0 = step_of(p, 0, &ok0);
        it.s = __builtin_amdgcn_raw_buffer_load_b128(rs, ok0 ? row * nblk : kSentinel, ok0 ? t0 * 4 : 0, 0);
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
                        if (argmax) {
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

    if (argmax && wave == 0) {
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

template <int MP, int NW>
hipError_t launch_one(const GemmArgs& a, int m0, int blocks, size_t lds, int max_lds, hipStream_t stream)
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
    hipLaunchKernelGGL(kern, dim3(blocks), dim3((NW + 1) * 64), lds, stream, a, m0);
    return hipGetLastError();
}

size_t lds_need(int k, int mp, int nw) { return (size_t)k * 2 * mp + (size_t)2 * nw * 64 * 16; }

}  // namespace

bool mfma_can_run(const GemmArgs& a, const DeviceInfo& dev)
{
    return a.k % 128 == 0 && lds_need(a.k, 4, 8) <= (size_t)dev.lds_bytes;
}

hipError_t launch_mfma(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    if (!mfma_can_run(a, dev))
        return hipErrorInvalidValue;
    constexpr int NW = 8;
    const int n_tiles = (a.n + 15) / 16;
    int first_blocks = 0;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        // the widest pass whose activation copy fits the LDS, but no wider than needed
        int mp = left > 8 ? 16 : (left > 4 ? 8 : 4);
        while (mp > 4 && lds_need(a.k, mp, NW) > (size_t)dev.lds_bytes)
            mp >>= 1;
        const size_t lds = lds_need(a.k, mp, NW);
        int per_cu = (int)((size_t)dev.lds_bytes / lds);
        per_cu = per_cu < 1 ? 1 : (per_cu > 2 ? 2 : per_cu);          // 9 waves each: a third one would not fit the SIMDs evenly
        int blocks = n_tiles < dev.cus * per_cu ? n_tiles : dev.cus * per_cu;
        if (blocks > gemv_max_parts(dev))
            blocks = gemv_max_parts(dev);
        if (m0 == 0)
            first_blocks = blocks;
        // the argmax partial arrays are indexed by workgroup: keep the grid the same for all passes
        if (a.part_val != nullptr)
            blocks = first_blocks < blocks ? first_blocks : blocks;
        hipError_t e;
        if (mp == 16)
            e = launch_one<16, NW>(a, m0, blocks, lds, dev.lds_bytes, stream);
        else if (mp == 8)
            e = launch_one<8, NW>(a, m0, blocks, lds, dev.lds_bytes, stream);
        else
            e = launch_one<4, NW>(a, m0, blocks, lds, dev.lds_bytes, stream);
        if (e != hipSuccess)
            return e;
        if (a.part_val != nullptr && blocks != first_blocks)
            return hipErrorInvalidValue;                           // cannot happen: LDS need only shrinks
        m0 += mp;
    }
    if (parts_used)
        *parts_used = first_blocks;
    return hipSuccess;
}

}  // namespace mxfp4
