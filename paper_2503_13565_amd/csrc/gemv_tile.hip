// The decode step (one or two activation rows) on the tile-major copy of the weights, so that one
// stored layout serves both the draft's single-row steps and the verification passes (arXiv
// 2503.13565, section 3.3: the intermediate MXFP4 model both drafts and verifies; section 3.5 lists the
// memory of a second model copy as a limitation; sections 3.4.3 and 4.4 for the product, Eq. 2).
//
// Tile-major tensors (made by tile_repack_kernel): q as [tile of 16 rows][step of 128 elements][lane =
// i + 16 g][16 bytes], lane (i, g) holding block 4 step + g of row 16 tile + i; scale bytes as
// [tile][item of 4 steps][row i][16 bytes], dword = step, byte = g.  A wave load is one contiguous
// KiB, as in the row-major decode kernel, but it is 16 rows x 128 elements instead of one row x 2048.
//
// One workgroup of 16 waves per compute unit walks the tiles b, b + G, ...; inside a tile the waves
// split K: wave w takes the steps [w spw, (w + 1) spw), the same for every tile, so the 32 spw
// activations a lane meets never change and sit in registers (one row: up to four steps per wave, K <=
// 8192; two rows: two; else they are read from the LDS copy every step).  A wave's steps of one tile are in flight (32 KiB per compute unit at
// K = 4096); each buffer is refilled with the next tile's step as soon as it has been used.  A
// lane accumulates its row over its blocks; at a tile's end the four lanes of a row are added, the wave
// leaves 16 partial sums in LDS and counts itself in at the tile's LDS counter; the wave that completes
// the count adds the partial sums in wave order (the same value whoever adds them) and keeps the 16
// outputs in LDS, or the best of them for the fused pick; the outputs are stored when the workgroup
// is done.  No wave waits for another before that.
#include "common.h"
#include "kernels.h"

namespace mxfp4 {

namespace {

constexpr int kOobT = 0x7FFFFFF0;        // lane offset beyond any descriptor: the load returns zero
constexpr int kWavesT = 16;

struct TPos {
    int j;      // tile of this workgroup's sequence
    int s;      // step of this wave's range
};

// kRegs: the wave's activations in registers (SPW steps of 16 dwords per row), else from LDS.
template <int MT, int SPW, bool kRegs, int NW>
__global__ __launch_bounds__(NW * 64) void gemv_tile_kernel(const uint16_t* __restrict__ x,
                                                                 const uint8_t* __restrict__ qt,
                                                                 const uint8_t* __restrict__ st, void* out, int n,
                                                                 int k, int m, int ldx, int ldy, int parts,
                                                                 int spw_arg)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Lane 4 i + g takes the layout's unit i + 16 g (block 4 step + g of the tile's row i): a wave load
    // is still the whole contiguous KiB, and the four lanes of a row are neighbours, so their sum is
    // two DPP steps.
    const int i = lane >> 2, g = lane & 3;
    const int unit = i + 16 * g;
    const int steps = k >> 7, n_items = (steps + 3) >> 2, n_tiles = (n + 15) >> 4;
    const int xchunks = k >> 3;
    const int G = gridDim.x, b = blockIdx.x;
    const int tiles_wg = (n_tiles - b + G - 1) / G;
    const int spw = kRegs ? SPW : spw_arg;                           // steps per wave and tile
    const int s_begin = min(wave * spw, steps);
    const int nsteps = min(s_begin + spw, steps) - s_begin;          // 0 for the waves beyond K
    // waves that count themselves in at a tile's end: in the register form all of them (those beyond
    // K add zeros), else those that hold steps
    const int active = kRegs ? NW : (steps + spw - 1) / spw;
    const bool argmax = parts > 0;

    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                  // [MT][K / 8] chunks, natural order
    float* part = reinterpret_cast<float*>(smem + (size_t)MT * k * 2);      // [tile][MT][row 16][wave 16]
    const int tiles_cap = (n_tiles + G - 1) / G;
    float* fin = part + (size_t)tiles_cap * NW * MT * 16;              // finished outputs [tile][MT][16]
    int* cnt = reinterpret_cast<int*>(fin + (size_t)tiles_cap * MT * 16);

    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(qt), 0,
                                                                        n_tiles * steps * 1024, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(st), 0,
                                                                        n_tiles * n_items * 256, 0x00020000);
    auto valid = [&](const TPos& p) { return nsteps > 0 && p.j < tiles_wg; };
    auto advance = [&](TPos& p) {
        if (++p.s >= nsteps) {
            p.s = 0;
            ++p.j;
        }
    };
    // Always the same two loads per step: past the wave's last position the lane offset is out of the
    // descriptor's range (no memory touched, zero back).
    // Register form: two buffers (SPW odd: SPW) hold the next steps of the wave's sequence; a buffer is
    // refilled with the step that many ahead, of this tile or the next, as soon as it has been used
    // (2 KiB of a wave in flight); steps beyond the wave's range load nothing and count as zero
    // weights.  Else: two buffers walk the wave's positions.
    constexpr int kBufs = kRegs ? (SPW % 2 == 0 ? 2 : SPW) : 2;     // divides SPW: step s always uses buffer s % kBufs
    u32x4_t bq[kBufs];
    uint32_t bs[kBufs];
    auto issue_at = [&](const bool live, const int j, const int s, const int d) {
        const int tile = b + (live ? j : 0) * G;
        const int T = s_begin + s;
        bq[d] = __builtin_amdgcn_raw_buffer_load_b128(rq, live ? unit * 16 : kOobT, (tile * steps + T) * 1024, 2);
        // the step's four scale bytes of the lane's row as one dword (the four lanes of a row read the
        // same one); byte g is the lane's
        bs[d] = __builtin_amdgcn_raw_buffer_load_b32(rs, live ? i * 16 : kOobT,
                                                     (tile * n_items + (T >> 2)) * 256 + (T & 3) * 4, 0);
    };
    auto issue = [&](const TPos& p, const int d) { issue_at(valid(p), p.j, p.s, d); };

    TPos pos[2];
    TPos load{0, 0};
    if constexpr (kRegs) {
#pragma unroll
        for (int s = 0; s < kBufs; ++s) {
            issue_at(s < nsteps && tiles_wg > 0, 0, s, s);
            __builtin_amdgcn_sched_barrier(0);       // the loop's order of loads: the waits then count alike
        }
    } else {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            pos[d] = load;
            issue(load, d);
            advance(load);
        }
    }
    for (int c = tid; c < xchunks; c += NW * 64) {
#pragma unroll
        for (int r = 0; r < MT; ++r) {
            const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(x + (int64_t)min(r, m - 1) * ldx);
            xs[r * xchunks + c] = xp[c];
        }
    }
    for (int t = tid; t < tiles_cap; t += NW * 64)
        cnt[t] = 0;
    lds_barrier();

    // the chunks a lane meets in step s of its range: 4 (s_begin + s) + g, four 16-byte chunks each
    u32x4_t xr[kRegs ? MT : 1][kRegs ? SPW : 1][4];
    if constexpr (kRegs) {
#pragma unroll
        for (int r = 0; r < MT; ++r)
#pragma unroll
            for (int s = 0; s < SPW; ++s) {
                const int blk = min(4 * (s_begin + s) + g, (k >> 5) - 1);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    xr[r][s][c] = xs[r * xchunks + blk * 4 + c];
            }
    }

    float acc[MT];
    float best_val[MT];
    int best_idx[MT];
#pragma unroll
    for (int r = 0; r < MT; ++r) {
        acc[r] = 0.f;
        best_val[r] = -INFINITY;
        best_idx[r] = 0x7FFFFFFF;
    }

    // End of a tile for this wave, in two parts.  post: the four lanes of a row add up, the wave leaves
    // its 16 partial sums in the tile's slot ([MT][row 16][wave 16] floats) and lane 0 counts the wave
    // in; nothing waits.  complete, some instructions later (the counter's answer has arrived by
    // then): the wave that completed the count adds, per row, the 16 waves' partial sums in wave order
    // (64 contiguous bytes, four reads in flight) and keeps the 16 outputs, or the best of them.  A
    // wave's LDS operations are performed in order, so the partial sums are in place when the count
    // goes up.  Whoever adds, the order and therefore the value are the same.
    auto post = [&](const int j) -> int {
#pragma unroll
        for (int r = 0; r < MT; ++r) {
            float v = acc[r];
            acc[r] = 0.f;
            v += dpp_f32<0xB1>(v);                   // quad_perm [1,0,3,2]
            v += dpp_f32<0x4E>(v);                   // quad_perm [2,3,0,1]: the row's sum in its four lanes
            if (g == 0)
                part[((size_t)(j * MT + r) * 16 + i) * NW + wave] = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        int arrived = 0;
        if (lane == 0)
            arrived = __hip_atomic_fetch_add(cnt + j, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return arrived;
    };
    auto complete = [&](const int j, const int arrived_lane0) {
        if (__builtin_amdgcn_readfirstlane(arrived_lane0) != active - 1)
            return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        const int row = (b + j * G) * 16 + lane;
        if (lane < 16) {
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                const f32x4_t* pp = reinterpret_cast<const f32x4_t*>(part + ((size_t)(j * MT + r) * 16 + lane) * NW);
                f32x4_t pq[NW / 4];
#pragma unroll
                for (int c = 0; c < NW / 4; ++c)
                    pq[c] = pp[c];
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w)
                    v += w < active ? pq[w >> 2][w & 3] : 0.f;      // a wave that holds no steps never wrote its slot
                if (argmax) {
                    if (row < n && (v > best_val[r] || (v == best_val[r] && row < best_idx[r]))) {
                        best_val[r] = v;
                        best_idx[r] = row;
                    }
                } else {
                    // kept in LDS until the kernel's end: a store here would sit in front of the
                    // wave's next weight loads in the memory counter, and its acknowledgement takes
                    // longer than a tile (measured: 1.7 us per launch on the 7B LM head)
                    fin[(j * MT + r) * 16 + lane] = v;
                }
            }
        }
    };

    // step `s` of the wave's range from buffer d (register form: both constants, d = s % kBufs)
    auto compute = [&](const int s, const int d) {
        const u32x4_t wq = bq[d];
        // the convert reads only the exponent field of its scale operand (as E8M0)
        const float sc = __uint_as_float(((bs[d] >> (8 * g)) & 0xFFu) << 23);
        u32x4_t xv[MT][4];
        if constexpr (kRegs) {
#pragma unroll
            for (int r = 0; r < MT; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    xv[r][c] = xr[r][s][c];
        } else {
            const int blk = 4 * (s_begin + s) + g;
#pragma unroll
            for (int r = 0; r < MT; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    xv[r][c] = xs[r * xchunks + blk * 4 + c];
        }
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) {
            const uint32_t wd = wq[dw];                              // eight weights
            const bf16x2_t w2[4] = {__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wd, sc, 0),
                                    __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wd, sc, 1),
                                    __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wd, sc, 2),
                                    __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wd, sc, 3)};
#pragma unroll
            for (int by = 0; by < 4; ++by) {
#pragma unroll
                for (int r = 0; r < MT; ++r) {
                    // through a scalar: a bit cast applied directly to a vector element reads element 0
                    const uint32_t xd = xv[r][dw][by];
                    acc[r] = __builtin_amdgcn_fdot2_f32_bf16(w2[by], __builtin_bit_cast(bf16x2_t, xd), acc[r], false);
                }
            }
        }
    };

    if constexpr (kRegs) {
        int pending = 0;                             // lane 0: the count the wave drew for the previous tile
        for (int j = 0; j < tiles_wg; ++j) {
#pragma unroll
            for (int s = 0; s < SPW; ++s) {
                compute(s, s % kBufs);
                if (s == 0 && j > 0)
                    complete(j - 1, pending);
                // the refill leaves right behind the step that freed the buffer, not after the tile's
                // last step (left alone, the compiler sinks the multiply-adds below the loads)
#pragma unroll
                for (int r = 0; r < MT; ++r)
                    asm volatile("" : "+v"(acc[r])::"memory");
                __builtin_amdgcn_sched_barrier(0);
                // the step kBufs ahead: of this tile, or of the next
                const int sn = s + kBufs < SPW ? s + kBufs : s + kBufs - SPW;
                const int jn = s + kBufs < SPW ? j : j + 1;
                issue_at(sn < nsteps && jn < tiles_wg, jn, sn, s % kBufs);
                __builtin_amdgcn_sched_barrier(0);
            }
            pending = post(j);
        }
        if (tiles_wg > 0)
            complete(tiles_wg - 1, pending);
    } else {
        // Every trip issues the same loads whether or not buffer 1 still had work, so that every
        // path into the loop head carries the same queue of outstanding loads.
        while (valid(pos[0])) {
#pragma unroll
            for (int d = 0; d < 2; ++d) {
                if (d == 0 || valid(pos[d])) {
                    compute(pos[d].s, d);
                    if (pos[d].s == nsteps - 1)
                        complete(pos[d].j, post(pos[d].j));
                }
                pos[d] = load;
                issue(load, d);
                advance(load);
            }
        }
    }

    if (!argmax) {
        // every tile of the workgroup has been finished by one of its waves: store them all
        __syncthreads();
        for (int o = tid; o < tiles_wg * MT * 16; o += NW * 64) {
            const int j = o / (MT * 16), r = (o >> 4) % MT, row = (b + j * G) * 16 + (o & 15);
            if (row < n)
                static_cast<uint16_t*>(out)[(int64_t)r * ldy + row] = f32_to_bf16_rne(fin[o]);
        }
    }
    if (argmax) {
        // the finishing waves hold candidates in lanes 0..15: best of the wave, then of the workgroup
#pragma unroll
        for (int r = 0; r < MT; ++r) {
            for (int o = 32; o > 0; o >>= 1) {
                const float v = __shfl_xor(best_val[r], o);
                const int ix = __shfl_xor(best_idx[r], o);
                if (v > best_val[r] || (v == best_val[r] && ix < best_idx[r])) {
                    best_val[r] = v;
                    best_idx[r] = ix;
                }
            }
        }
        __syncthreads();
        float* wval = reinterpret_cast<float*>(smem);
        int* widx = reinterpret_cast<int*>(smem) + NW * MT;
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                wval[wave * MT + r] = best_val[r];
                widx[wave * MT + r] = best_idx[r];
            }
        }
        __syncthreads();
        if (tid < MT && tid < m) {
            float bv = wval[tid];
            int bi = widx[tid];
            for (int w = 1; w < NW; ++w) {
                const float v = wval[w * MT + tid];
                const int ix = widx[w * MT + tid];
                if (v > bv || (v == bv && ix < bi)) {
                    bv = v;
                    bi = ix;
                }
            }
            float* part_val = static_cast<float*>(out);
            int32_t* part_idx = reinterpret_cast<int32_t*>(part_val + (int64_t)m * parts);
            part_val[(int64_t)tid * parts + b] = bv;
            part_idx[(int64_t)tid * parts + b] = bi;
        }
    }
}

size_t gemv_tile_lds(int mt, int n, int k, int blocks, int nw = kWavesT)
{
    const int n_tiles = (n + 15) / 16;
    const int tiles_cap = (n_tiles + blocks - 1) / blocks;
    return (size_t)mt * k * 2 + (size_t)tiles_cap * (nw * mt * 16 * 4 + mt * 64 + 4);
}

int gemv_tile_blocks(int n, const DeviceInfo& dev)
{
    const int n_tiles = (n + 15) / 16;
    return n_tiles < dev.cus ? n_tiles : dev.cus;
}

template <int MT, int SPW, bool kRegs, int NW = kWavesT>
hipError_t launch_k(const GemmArgs& a, int blocks, size_t lds, int spw, int max_lds, hipStream_t stream)
{
    auto kern = gemv_tile_kernel<MT, SPW, kRegs, NW>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (lds > 64 * 1024)
        if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), max_lds); e != hipSuccess)
            return e;
    const bool argmax = a.part_val != nullptr;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, stream, a.x, a.q, a.s,
                       argmax ? static_cast<void*>(a.part_val) : static_cast<void*>(a.y), a.n, a.k, a.m, (int)a.ldx,
                       (int)a.ldy, argmax ? a.parts : 0, spw);
    return hipGetLastError();
}

template <int MT>
hipError_t launch_mt(const GemmArgs& a, int blocks, size_t lds, int max_lds, hipStream_t stream)
{
    // K of 61 to 72 steps (K = 8192): 12 waves of six steps in registers, 9.94 -> 9.67 us on 8192 x 8192 and
    // 47.8 -> 44.3 on 57344 x 8192 against 16 waves of four; at K = 4096 16 waves stay ahead of 12 and 8
    // (7.4 / 7.8 / 8.9 us on the 7B qkv projection).
    if constexpr (MT == 1) {
        if ((a.k / 128 + 11) / 12 == 6)
            return launch_k<MT, 6, true, 12>(a, blocks, lds, 6, max_lds, stream);
    }
    const int spw = (a.k / 128 + kWavesT - 1) / kWavesT;
    switch (spw) {
    case 1:
        return launch_k<MT, 1, true>(a, blocks, lds, spw, max_lds, stream);
    case 2:
        return launch_k<MT, 2, true>(a, blocks, lds, spw, max_lds, stream);
    case 3:
        if constexpr (MT == 1)                      // two rows of three steps spill
            return launch_k<MT, 3, true>(a, blocks, lds, spw, max_lds, stream);
        break;
    case 4:
        if constexpr (MT == 1)
            return launch_k<MT, 4, true>(a, blocks, lds, spw, max_lds, stream);
        break;
    }                                                // (six steps in registers spill: 11.3 against 8.2 us on the 7B down projection)
    return launch_k<MT, 1, false>(a, blocks, lds, spw, max_lds, stream);
}

}  // namespace

// One or two activation rows, K a multiple of 128, the workgroup's LDS holds the activation rows and
// a slot of partial sums per tile it owns.  a.q and a.s are the tile-major tensors.
bool gemv_tile_can_run(const GemmArgs& a, const DeviceInfo& dev)
{
    if (a.m < 1 || a.m > 2 || a.k % 128 != 0 || a.n < 1)
        return false;
    const int blocks = gemv_tile_blocks(a.n, dev);
    return gemv_tile_lds(a.m, a.n, a.k, blocks) + 512 <= (size_t)dev.lds_bytes && blocks <= gemv_max_parts(dev);
}

hipError_t launch_gemv_tile(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    const int blocks = gemv_tile_blocks(a.n, dev);
    size_t lds = gemv_tile_lds(a.m, a.n, a.k, blocks);
    if (lds < 512)
        lds = 512;                                  // the argmax combine needs a few bytes
    if (parts_used)
        *parts_used = blocks;
    return a.m == 2 ? launch_mt<2>(a, blocks, lds, dev.lds_bytes, stream)
                    : launch_mt<1>(a, blocks, lds, dev.lds_bytes, stream);
}

}  // namespace mxfp4
