// A chain of dependent one-token products in one persistent launch (arXiv 2503.13565, section
// 3.2: a decode step is bound by streaming the model's weights in; section 3.4.3 and Eq. 2 for the
// product itself; section 4.4: the product with one token must run at memory speed).
//
// The linear layers of a decode step read each other's outputs, so they cannot run side by side;
// launched one by one, each pays the gap between launches, the latency of its first data and its
// tail, which together cost as much as streaming the weights does.  Here one workgroup per compute
// unit stays resident for the whole chain.  Link p + 1 starts when every workgroup has published
// its part of link p's output (a grid-wide barrier), but only its activations depend on link p:
// every compute wave keeps kD weight loads in flight across the barrier, so the memory system
// streams the next link's weights while the barrier, the broadcast of the new activation row and
// its staging in LDS take place.
//
// Roles.  Waves 0 .. kCompute - 1 of a workgroup stream and multiply.  A compute wave walks a flat
// sequence of steps (link, weight row, 64 scale blocks of that row); step f uses ring slot f % kD of
// its registers and, once consumed, reloads it with step f + kD, whatever link that step belongs
// to.  Decode and multiply-add per step are those of the single-call decode kernel (scaled
// FP4->BF16 convert with the block's scale, v_dot2_f32_bf16, FP32 accumulation, fixed-order wave
// sum), so a link's outputs have the bits of the single call.  The last wave is the service wave:
// it never loads weights.  Per link it takes the finished row sums from LDS, applies the epilogue,
// publishes the outputs with device-scope stores, signals the workgroup's arrival, waits for all
// the others, fetches the next activation row (device-scope loads) into LDS and releases the
// compute waves.  Two workgroup barriers per link keep the two roles in step; they wait for LDS
// traffic only, never for the weight loads in flight.
//
// Grid barrier.  Workgroup b publishes flag[b] = epoch (a device-scope store behind a drain of its
// output stores).  Workgroup 0 polls all flags and then publishes one `go` word that the others
// poll: two memory round trips, 1.9 us measured for 256 workgroups, against 2.7 us when every
// workgroup polls every flag and 3.6 to 3.9 us for one atomic counter.  Epochs only grow (every
// launch adds its link count to every flag), so nothing is ever reset and a launch can be replayed
// from a graph; a workgroup learns the current epoch from its own flag.  Every wait is bounded by
// the clock: when the bound expires the workgroup writes a status word, releases its compute
// waves with an abort mark and all waves end normally; the status is sticky until the caller
// re-initialises the workspace.
#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

namespace {

constexpr int kWaves = 16;                // of a workgroup
constexpr int kCompute = kWaves - 1;      // waves that stream weights
#ifndef MXFP4_CHAIN_D
#define MXFP4_CHAIN_D 8
#endif
constexpr int kD = MXFP4_CHAIN_D;         // weight steps in flight per compute wave
constexpr int kSc1 = 16;                  // cache policy of buffer instructions: device scope
constexpr int kGroup = 16;                // consecutive weight rows dealt to a workgroup at a time
constexpr int kBatch = 24;                // 16-byte loads in flight per lane when an activation row is fetched
constexpr int kOut = 0x7FFFFFF0;          // a lane offset beyond every descriptor: touches no memory

// workspace (32-bit words): flags, then the go word and the status word in lines of their own,
// then the partial winners of the fused pick; behind these 16 KB, scratch for a pick that the
// caller's mode sends to the ordinary two-launch form
constexpr int kFlagWords = 1024;
constexpr int kGoWord = 1024;
constexpr int kStatusWord = 1056;
constexpr int kPartValWord = 2048;
constexpr int kPartIdxWord = 3072;
constexpr size_t kSyncBytes = 16384;       // flags, go and status words, partial winners
constexpr size_t kWorkspaceBytes = 65536;  // + the scratch of a pick that runs as launches of its own

struct ChainLink {
    const uint8_t* q;
    const uint8_t* s;
    const uint16_t* x;
    uint16_t* y;                // null: the fused pick (last link only)
    const uint16_t* bias;
    const uint16_t* residual;
    int n, k;
    int act;
    int rot;                    // weight rows dealt to the waves before this link, modulo kCompute
    int chunk;                  // most weight rows of the link in one workgroup
    int pad;
};
static_assert(sizeof(ChainLink) == 72, "kernel argument layout");
static_assert(kStatusWord * 4 == MXFP4_CHAIN_STATUS_OFFSET, "the header names the status word's place");

struct ChainArgs {
    uint32_t* ws;
    int32_t* argmax_out;
    float* max_out;
    int count;
    int wait_ticks;             // bound of one wait, in ticks of the 100 MHz clock
    int phantom;                // test only: flags beyond the grid that no workgroup ever sets
    int x_chunks;               // 16-byte chunks of the activation buffer in LDS
    ChainLink links[kChainMaxLinks];
};

struct Cursor {
    int p, row, t;              // link, index of the weight row among the workgroup's, step within the row
    int steps, nblk, cnt;       // cnt: weight rows of the link that belong to this workgroup
    bool pick, gated;
    __amdgpu_buffer_rsrc_t rq, rs;
};

__global__ __launch_bounds__(kWaves * 64) void chain_kernel(const ChainArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.x, G = gridDim.x;

    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                     // [step][j][lane] chunks
    float* ybuf = reinterpret_cast<float*>(xs + a.x_chunks);            // row sums of the link, [chunk]
    float* wbv = ybuf + kChainMaxChunk;                                 // the waves' winners
    int* wbi = reinterpret_cast<int*>(wbv + kWaves);
    int* abort_mark = wbi + kWaves;

    // Weight rows are dealt to the workgroups in groups of kGroup consecutive rows, round robin (group
    // g G + b is the g-th of workgroup b): all workgroups sweep through a link's weights side by side,
    // and a workgroup's outputs, bias and residual values come in runs of kGroup.  (One contiguous run
    // of all its rows per workgroup: the workgroups finished a link up to 4 us apart and the stream
    // ran at half the speed.  Single rows round robin: every 2-byte access of the service wave hits a
    // cache line of its own, 1.4 us to store a link's outputs.)  A gate pair never straddles groups.
    auto rows_of = [&](int n, bool) {
        const int groups = (n + kGroup - 1) / kGroup;
        if (b >= groups)
            return 0;
        const int mine = (groups - b + G - 1) / G;
        const bool owns_last = (groups - 1) % G == b;
        return mine * kGroup - (owns_last ? groups * kGroup - n : 0);
    };
    auto global_row = [&](int r, bool) { return ((r / kGroup) * G + b) * kGroup + r % kGroup; };
    auto load_link = [&](Cursor& c, int p) {
        const ChainLink& L = a.links[p];
        c.p = p;
        c.nblk = L.k >> 5;
        c.steps = (c.nblk + 63) >> 6;
        c.gated = L.act == MXFP4_ACT_SWIGLU;
        c.cnt = rows_of(L.n, c.gated);
        c.pick = L.y == nullptr;
        const int r = wave - L.rot;
        c.row = r < 0 ? r + kCompute : r;
        c.t = 0;
        c.rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(L.q), 0, L.n * c.nblk * 16, 0x00020000);
        c.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(L.s), 0, L.n * c.nblk, 0x00020000);
    };

    if (wave < kCompute) {
        // ---- compute wave ----------------------------------------------------------------------
        u32x4_t bq[kD];
        uint32_t bs[kD];
        Cursor I, C;
        load_link(I, 0);
        while (I.row >= I.cnt) {                    // no rows of this link for this wave
            if (I.p + 1 >= a.count) {
                I.p = a.count;
                break;
            }
            load_link(I, I.p + 1);
        }
        // A step always issues the same two loads, so that the in-order load counter can be waited
        // on exactly; past the end of the chain, or of a ragged K, the lane offset leaves the
        // descriptor's range: such loads touch no memory and return zero.
        // The loads are issued and waited for by hand (inline assembly).  With compiler-tracked
        // loads the wait in front of the loop's first slot came out as "all loads" (the state merged
        // at the loop header), which empties the ring once per turn.  A slot's registers are written
        // by the load and handed to the compiler only by the wait that follows kD - 1 steps later.
        auto issue = [&](int d) {
            const bool live = I.p < a.count;
            const bool vb = I.t * 64 + lane < I.nblk;
            const int grow = global_row(I.row, I.gated);
            asm volatile("buffer_load_dwordx4 %0, %2, %4, %5 offen nt\n\t"
                         "buffer_load_dword %1, %3, %6, %7 offen"
                         : "=&v"(bq[d]), "=&v"(bs[d])
                         : "v"((live && vb) ? lane * 16 : kOut), "v"(live ? (lane & 15) * 4 : kOut), "s"(I.rq),
                           "s"(grow * (I.nblk * 16) + I.t * 1024), "s"(I.rs), "s"(grow * I.nblk + I.t * 64)
                         : "memory");
            if (live && ++I.t == I.steps) {
                I.t = 0;
                I.row += kCompute;
                while (I.row >= I.cnt) {
                    if (I.p + 1 >= a.count) {
                        I.p = a.count;
                        break;
                    }
                    load_link(I, I.p + 1);
                }
            }
        };
#pragma unroll
        for (int d = 0; d < kD; ++d)
            issue(d);

        lds_barrier();                              // the first activation row is staged
        bool stop = __builtin_amdgcn_readfirstlane(*abort_mark) != 0;   // (uniform: scalar branches)
        load_link(C, 0);

        float acc = 0.f;
        float best_val = -INFINITY;
        int best_idx = 0x7FFFFFFF;
        const int sh_top = (3 - (lane & 3)) * 8;    // brings this lane's scale byte to bits 31:24
        while (!stop) {
#pragma unroll
            for (int d = 0; d < kD; ++d) {
                // the wave has no (more) rows in link C.p: hand the link over, take the next one
                while (!stop && C.row >= C.cnt) {
                    if (C.pick && lane == 0) {
                        wbv[wave] = best_val;
                        wbi[wave] = best_idx;
                    }
                    lds_barrier();                  // this workgroup's part of the link is in LDS
                    if (C.p + 1 >= a.count) {
                        stop = true;
                        break;
                    }
                    lds_barrier();                  // the next activation row is staged
                    stop = __builtin_amdgcn_readfirstlane(*abort_mark) != 0;
                    load_link(C, C.p + 1);
                }
                if (stop)
                    break;
                // step by step: a slot's reload goes out when the slot has been consumed, into the
                // same registers (a reload hoisted above its slot's last use would need other
                // registers, and copies at the loop's end that wait for every load in flight)
                __builtin_amdgcn_sched_barrier(0);
                // two loads per step: the slot's pair has landed when at most 2 (kD - 1) are in flight
                asm volatile("s_waitcnt vmcnt(%2)" : "+v"(bq[d]), "+v"(bs[d]) : "n"(2 * (kD - 1)) : "memory");
                const uint32_t dw = (uint32_t)__builtin_amdgcn_ds_bpermute((lane >> 2) * 4, (int)bs[d]);
                float sc = __uint_as_float((dw << sh_top) >> 1);
                sc = (C.t * 64 + lane < C.nblk) ? sc : 1.0f;         // no NaN from a neighbour's scale byte
                const u32x4_t* xb = xs + C.t * 256 + lane;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u32x4_t xv = xb[j * 64];
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
                // (the sum is pinned here: code motion across blocks would otherwise sink the whole
                // multiply-add chain below the reload and the cursor's branches)
                asm volatile("" : "+v"(acc) : : "memory");
                __builtin_amdgcn_sched_barrier(0);
                issue(d);
                if (++C.t == C.steps) {
                    const float v = wave_sum(acc);
                    acc = 0.f;
                    if (C.pick) {
                        const int grow = global_row(C.row, false);      // the lower index wins among equal values
                        if (v > best_val || (v == best_val && grow < best_idx)) {
                            best_val = v;
                            best_idx = grow;
                        }
                    } else if (lane == 0) {
                        ybuf[C.row] = v;
                    }
                    C.t = 0;
                    C.row += kCompute;
                }
            }
        }
        return;
    }

    // ---- service wave --------------------------------------------------------------------------
    __builtin_amdgcn_s_setprio(3);
    const __amdgpu_buffer_rsrc_t rws = __builtin_amdgcn_make_buffer_rsrc(a.ws, 0, (int)kSyncBytes, 0x00020000);
    const int n_flags = G + a.phantom;
    const uint32_t base = __builtin_amdgcn_raw_buffer_load_b32(rws, b * 4, 0, kSc1);
    const uint32_t status0 = __builtin_amdgcn_raw_buffer_load_b32(rws, kStatusWord * 4, 0, kSc1);

    // activation row of link p -> LDS: 16-byte chunk c of the row (8 elements: quarter c % 4 of scale
    // block c / 4) goes to [step][quarter][block % 64]; zeros behind the row's end
    auto stage_x = [&](int p) {
        const ChainLink& L = a.links[p];
        const int chunks = L.k >> 3;
        const int steps = ((L.k >> 5) + 63) >> 6;
        const __amdgpu_buffer_rsrc_t rx =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(L.x), 0, L.k * 2, 0x00020000);
        auto slot = [](int c) { return (((c >> 8) * 4 + (c & 3)) << 6) + ((c >> 2) & 63); };
        constexpr int kB = kBatch;                  // loads in flight per lane: a row of 12288 elements at once
        for (int c0 = 0; c0 < chunks; c0 += 64 * kB) {
            u32x4_t v[kB];
#pragma unroll
            for (int u = 0; u < kB; ++u)            // past the end: zero
                v[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, (c0 + u * 64 + lane) * 16, 0, kSc1);
#pragma unroll
            for (int u = 0; u < kB; ++u) {
                const int c = c0 + u * 64 + lane;
                if (c < steps * 256)
                    xs[slot(c)] = v[u];
            }
        }
        for (int c = (chunks + 64 * kBatch - 1) / (64 * kBatch) * (64 * kBatch) + lane; c < steps * 256; c += 64)
            xs[slot(c)] = u32x4_t{0, 0, 0, 0};
    };
    // wait until every workgroup has published `epoch` (workgroup 0: all flags, then the go word;
    // the others: the go word); false when the clock bound expires first
    auto wait_epoch = [&](uint32_t epoch, bool all_flags) {
        const uint64_t t0 = __builtin_amdgcn_s_memrealtime();
        for (;;) {
            bool ok = true;
            if (all_flags) {
                for (int f0 = 0; f0 < n_flags; f0 += 256) {
                    const u32x4_t f = __builtin_amdgcn_raw_buffer_load_b128(rws, (f0 + lane * 4) * 4, 0, kSc1);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        ok = ok && (f0 + lane * 4 + j >= n_flags || (int)(f[j] - epoch) >= 0);
                }
            } else {
                const uint32_t g = __builtin_amdgcn_raw_buffer_load_b32(rws, kGoWord * 4, 0, kSc1);
                ok = (int)(g - epoch) >= 0;
            }
            if (__builtin_amdgcn_ballot_w64(ok) == ~0ull)
                return true;
            if ((int64_t)(__builtin_amdgcn_s_memrealtime() - t0) > (int64_t)a.wait_ticks)
                return false;
            __builtin_amdgcn_s_sleep(1);
        }
    };

#ifdef MXFP4_CHAIN_TRACE
    // measurement build only: time stamps (10 ns ticks) of the service wave's stages per link, in
    // the memory behind the workspace proper: [workgroup][link][8]
    auto stamp = [&](int p, int i) {
        if (lane == 0)
            a.ws[kWorkspaceBytes / 4 + (b * kChainMaxLinks + p) * 8 + i] = (uint32_t)__builtin_amdgcn_s_memrealtime();
    };
#else
    auto stamp = [](int, int) {};
#endif
    bool aborted = status0 != 0;                    // an earlier launch on this workspace gave up
    if (lane == 0)
        *abort_mark = aborted ? 1 : 0;
    if (!aborted)
        stage_x(0);
    lds_barrier();                                  // the first activation row is staged
    if (aborted)
        return;

    for (int p = 0; p < a.count; ++p) {
        const ChainLink& L = a.links[p];
        const bool gated = L.act == MXFP4_ACT_SWIGLU;
        const int cnt = rows_of(L.n, gated);
        const bool last = p + 1 == a.count;
        const bool epi = gated || L.bias || L.residual;
        const int cols = gated ? L.n >> 1 : L.n;
        const int units = gated ? cnt >> 1 : cnt;   // outputs of this workgroup
        // column of the workgroup's u-th output (a gated output is a pair of rows)
        auto col_of = [&](int u) { return gated ? global_row(2 * u, true) >> 1 : global_row(u, false); };
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(L.bias), 0, L.bias ? L.n * 2 : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(L.residual), 0, L.residual ? cols * 2 : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(L.y, 0, L.y ? cols * 2 : 0, 0x00020000);
        // a link's bias and residual do not depend on its row sums: those of the first kPre outputs
        // per lane are fetched before the link's rows are awaited (absent operands: descriptors of
        // size zero, the loads return zero)
        constexpr int kPre = 4;
        uint32_t e_b0[kPre], e_b1[kPre], e_r[kPre];
        auto fetch_operands = [&](int u, uint32_t& b0, uint32_t& b1, uint32_t& r) {
            const int col = col_of(u);
            const int row = gated ? 2 * col : col;
            b0 = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rb, u < units ? row * 2 : kOut, 0, kSc1);
            b1 = gated ? (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rb, u < units ? row * 2 + 2 : kOut, 0, kSc1) : 0u;
            r = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rr, u < units ? col * 2 : kOut, 0, kSc1);
        };
        if (epi) {
#pragma unroll
            for (int i = 0; i < kPre; ++i)
                fetch_operands(lane + 64 * i, e_b0[i], e_b1[i], e_r[i]);
        }

        stamp(p, 0);
        lds_barrier();                              // this workgroup's part of link p is in LDS
        stamp(p, 1);
        if (L.y) {
            auto finish = [&](int u, uint32_t b0, uint32_t b1, uint32_t r) {
                if (u >= units)
                    return;
                const int col = col_of(u);
                float v;
                if (gated) {
                    const float g = ybuf[2 * u] + bf16_bits_to_f32(b0), up = ybuf[2 * u + 1] + bf16_bits_to_f32(b1);
                    v = silu_gate(g, up) + bf16_bits_to_f32(r);
                } else {
                    v = ybuf[u];
                    if (epi)
                        v = (v + bf16_bits_to_f32(b0)) + bf16_bits_to_f32(r);
                }
                __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16_rne(v), ry, col * 2, 0, kSc1);
            };
#pragma unroll
            for (int i = 0; i < kPre; ++i)
                finish(lane + 64 * i, epi ? e_b0[i] : 0u, epi ? e_b1[i] : 0u, epi ? e_r[i] : 0u);
            for (int u = lane + 64 * kPre; u < units; u += 64) {
                uint32_t b0 = 0, b1 = 0, r = 0;
                if (epi)
                    fetch_operands(u, b0, b1, r);
                finish(u, b0, b1, r);
            }
        } else {
            // the fused pick: this workgroup's winner among its waves
            float bv = lane < kCompute ? wbv[lane] : -INFINITY;
            int bi = lane < kCompute ? wbi[lane] : 0x7FFFFFFF;
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) {
                const float v = __shfl_xor(bv, off);
                const int i = __shfl_xor(bi, off);
                if (v > bv || (v == bv && i < bi)) {
                    bv = v;
                    bi = i;
                }
            }
            if (lane == 0) {
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(bv), rws, (kPartValWord + b) * 4, 0, kSc1);
                __builtin_amdgcn_raw_buffer_store_b32((uint32_t)bi, rws, (kPartIdxWord + b) * 4, 0, kSc1);
            }
        }
        stamp(p, 2);
        drain_vmem();                               // the outputs have left before the flag does
        stamp(p, 3);
        const uint32_t epoch = base + (uint32_t)p + 1u;
        if (lane == 0)
            __builtin_amdgcn_raw_buffer_store_b32(epoch, rws, b * 4, 0, kSc1);
        if (last) {
            if (!L.y && b == 0) {
                // second stage of the pick: the lowest index among the largest accumulators
                if (!wait_epoch(epoch, true)) {
                    if (lane == 0)
                        __builtin_amdgcn_raw_buffer_store_b32(0x100u + (uint32_t)p, rws, kStatusWord * 4, 0, kSc1);
                    return;
                }
                float bv = -INFINITY;
                int bi = 0x7FFFFFFF;
                for (int w = lane; w < G; w += 64) {
                    const float v = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rws, (kPartValWord + w) * 4, 0, kSc1));
                    const int i = (int)__builtin_amdgcn_raw_buffer_load_b32(rws, (kPartIdxWord + w) * 4, 0, kSc1);
                    if (v > bv || (v == bv && i < bi)) {
                        bv = v;
                        bi = i;
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
                    a.argmax_out[0] = bi == 0x7FFFFFFF ? 0 : bi;
                    if (a.max_out)
                        a.max_out[0] = bv;
                }
            }
            return;
        }
        bool ok = wait_epoch(epoch, b == 0);
        if (ok && b == 0 && lane == 0)
            __builtin_amdgcn_raw_buffer_store_b32(epoch, rws, kGoWord * 4, 0, kSc1);
        stamp(p, 4);
        if (!ok) {
            if (lane == 0) {
                __builtin_amdgcn_raw_buffer_store_b32(0x100u + (uint32_t)p, rws, kStatusWord * 4, 0, kSc1);
                *abort_mark = 1;
            }
        } else {
            stage_x(p + 1);
        }
        stamp(p, 5);
        lds_barrier();                              // the next activation row is staged (or the abort mark set)
        stamp(p, 6);
        if (!ok)
            return;
    }
}

__global__ __launch_bounds__(256) void chain_ws_init_kernel(uint32_t* ws, int words)
{
    for (int i = blockIdx.x * 256 + threadIdx.x; i < words; i += gridDim.x * 256)
        ws[i] = 0;
}

}  // namespace

size_t chain_workspace_bytes() { return kWorkspaceBytes; }
size_t chain_pick_area_offset() { return kSyncBytes; }

hipError_t launch_chain_ws_init(void* ws, hipStream_t stream)
{
    hipLaunchKernelGGL(chain_ws_init_kernel, dim3(4), dim3(256), 0, stream, static_cast<uint32_t*>(ws),
                       (int)(kSyncBytes / 4));
    return hipGetLastError();
}

static int chain_steps(int k) { return ((k >> 5) + 63) >> 6; }

// most weight rows of a link that one workgroup gets (whole groups of kGroup rows)
static int chain_rows_per_workgroup(int n, int, int workgroups)
{
    const int groups = (n + kGroup - 1) / kGroup;
    return (groups + workgroups - 1) / workgroups * kGroup;
}

bool chain_can_run(const ChainItem* items, int count, const DeviceInfo& dev)
{
    if (count < 1 || dev.cus > kFlagWords)
        return false;
    size_t x_bytes = 0;
    for (int i = 0; i < count; ++i) {
        const ChainItem& it = items[i];
        if (it.k % 128 != 0 || it.k < 128 || it.n < 1)
            return false;
        if (!it.y && (i != count - 1 || it.bias || it.residual || it.act != MXFP4_ACT_NONE))
            return false;                           // the pick ends a chain and takes no epilogue
        if (it.act == MXFP4_ACT_SWIGLU && it.n % 2 != 0)
            return false;
        const int chunk = chain_rows_per_workgroup(it.n, it.act, dev.cus);
        if (chunk > kChainMaxChunk)
            return false;
        x_bytes = max(x_bytes, (size_t)chain_steps(it.k) * 4096);
    }
    return x_bytes + kChainMaxChunk * 4 + 256 <= (size_t)dev.lds_bytes;
}

hipError_t launch_chain(const ChainItem* items, int count, const DeviceInfo& dev, void* ws, int wait_ticks,
                        int phantom, hipStream_t stream)
{
    if (!chain_can_run(items, count, dev) || phantom < 0 || dev.cus + phantom > kFlagWords)
        return hipErrorInvalidValue;
    static LdsLimit lds_limit;
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(chain_kernel), 160 * 1024); e != hipSuccess)
        return e;
    // the grid barrier needs every workgroup resident: one per compute unit must fit
    {
        size_t worst = 0;
        for (int i = 0; i < count; ++i)
            worst = max(worst, (size_t)chain_steps(items[i].k) * 4096);
        int per_cu = 0;
        if (hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, chain_kernel, kWaves * 64,
                                                                        worst + kChainMaxChunk * 4 + 256);
            e != hipSuccess)
            return e;
        if (per_cu < 1)
            return hipErrorLaunchOutOfResources;
    }
    int rot = 0;
    for (int i0 = 0; i0 < count; i0 += kChainMaxLinks) {
        const int c = min(kChainMaxLinks, count - i0);
        ChainArgs a{};
        a.ws = static_cast<uint32_t*>(ws);
        a.count = c;
        a.wait_ticks = wait_ticks;
        a.phantom = phantom;
        size_t x_bytes = 0;
        for (int i = 0; i < c; ++i) {
            const ChainItem& it = items[i0 + i];
            ChainLink& L = a.links[i];
            L.q = it.q;
            L.s = it.s;
            L.x = it.x;
            L.y = it.y;
            L.bias = it.bias;
            L.residual = it.residual;
            L.n = it.n;
            L.k = it.k;
            L.act = it.act;
            L.chunk = chain_rows_per_workgroup(it.n, it.act, dev.cus);
            L.rot = rot;
            rot = (rot + L.chunk) % kCompute;
            if (!it.y) {
                a.argmax_out = it.argmax_out;
                a.max_out = it.max_out;
            }
            x_bytes = max(x_bytes, (size_t)chain_steps(it.k) * 4096);
        }
        a.x_chunks = (int)(x_bytes / 16);
        const size_t lds = x_bytes + kChainMaxChunk * 4 + 256;
        hipLaunchKernelGGL(chain_kernel, dim3(dev.cus), dim3(kWaves * 64), lds, stream, a);
        if (hipError_t e = hipGetLastError(); e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

}  // namespace mxfp4
