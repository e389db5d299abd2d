// The unquantised counterpart: y = x * W^T with BF16 weights, for the few activation rows of a
// decode or verification step (arXiv 2503.13565, section 3.2: the target model verifies in BF16;
// section 3.4.3: its 2 bytes per weight are what the 0.53 bytes of MXFP4 are measured against,
// the 3.76x of the paper).  Same boundary conventions and the same pipeline discipline as the
// MXFP4 GEMV: a wave walks groups of R weight rows, one 16-byte load per lane and row (8 weights,
// 1 KiB contiguous per wave instruction), activations staged once per workgroup in LDS,
// v_dot2_f32_bf16 with FP32 accumulation, DPP reduction at the end of a row group, outputs held
// one per lane and stored 64 at a time.  At 2 bytes per weight the vector ALUs keep up with the
// memory system for up to 8 activation rows per pass (4 dot2 per 16 bytes and row), so no matrix
// core path is needed; more rows take more passes.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

namespace {

constexpr int kSentinelB = 0x7FFFFFF0;   // lane offset beyond any descriptor: the load returns zero

struct BPos {
    int g;      // row group
    int t;      // step along K (64 chunks of 8 elements per step)
};

__device__ __forceinline__ void lds_barrier_b()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// MT activation rows per pass, R weight rows per group, NW waves per workgroup; two register
// buffers of one step each.
template <int MT, int R, int NW>
__global__ __launch_bounds__(NW * 64) void bf16_gemv_kernel(Bf16Args a, int m0)
{
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                  // [MT][K / 8] chunks
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int chunks = a.k >> 3;
    const int steps = (chunks + 63) >> 6;
    const int tail = chunks - (steps - 1) * 64;                      // chunks in the last step (1..64)
    const int n_groups = (a.n + R - 1) / R;
    const int total_waves = gridDim.x * NW;
    const int first_group = (int)blockIdx.x * NW + wave;
    const int row_bytes = (int)a.ldw * 2;
    const bool argmax = a.part_val != nullptr;

    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(a.w), 0, (int)((a.n - 1) * a.ldw + a.k) * 2, 0x00020000);

    auto valid = [&](const BPos& p) { return p.g < n_groups; };
    auto advance = [&](BPos& p) {
        if (++p.t == steps) {
            p.t = 0;
            p.g += total_waves;
        }
    };
    // Always R loads per step: past the wave's last position, and for the lanes beyond a ragged
    // last step, the lane offset is out of the descriptor's range (no memory touched, zero back).
    auto issue = [&](const BPos& p, u32x4_t (&w)[R]) {
        const bool live = valid(p) && (p.t < steps - 1 || lane < tail);
        const int voff = live ? lane * 16 : kSentinelB;
        const int g = valid(p) ? p.g : 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = min(g * R + r, a.n - 1);                  // ragged N: re-read the last row
            w[r] = __builtin_amdgcn_raw_buffer_load_b128(rw, voff, row * row_bytes + p.t * 1024, 2);
        }
    };

    // Prologue: activation loads first, weight loads right behind them; only the activations are
    // waited for before the LDS copy.
    u32x4_t buf[2][R];
    BPos pos[2];
    BPos load{first_group, 0};
    {
        constexpr int T = NW * 64;
        constexpr int kSlots = MT >= 8 ? 1 : 8 / MT;                 // 8 activation loads in flight per batch
        u32x4_t xr[MT][kSlots];
        auto x_load = [&](int c0) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const int msrc = min(m0 + m, a.m - 1);               // ragged M: repeat the last row
                const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
#pragma unroll
                for (int i = 0; i < kSlots; ++i)
                    xr[m][i] = xp[min(c0 + i * T, chunks - 1)];
            }
        };
        auto x_store = [&](int c0) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int i = 0; i < kSlots; ++i)
                    xs[m * chunks + min(c0 + i * T, chunks - 1)] = xr[m][i];   // clamped duplicates rewrite the same data
        };
        x_load(tid);
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            pos[d] = load;
            issue(load, buf[d]);
            advance(load);
        }
        x_store(tid);
        for (int c0 = tid + kSlots * T; c0 < chunks; c0 += kSlots * T) {   // long rows: the rest, batch by batch
            x_load(c0);
            x_store(c0);
        }
    }
    lds_barrier_b();

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

    // Stores and loads share one completion counter but complete out of order with respect to
    // each other, so the counter is drained after the stores; the main loop only sees loads.
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
        __builtin_amdgcn_s_waitcnt(0x0F70);                          // vmcnt(0), other counters untouched
    };

    auto compute = [&](const BPos& p, const u32x4_t (&w)[R]) {
        const int c = min(p.t * 64 + lane, chunks - 1);               // beyond the tail the weights are zero
        u32x4_t xv[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m)
            xv[m] = xs[m * chunks + c];
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t wd = w[r][j];                          // (a bit cast needs a plain object,
#pragma unroll                                                        //  not a vector element)
                for (int m = 0; m < MT; ++m) {
                    const uint32_t xd = xv[m][j];
                    acc[r][m] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, wd),
                                                                __builtin_bit_cast(bf16x2_t, xd), acc[r][m], false);
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

// The decode step (one activation row) in the frame of the MXFP4 register GEMV: one workgroup of
// 16 waves per compute unit; the activation row staged once through LDS and then held in
// registers (a lane owns elements [8 lane, 8 lane + 8) of every 512-element step); weight rows
// dealt to the waves through an LDS counter, fetched one row ahead; D steps of 1 KiB per wave in
// flight; every step issues the same loads (a lane past a ragged K, or a wave out of rows, reads
// through an offset outside the descriptor: no memory touched, zero back), so the in-order load
// counter is waited on exactly; scalar, preloaded kernel arguments.
// NS: steps per row the instance is unrolled for (K <= 512 NS), a multiple of D.
template <int NS, int D, int NW>
__global__ __launch_bounds__(NW * 64) void bf16_reg_kernel(const uint16_t* __restrict__ x,
                                                           const uint16_t* __restrict__ w, void* out, int n, int k,
                                                           int ldw, int m0, int ldy, int parts)
{
    static_assert(NS % D == 0, "the buffer of a step must be known at compile time");
    constexpr int T = NW * 64;
    constexpr int XPR = (NS * 64 + T - 1) / T;                       // activation chunks per thread
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int chunks = k >> 3;
    // activation loads first: nothing may sit in front of them in the compute unit's load queue
    u32x4_t xl[XPR];
#pragma unroll
    for (int i = 0; i < XPR; ++i)
        xl[i] = reinterpret_cast<const u32x4_t*>(x)[min(tid + i * T, chunks - 1)];

    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                  // [NS * 64] chunks, zero past K
    int* ctr = reinterpret_cast<int*>(smem + (size_t)NS * 1024);
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool argmax = parts > 0;
    const int G = gridDim.x, b = blockIdx.x;
    const int row_bytes = ldw * 2;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(w), 0, ((n - 1) * ldw + k) * 2, 0x00020000);
    if (tid == 0)
        *ctr = NW;                                                   // indices 0 .. NW-1 are the waves' first rows
    auto row_of = [&](int i) { return i * G + b; };

    u32x4_t buf[D];
    auto issue = [&](int row, int t, int d) {
        const bool live = row < n && (t * 64 + lane) < chunks;
        buf[d] = __builtin_amdgcn_raw_buffer_load_b128(rw, live ? lane * 16 : kSentinelB,
                                                       (row < n ? row : 0) * row_bytes + t * 1024, 2);
    };
    int row = row_of(wave);
#pragma unroll
    for (int d = 0; d < D; ++d)
        issue(row, d, d);

#pragma unroll
    for (int i = 0; i < XPR; ++i) {
        const int c = tid + i * T;
        if (c < NS * 64)
            xs[c] = c < chunks ? xl[i] : u32x4_t{0, 0, 0, 0};
    }
    lds_barrier_b();
    u32x4_t xr[NS];
#pragma unroll
    for (int t = 0; t < NS; ++t)
        xr[t] = xs[t * 64 + lane];

    float best_val = -INFINITY;
    int best_idx = 0x7FFFFFFF;
    float res = 0.f;                    // finished outputs, one per lane
    int rowv = 0, slots = 0;
    auto flush = [&]() {
        if (lane < slots && rowv < n)
            static_cast<uint16_t*>(out)[(int64_t)m0 * ldy + rowv] = f32_to_bf16_rne(res);
        slots = 0;
        drain_vmem();                   // stores and loads share the counter: the loop only ever sees loads
    };
    auto fetch = [&]() {
        int v = 0;
        if (lane == 0)
            v = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return __builtin_amdgcn_readfirstlane(v);
    };
    int i_next = fetch();
    float acc = 0.f;
    while (row < n) {
        const int row_n = row_of(i_next);
        i_next = fetch();               // consumed one trip later: its latency is hidden
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            const int d = t % D;
            const u32x4_t wv = buf[d];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t wd = wv[j], xd = xr[t][j];            // (a bit cast needs a plain object)
                acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, wd),
                                                      __builtin_bit_cast(bf16x2_t, xd), acc, false);
            }
            const int tn = t + D;
            if (tn < NS)
                issue(row, tn, d);
            else
                issue(row_n, tn - NS, d);
        }
        const float v = wave_sum(acc);
        acc = 0.f;
        if (argmax) {
            // rows arrive in any order: the lower index wins among equal values
            if (v > best_val || (v == best_val && row < best_idx)) {
                best_val = v;
                best_idx = row;
            }
        } else {
            res = (lane == slots) ? v : res;
            rowv = (lane == slots) ? row : rowv;
            if (++slots == 64)
                flush();
        }
        row = row_n;
    }
    if (!argmax && slots > 0)
        flush();
    if (argmax) {
        __syncthreads();
        float* wvals = reinterpret_cast<float*>(smem);
        int* widx = reinterpret_cast<int*>(smem) + NW;
        if (lane == 0) {
            wvals[wave] = best_val;
            widx[wave] = best_idx;
        }
        __syncthreads();
        if (tid == 0) {
            float bv = wvals[0];
            int bi = widx[0];
            for (int i = 1; i < NW; ++i) {
                if (wvals[i] > bv || (wvals[i] == bv && widx[i] < bi)) {
                    bv = wvals[i];
                    bi = widx[i];
                }
            }
            float* part_val = static_cast<float*>(out);
            int32_t* part_idx = reinterpret_cast<int32_t*>(part_val + parts);     // one activation row
            part_val[b] = bv;
            part_idx[b] = bi;
        }
    }
}

template <int NS, int D, int NW>
hipError_t launch_reg_b(const Bf16Args& a, int blocks, hipStream_t stream)
{
    const bool argmax = a.part_val != nullptr;
    const size_t lds = (size_t)NS * 1024 + 64;
    hipLaunchKernelGGL((bf16_reg_kernel<NS, D, NW>), dim3(blocks), dim3(NW * 64), lds, stream, a.x, a.w,
                       argmax ? static_cast<void*>(a.part_val) : static_cast<void*>(a.y), a.n, a.k, (int)a.ldw, 0,
                       (int)a.ldy, argmax ? a.parts : 0);
    return hipGetLastError();
}

// One activation row, K a multiple of 8 up to 8192 (16 steps of activations in registers; with 22
// steps, the 7B down projection, it is 12 % slower than the general kernel), rows
// 16-byte aligned, enough rows to give every compute unit a workgroup's worth; in the argmax form
// the index array directly behind the one row of values.
bool bf16_reg_can_run(const Bf16Args& a, const DeviceInfo& dev)
{
    if (a.m != 1 || a.k % 8 != 0 || a.k > 8192 || a.n < dev.cus * 8)
        return false;
    if (a.ldw > 0x3FFFFFFF || a.ldy > 0x7FFFFFFF)
        return false;
    if (a.part_val && a.part_idx != reinterpret_cast<int32_t*>(a.part_val + a.parts))
        return false;
    return true;
}

hipError_t launch_bf16_reg(const Bf16Args& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    const int steps = (a.k + 511) / 512;
    // 12 waves per workgroup beyond K = 4096 and, up to there, beyond 40 rows per compute unit; else 16
    // (us per launch, 16 -> 12 waves: 8192 x 8192 26.9 -> 24.7, 12288 x 4096 18.0 -> 17.8, 32000 x 4096 42.9 ->
    // 42.2, but 4096 x 4096 7.4 -> 8.0; two workgroups of 8 or 12 per unit, or one of 8: slower)
    const int nw = steps > 8 || a.n > 40 * dev.cus ? 12 : 16;
    const int blocks = dev.cus < (a.n + nw - 1) / nw ? dev.cus : (a.n + nw - 1) / nw;
    if (parts_used)
        *parts_used = blocks;
    // (four steps in flight: 2 % faster on the largest matrices, 5 % slower on the smallest; one: 7 to 20 % slower)
    if (steps > 8)
        return launch_reg_b<16, 2, 12>(a, blocks, stream);
    return nw == 12 ? launch_reg_b<8, 2, 12>(a, blocks, stream) : launch_reg_b<8, 2, 16>(a, blocks, stream);
}

// Verification passes (three and more activation rows) on the matrix cores: the frame of the
// MXFP4 tile kernel without the decode.  A tile is 16 weight rows; in step T (128 elements of K)
// lane (i = lane % 16, g = lane / 16) loads, for each of the four v_mfma_f32_16x16x32_bf16 of the
// step, the 8 weights [128 T + 32 j + 8 g, + 8) of row i straight into the instruction's operand
// (64 bytes of a row per wave load); the MP activation rows of the pass sit in LDS as 16-byte
// chunks [chunk][row ^ (chunk % MP)] (the copy's writes and the loop's 128-bit reads are then
// free of bank conflicts); NW compute waves split the steps of a tile, keep D steps in flight
// each, leave their partial tiles in LDS; one more wave, which never loads, adds them in a fixed
// order and stores or tracks the argmax; one barrier per tile.  Every position-dependent condition
// is an arithmetic mask on the offsets, so every trip issues the same loads.
typedef __attribute__((ext_vector_type(4))) float bf_f32x4_t;

template <int MP, int NW, int D>
__global__ __launch_bounds__((NW + 1) * 64) void bf16_mfma_kernel(const uint16_t* __restrict__ x,
                                                                  const uint16_t* __restrict__ w, void* out, int n,
                                                                  int k, int ldw, int m, int m0, int ldx, int ldy,
                                                                  int parts)
{
    constexpr int T = (NW + 1) * 64;
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);
    const int tid = threadIdx.x;
    const int steps = k >> 7;
    const int chunks = steps * 16;                                      // 16-byte chunks per activation row
    constexpr int XB = 16 / MP;
    const int xpr = (chunks + T - 1) / T;
    u32x4_t xl[XB][MP];
    auto x_load = [&](int i0) {
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            const int kc = min(tid + (i0 + i) * T, chunks - 1);
#pragma unroll
            for (int mm = 0; mm < MP; ++mm) {
                const int msrc = min(m0 + mm, m - 1);                   // ragged M: repeat the last row
                xl[i][mm] = reinterpret_cast<const u32x4_t*>(x + (int64_t)msrc * ldx)[kc];
            }
        }
    };
    x_load(0);

    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int row_bytes = ldw * 2;
    const int spw = (steps + NW - 1) / NW;                              // steps per wave and tile
    const int n_tiles = (n + 15) >> 4;
    const int G = gridDim.x, b = blockIdx.x;
    bf_f32x4_t* red = reinterpret_cast<bf_f32x4_t*>(smem + (size_t)chunks * 16 * MP);   // [2][NW][64]
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(w), 0, ((n - 1) * ldw + k) * 2, 0x00020000);

    struct Item {
        u32x4_t w[4];
    };
    Item buf[D];
    int ld_tile = b, ld_loc = 0;
    auto issue = [&](Item& it) {
        const int live = (int)(ld_tile < n_tiles);
        const int step = wave + NW * ld_loc;
        const int mk = -(live & (int)(step < steps) & (int)(wave < NW));   // all ones when the step exists
        const int row = min(ld_tile * live * 16 + li, n - 1);             // ragged N: repeat the last row
        const int vq = row * row_bytes + lg * 16;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            it.w[j] = __builtin_amdgcn_raw_buffer_load_b128(rw, (vq & mk) | (kSentinelB & ~mk),
                                                            ((step * 256 + j * 64) & mk) | ((j * 16) & ~mk), 0);
        const int wrap = (int)(ld_loc + 1 == spw);
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
    auto x_store = [&](int i0) {
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            const int kc = tid + (i0 + i) * T;
            if (kc < chunks) {
#pragma unroll
                for (int mm = 0; mm < MP; ++mm)
                    xs[kc * MP + (mm ^ (kc & (MP - 1)))] = xl[i][mm];
            }
        }
    };
    x_store(0);
#pragma unroll 1
    for (int i0 = XB; i0 < xpr; i0 += XB) {
        x_load(i0);
        x_store(i0);
    }
    lds_barrier_b();

    const bool argmax = parts > 0;
    if (wave == NW) {
        // Epilogue wave: one barrier per tile, like the compute waves; no loads of its own.
        const int m_valid = min(MP, m - m0);
        float best_val = -INFINITY;
        int best_idx = 0x7FFFFFFF;
        int done = 0;
        for (int tile = b; tile < n_tiles; tile += G, ++done) {
            const bf_f32x4_t* slot = red + (size_t)(done & 1) * NW * 64;
            lds_barrier_b();                                            // partial tiles of `tile` are in LDS
            bf_f32x4_t sum = slot[lane];
#pragma unroll
            for (int v = 1; v < NW; ++v)
                sum += slot[v * 64 + lane];
            // lane (li, lg) holds weight rows 4 lg + r of the tile for activation row li
            if (li < m_valid) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = tile * 16 + 4 * lg + r;
                    if (row < n) {
                        if (argmax) {
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
        if (argmax) {
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

    bf_f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};   // two chains: even and odd j
    const int col = li & (MP - 1);
    int c_tile = b, c_loc = 0, done = 0;
    // Positions only grow, so the walk ends when buffer 0 runs dry; every trip issues the same loads.
    while (c_tile < n_tiles) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d == 0 || c_tile < n_tiles) {
                const Item& it = buf[d];
                const int step = wave + NW * c_loc;
                const int Tq = step < steps ? step : 0;                 // a step that does not exist has zero weights
                u32x4_t xb[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    xb[j] = xs[(Tq * 16 + 4 * j + lg) * MP + (col ^ ((4 * j + lg) & (MP - 1)))];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u32x4_t wv = it.w[j];
                    if (j & 1)
                        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wv),
                                                                       __builtin_bit_cast(bf16x8_t, xb[j]), acc1, 0, 0, 0);
                    else
                        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wv),
                                                                       __builtin_bit_cast(bf16x8_t, xb[j]), acc0, 0, 0, 0);
                }
                if (c_loc == spw - 1) {
                    bf_f32x4_t* slot = red + (size_t)(done & 1) * NW * 64;
                    slot[wave * 64 + lane] = acc0 + acc1;
                    acc0 = bf_f32x4_t{0.f, 0.f, 0.f, 0.f};
                    acc1 = bf_f32x4_t{0.f, 0.f, 0.f, 0.f};
                    lds_barrier_b();
                    ++done;
                }
                if (++c_loc == spw) {
                    c_loc = 0;
                    c_tile += G;
                }
            }
            issue(buf[d]);
        }
    }
}

size_t bf16_mfma_lds(int k, int mp, int nw) { return (size_t)k * 2 * mp + (size_t)2 * nw * 1024; }
int bf16_pass_width(int left) { return left > 8 ? 16 : (left > 4 ? 8 : 4); }

template <int MP, int NW>
hipError_t launch_mfma_b(const Bf16Args& a, int m0, int blocks, size_t lds, int max_lds, hipStream_t stream)
{
    auto kern = bf16_mfma_kernel<MP, NW, 2>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), max_lds); e != hipSuccess)
        return e;
    const bool argmax = a.part_val != nullptr;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3((NW + 1) * 64), lds, stream, a.x, a.w,
                       argmax ? static_cast<void*>(a.part_val) : static_cast<void*>(a.y), a.n, a.k, (int)a.ldw, a.m,
                       m0, (int)a.ldx, (int)a.ldy, argmax ? a.parts : 0);
    return hipGetLastError();
}

// Three and more rows, K % 128 == 0, the widest pass's activation rows fit the LDS beside the
// partial tiles; 32-bit leading dimensions; the argmax index array directly behind the values.
bool bf16_mfma_can_run(const Bf16Args& a, const DeviceInfo& dev)
{
    if (a.m < 3 || a.k % 128 != 0 || a.n < 16)
        return false;
    if (a.ldx > 0x7FFFFFFF || a.ldy > 0x7FFFFFFF || a.ldw > 0x3FFFFFFF)
        return false;
    if (a.part_val && a.part_idx != reinterpret_cast<int32_t*>(a.part_val + (size_t)a.m * a.parts))
        return false;
    return bf16_mfma_lds(a.k, bf16_pass_width(a.m), 4) <= (size_t)dev.lds_bytes;
}

hipError_t launch_bf16_mfma(const Bf16Args& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    const int n_tiles = (a.n + 15) / 16;
    // two workgroups of four compute waves per compute unit when two copies of the widest pass's
    // activations fit, else one of eight (what the MXFP4 tile kernel settled on)
    const int widest = bf16_pass_width(a.m);
    const bool two = 2 * bf16_mfma_lds(a.k, widest, 4) + 2048 <= (size_t)dev.lds_bytes;
    const bool wide = !two && bf16_mfma_lds(a.k, widest, 8) <= (size_t)dev.lds_bytes;
    int blocks = dev.cus * (two ? 2 : 1);
    blocks = blocks > n_tiles ? n_tiles : blocks;
    blocks = blocks > gemv_max_parts(dev) ? gemv_max_parts(dev) : blocks;
    if (parts_used)
        *parts_used = blocks;                       // every pass uses the same grid: the partials line up
    for (int m0 = 0; m0 < a.m;) {
        const int mp = bf16_pass_width(a.m - m0);
        const size_t lds = bf16_mfma_lds(a.k, mp, wide ? 8 : 4);
        hipError_t e;
        if (wide)
            e = mp == 16  ? launch_mfma_b<16, 8>(a, m0, blocks, lds, dev.lds_bytes, stream)
                : mp == 8 ? launch_mfma_b<8, 8>(a, m0, blocks, lds, dev.lds_bytes, stream)
                          : launch_mfma_b<4, 8>(a, m0, blocks, lds, dev.lds_bytes, stream);
        else
            e = mp == 16  ? launch_mfma_b<16, 4>(a, m0, blocks, lds, dev.lds_bytes, stream)
                : mp == 8 ? launch_mfma_b<8, 4>(a, m0, blocks, lds, dev.lds_bytes, stream)
                          : launch_mfma_b<4, 4>(a, m0, blocks, lds, dev.lds_bytes, stream);
        if (e != hipSuccess)
            return e;
        m0 += mp;
    }
    return hipSuccess;
}

// The same product when the MT activation rows of a pass do not fit the LDS whole: K is cut into
// phases of `phase_steps` steps.  For every phase the workgroup stages that part of the activation
// rows, every wave walks all of its row groups over the phase's K range and adds the partial sums
// to the outputs it holds, one row per lane (at most 64 rows per wave: the host checks), and only
// after the last phase rounds and stores them.  The weights are still read once; the cost is one
// pipeline start per phase.  Fixed order of additions: deterministic.
template <int MT, int R, int NW>
__global__ __launch_bounds__(NW * 64) void bf16_phased_kernel(Bf16Args a, int m0, int phase_steps)
{
    extern __shared__ __align__(16) uint8_t smem[];
    u32x4_t* xs = reinterpret_cast<u32x4_t*>(smem);                  // [MT][phase_steps * 64] chunks
    constexpr int T = NW * 64;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int chunks = a.k >> 3;
    const int steps = (chunks + 63) >> 6;
    const int pc = phase_steps * 64;                                 // chunks per row and phase
    const int n_groups = (a.n + R - 1) / R;
    const int total_waves = gridDim.x * NW;
    const int first_group = (int)blockIdx.x * NW + wave;
    const int row_bytes = (int)a.ldw * 2;
    const bool argmax = a.part_val != nullptr;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(a.w), 0, (int)((a.n - 1) * a.ldw + a.k) * 2, 0x00020000);

    float res[MT];               // lane s holds the running output of the wave's s-th row
#pragma unroll
    for (int m = 0; m < MT; ++m)
        res[m] = 0.f;
    float acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MT; ++m)
            acc[r][m] = 0.f;

    for (int t_lo = 0; t_lo < steps; t_lo += phase_steps) {
        const int t_hi = min(steps, t_lo + phase_steps);
        __syncthreads();                                             // everyone is done with the previous phase's rows
        for (int c = tid; c < pc; c += T) {
            const int cg = t_lo * 64 + c;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const int msrc = min(m0 + m, a.m - 1);               // ragged M: repeat the last row
                const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(a.x + (int64_t)msrc * a.ldx);
                xs[m * pc + c] = cg < chunks ? xp[cg] : u32x4_t{0, 0, 0, 0};
            }
        }
        __syncthreads();

        auto valid = [&](const BPos& p) { return p.g < n_groups; };
        auto advance = [&](BPos& p) {
            if (++p.t == t_hi) {
                p.t = t_lo;
                p.g += total_waves;
            }
        };
        auto issue = [&](const BPos& p, u32x4_t (&w)[R]) {
            const bool live = valid(p) && p.t * 64 + lane < chunks;
            const int voff = live ? lane * 16 : kSentinelB;
            const int g = valid(p) ? p.g : 0;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = min(g * R + r, a.n - 1);              // ragged N: re-read the last row
                w[r] = __builtin_amdgcn_raw_buffer_load_b128(rw, voff, row * row_bytes + p.t * 1024, 2);
            }
        };
        u32x4_t buf[2][R];
        BPos pos[2];
        BPos load{first_group, t_lo};
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            pos[d] = load;
            issue(load, buf[d]);
            advance(load);
        }
        int slot = 0;                                                // first row slot of the group being summed
        auto compute = [&](const BPos& p, const u32x4_t (&w)[R]) {
            u32x4_t xv[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m)
                xv[m] = xs[m * pc + (p.t - t_lo) * 64 + lane];        // zero past K, as are the weights
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t wd = w[r][j];
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        const uint32_t xd = xv[m][j];
                        acc[r][m] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, wd),
                                                                    __builtin_bit_cast(bf16x2_t, xd), acc[r][m], false);
                    }
                }
            }
            if (p.t == t_hi - 1) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        const float v = wave_sum(acc[r][m]);
                        acc[r][m] = 0.f;
                        res[m] += (lane == slot + r) ? v : 0.f;
                    }
                slot += R;
            }
        };
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
    }

    // lane s holds row (first_group + (s / R) * total_waves) * R + s % R
    const int j = lane / R, r = lane - j * R;
    const int grp = first_group + j * total_waves;
    const int row = grp * R + r;
    const bool own = grp < n_groups && row < a.n;
    if (!argmax) {
        if (own) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
                if (m0 + m < a.m)
                    a.y[(int64_t)(m0 + m) * a.ldy + row] = f32_to_bf16_rne(res[m]);
        }
        return;
    }
    __syncthreads();
    float* wv = reinterpret_cast<float*>(smem);
    int* wi = reinterpret_cast<int*>(smem) + NW * MT;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        float bv = own ? res[m] : -INFINITY;
        int bi = own ? row : 0x7FFFFFFF;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float v = __shfl_xor(bv, off);
            const int i = __shfl_xor(bi, off);
            if (v > bv || (v == bv && i < bi)) {
                bv = v;
                bi = i;
            }
        }
        if (lane == 0) {
            wv[wave * MT + m] = bv;
            wi[wave * MT + m] = bi;
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

template <int MT, int R>
hipError_t launch_phased(const Bf16Args& a, int m0, int blocks, int phase_steps, int max_lds, hipStream_t stream)
{
    auto kern = bf16_phased_kernel<MT, R, 16>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), max_lds); e != hipSuccess)
        return e;
    const size_t lds = (size_t)MT * phase_steps * 1024;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(16 * 64), lds, stream, a, m0, phase_steps);
    return hipGetLastError();
}

template <int MT, int R, int NW>
hipError_t launch_b(const Bf16Args& a, int m0, int blocks, size_t lds, int max_lds, hipStream_t stream)
{
    auto kern = bf16_gemv_kernel<MT, R, NW>;
    static LdsLimit lds_limit;                      // of this kernel instance
    if (hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), max_lds); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, stream, a, m0);
    return hipGetLastError();
}

template <int MT>
hipError_t launch_rows(const Bf16Args& a, int m0, int r, int nw, int blocks, size_t lds, int max_lds,
                       hipStream_t stream)
{
#define MXFP4_BF16_CASE(NW_)                                                              \
    if (nw == NW_)                                                                        \
        return r == 2 ? launch_b<MT, 2, NW_>(a, m0, blocks, lds, max_lds, stream)         \
                      : launch_b<MT, 1, NW_>(a, m0, blocks, lds, max_lds, stream);
    MXFP4_BF16_CASE(4)
    MXFP4_BF16_CASE(8)
    MXFP4_BF16_CASE(16)
#undef MXFP4_BF16_CASE
    return hipErrorInvalidValue;
}

}  // namespace

// Largest K whose activation copy (one row) fits the LDS.
bool bf16_can_run(const Bf16Args& a, const DeviceInfo& dev) { return (size_t)a.k * 2 <= (size_t)dev.lds_bytes; }

hipError_t launch_bf16_gemv(const Bf16Args& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream)
{
    static const bool general_only = [] {
        const char* e = knob("MXFP4_BF16_GENERAL");                // measurement only
        return e && atoi(e) != 0;
    }();
    if (!general_only && bf16_reg_can_run(a, dev))
        return launch_bf16_reg(a, dev, parts_used, stream);
    // Up to eight rows the vector-ALU kernel below is as fast or faster in one pass (7B shapes, µs:
    // 20.1 / 33.0 / 46.3 against 21.2 / 36.8 / 48.6 at four rows, equal at eight); from nine rows on
    // it needs two passes and the matrix cores one.
    static const int mfma_from = [] {
        const char* e = knob("MXFP4_BF16_MFMA_FROM");             // measurement only
        return e ? atoi(e) : 9;
    }();
    if (!general_only && a.m >= mfma_from && bf16_mfma_can_run(a, dev))
        return launch_bf16_mfma(a, dev, parts_used, stream);
    // two rows per group unless the matrix is so short that SIMDs would idle
    const int r = (a.n + 1) / 2 >= dev.cus * 16 ? 2 : 1;
    const int n_groups = (a.n + r - 1) / r;
    int first_blocks = 0;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        // the narrowest pass that takes all remaining rows (a ragged pass repeats its last row)
        int mt = left > 4 ? 8 : (left > 2 ? 4 : (left > 1 ? 2 : 1));
        if (mt == 8 && left <= 6 && (size_t)8 * a.k * 2 > (size_t)dev.lds_bytes &&
            (size_t)6 * a.k * 2 <= (size_t)dev.lds_bytes)
            mt = 6;                                                 // five or six rows that fit where eight do not
        // The rows of the pass do not fit the LDS whole: K in phases, still one pass over the weights,
        // when a wave's rows fit its 64 lanes (one workgroup of 16 waves per compute unit).
        if (mt >= 2 && (size_t)mt * a.k * 2 > (size_t)dev.lds_bytes && !general_only) {
            const int pblocks = dev.cus < (n_groups + 15) / 16 ? dev.cus : (n_groups + 15) / 16;
            const int groups_per_wave = (n_groups + pblocks * 16 - 1) / (pblocks * 16);
            const int fit_steps = (int)(((size_t)dev.lds_bytes - 16 * 1024) / ((size_t)mt * 1024));
            const int k_steps = (a.k / 8 + 63) / 64;
            const int n_phases = fit_steps > 0 ? (k_steps + fit_steps - 1) / fit_steps : 0;
            const int phase_steps = n_phases > 0 ? (k_steps + n_phases - 1) / n_phases : 0;   // even phases
            const bool parts_ok = a.part_val == nullptr || first_blocks == 0 || pblocks <= first_blocks;
            if (groups_per_wave * r <= 64 && phase_steps >= 4 && pblocks <= gemv_max_parts(dev) && parts_ok &&
                (m0 == 0 || a.part_val == nullptr || pblocks == first_blocks)) {
                hipError_t e;
                if (r == 2)
                    e = mt >= 6   ? launch_phased<8, 2>(a, m0, pblocks, phase_steps, dev.lds_bytes, stream)
                        : mt == 4 ? launch_phased<4, 2>(a, m0, pblocks, phase_steps, dev.lds_bytes, stream)
                                  : launch_phased<2, 2>(a, m0, pblocks, phase_steps, dev.lds_bytes, stream);
                else
                    e = mt >= 6   ? launch_phased<8, 1>(a, m0, pblocks, phase_steps, dev.lds_bytes, stream)
                        : mt == 4 ? launch_phased<4, 1>(a, m0, pblocks, phase_steps, dev.lds_bytes, stream)
                                  : launch_phased<2, 1>(a, m0, pblocks, phase_steps, dev.lds_bytes, stream);
                if (e != hipSuccess)
                    return e;
                if (m0 == 0)
                    first_blocks = pblocks;
                m0 += mt;
                continue;
            }
        }
        while (mt > 1 && (size_t)mt * a.k * 2 > (size_t)dev.lds_bytes)
            mt = mt == 6 ? 4 : mt >> 1;
        const size_t lds = (size_t)mt * a.k * 2 < 256 ? 256 : (size_t)mt * a.k * 2;   // the argmax combine needs a few bytes
        int per_cu = (int)((size_t)dev.lds_bytes / lds);
        per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
        // 16 waves per CU: larger workgroups when the activation copy leaves room for fewer of them
        const int nw = per_cu >= 3 ? 4 : (per_cu == 2 ? 8 : 16);
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
        case 6:
            e = launch_rows<6>(a, m0, r, nw, blocks, lds, dev.lds_bytes, stream);
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
