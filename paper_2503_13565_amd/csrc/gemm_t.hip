// The product along the rows of a stored MXFP4 tensor: y[m, k] = sum_n x[m, n] * dequant(W)[n, k]
// (arXiv 2503.13565, section 5 names a quantised attention cache as the next step: with one token
// per weight row and the blocks of section 3.4.3 along the head dimension, a new token is cast on
// its own when it is appended, the score side q K^T is the ordinary product, and the value side
// p V contracts over the rows, which is this kernel).  FP32 accumulation as in Eq. 2, with the block
// scale folded into the activation: x[m, n] * X[n, k / 32] is exact in FP32, the elements are the
// unscaled E2M1 values.
//
// A thread owns eight consecutive columns (one dword of nibbles) and every rpp-th row of its
// workgroup's run of rows; the K/8 threads of a row read it as one contiguous run of K/2 bytes.  The
// threads of a column group are summed through LDS, the workgroups through FP32 partials [G, M, K]
// and a second small kernel that adds them in index order and rounds to BF16 once.
#include "common.h"
#include "kernels.h"

namespace mxfp4 {

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;               // rows in flight per thread

template <int MT>
__global__ __launch_bounds__(kThreads) void gemm_t_kernel(const uint16_t* __restrict__ x, int64_t ldx, int m0, int m,
                                                          const uint32_t* __restrict__ q,
                                                          const uint8_t* __restrict__ s, int n, int k,
                                                          int rows_per_wg, float* __restrict__ part)
{
    extern __shared__ __align__(16) float red[];                    // [rpp][MT][K]
    const int cols = k >> 3;
    const int nblk = k >> 5;
    const int rpp = kThreads / cols;                                // rows per pass of the workgroup
    const int tid = threadIdx.x;
    const int c = tid % cols, rl = tid / cols;
    const bool active = rl < rpp;
    const int row0 = (int)blockIdx.x * rows_per_wg;
    const int row_end = min(n, row0 + rows_per_wg);

    float acc[MT][8];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e)
            acc[i][e] = 0.f;

    if (active) {
        for (int r0 = row0 + rl; r0 < row_end; r0 += rpp * kUnroll) {
            uint32_t qd[kUnroll];
            uint32_t sb[kUnroll];
            uint16_t xv[kUnroll][MT];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int r = r0 + u * rpp;
                const int rc = min(r, row_end - 1);                 // surplus slots re-read the last row, weight zero
                qd[u] = q[(int64_t)rc * cols + c];
                sb[u] = s[(int64_t)rc * nblk + (c >> 2)];
#pragma unroll
                for (int i = 0; i < MT; ++i)
                    xv[u][i] = x[(int64_t)min(m0 + i, m - 1) * ldx + rc];
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const bool live = r0 + u * rpp < row_end;
                const float scale = e8m0_to_f32(sb[u]);
                float w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    w[e] = e2m1_to_f32((qd[u] >> (4 * e)) & 0xFu);
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    const float t = live ? bf16_bits_to_f32(xv[u][i]) * scale : 0.f;
                    if (live) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            acc[i][e] = __builtin_fmaf(t, w[e], acc[i][e]);
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                red[((size_t)rl * MT + i) * k + c * 8 + e] = acc[i][e];
    }
    __syncthreads();
    for (int o = tid; o < MT * k; o += kThreads) {
        float v = 0.f;
        for (int r = 0; r < rpp; ++r)
            v += red[(size_t)r * MT * k + o];
        const int i = o / k, col = o - i * k;
        if (m0 + i < m)
            part[((size_t)blockIdx.x * m + m0 + i) * k + col] = v;
    }
}

__global__ __launch_bounds__(kThreads) void gemm_t_finish_kernel(const float* __restrict__ part, int groups, int m, int k,
                                                                 uint16_t* __restrict__ y, int64_t ldy)
{
    const int o = (int)blockIdx.x * kThreads + threadIdx.x;
    if (o >= m * k)
        return;
    // index order; eight loads in flight at a time (one by one, each add waits a memory round trip)
    float v = 0.f;
    int g = 0;
    for (; g + 8 <= groups; g += 8) {
        float p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            p[u] = part[(size_t)(g + u) * m * k + o];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v += p[u];
    }
    for (; g < groups; ++g)
        v += part[(size_t)g * m * k + o];
    const int i = o / k, col = o - i * k;
    y[(int64_t)i * ldy + col] = f32_to_bf16_rne(v);
}

int rows_per_pass(int k) { return kThreads / (k >> 3); }

}  // namespace

// Workgroups the launch uses: each takes a run of rows that is a multiple of the rows in flight.
int gemm_t_groups(int n, int k, const DeviceInfo& dev)
{
    const int quantum = rows_per_pass(k) * kUnroll;
    int groups = (n + quantum - 1) / quantum;
    const int cap = dev.cus * 4;
    return groups < 1 ? 1 : (groups > cap ? cap : groups);
}

bool gemm_t_can_run(int k) { return k >= 32 && k % 32 == 0 && k <= 2048; }

size_t gemm_t_workspace_bytes(int m, int n, int k, const DeviceInfo& dev)
{
    return (size_t)gemm_t_groups(n, k, dev) * m * k * sizeof(float);
}

hipError_t launch_gemm_t(const GemmArgs& a, const DeviceInfo& dev, float* part, hipStream_t stream)
{
    const int groups = gemm_t_groups(a.n, a.k, dev);
    const int quantum = rows_per_pass(a.k) * kUnroll;
    int rows_per_wg = (a.n + groups - 1) / groups;
    rows_per_wg = (rows_per_wg + quantum - 1) / quantum * quantum;
    for (int m0 = 0; m0 < a.m;) {
        const int left = a.m - m0;
        const int mt = left > 4 ? 8 : (left > 2 ? 4 : (left > 1 ? 2 : 1));
        const size_t lds = (size_t)rows_per_pass(a.k) * mt * a.k * sizeof(float);    // at most 64 KiB
        const uint32_t* q = reinterpret_cast<const uint32_t*>(a.q);
        switch (mt) {
        case 8:
            hipLaunchKernelGGL(gemm_t_kernel<8>, dim3(groups), dim3(kThreads), lds, stream, a.x, a.ldx, m0, a.m, q, a.s,
                               a.n, a.k, rows_per_wg, part);
            break;
        case 4:
            hipLaunchKernelGGL(gemm_t_kernel<4>, dim3(groups), dim3(kThreads), lds, stream, a.x, a.ldx, m0, a.m, q, a.s,
                               a.n, a.k, rows_per_wg, part);
            break;
        case 2:
            hipLaunchKernelGGL(gemm_t_kernel<2>, dim3(groups), dim3(kThreads), lds, stream, a.x, a.ldx, m0, a.m, q, a.s,
                               a.n, a.k, rows_per_wg, part);
            break;
        default:
            hipLaunchKernelGGL(gemm_t_kernel<1>, dim3(groups), dim3(kThreads), lds, stream, a.x, a.ldx, m0, a.m, q, a.s,
                               a.n, a.k, rows_per_wg, part);
            break;
        }
        if (hipError_t e = hipGetLastError(); e != hipSuccess)
            return e;
        m0 += mt;
    }
    const int outs = a.m * a.k;
    hipLaunchKernelGGL(gemm_t_finish_kernel, dim3((outs + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, part,
                       groups, a.m, a.k, a.y, a.ldy);
    return hipGetLastError();
}

}  // namespace mxfp4
