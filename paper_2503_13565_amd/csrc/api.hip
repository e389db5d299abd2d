// C ABI of the MXFP4 weight-only-quantised linear layer (include/mxfp4.h): argument checks,
// dispatch by the number of activation rows, and two plain streaming kernels used to measure
// the memory system.  All device work is enqueued on the caller's stream; nothing here
// synchronises, allocates or frees device memory.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "common.h"
#include "kernels.h"
#include "../../include/mxfp4.h"

namespace mxfp4 {

static thread_local char g_err[512] = "";
// Set while a grouped call checks its descriptors: run_gemm then does everything but launch.
static thread_local bool g_check_only = false;

// Every entry point starts here: no error text yet, and a HIP error left behind by earlier calls of
// the caller (the runtime keeps the last one until somebody reads it) must not be reported as the
// status of the launches that follow.
static void begin_call()
{
    g_err[0] = 0;
    (void)hipGetLastError();
}

static int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

static int hip_fail(hipError_t e, const char* what)
{
    return fail(MXFP4_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// Per-device facts, looked up once per device.
static int device_info(DeviceInfo* out)
{
    static DeviceInfo cache[64];
    static std::atomic<bool> have[64];              // set after the entry is complete (racing threads write the same values)
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64)
        return fail(MXFP4_ERR_HIP, "device ordinal %d out of range", dev);
    if (!have[dev].load(std::memory_order_acquire)) {
        int cus = 0, lds = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess)
            return hip_fail(e, "hipDeviceGetAttribute(cus)");
        e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
        if (e != hipSuccess)
            return hip_fail(e, "hipDeviceGetAttribute(lds)");
        cache[dev].cus = cus > 0 ? cus : 256;
        cache[dev].lds_bytes = lds > 0 ? lds : 64 * 1024;
        have[dev].store(true, std::memory_order_release);
    }
    *out = cache[dev];
    return MXFP4_OK;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static int check_weights(const void* q, const void* s, int64_t N, int64_t K)
{
    if (!q || !s)
        return fail(MXFP4_ERR_NULL, "q_packed or scales_e8m0 is NULL");
    if (N < 1 || N > 0x7FFFFFFF / 8)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > MXFP4_MAX_K)
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a multiple of 32 in [32, %d]", (long long)K, MXFP4_MAX_K);
    if (N * (K / 2) > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "N*K/2=%lld bytes of packed weights exceed 2 GiB - 1", (long long)(N * (K / 2)));
    if (!aligned(q, 16))
        return fail(MXFP4_ERR_ALIGN, "q_packed must be 16-byte aligned");
    if (!aligned(s, 4))
        return fail(MXFP4_ERR_ALIGN, "scales_e8m0 must be 4-byte aligned");
    return MXFP4_OK;
}

static int check_x(const void* x, int64_t M, int64_t ldx, int64_t K)
{
    if (!x)
        return fail(MXFP4_ERR_NULL, "x_bf16 is NULL");
    if (M < 1 || M > (1 << 20))
        return fail(MXFP4_ERR_SHAPE, "M=%lld out of range", (long long)M);
    if (ldx < K)
        return fail(MXFP4_ERR_SHAPE, "ldx=%lld < K=%lld", (long long)ldx, (long long)K);
    if (ldx % 8 != 0 || !aligned(x, 16))
        return fail(MXFP4_ERR_ALIGN, "x_bf16 must be 16-byte aligned with ldx %% 8 == 0");
    return MXFP4_OK;
}

// AUTO: the vector-ALU GEMV for one or two activation rows (its register-resident form when the
// shape allows), MFMA tiles from three rows on (each extra row costs the GEMV half an instruction
// per weight; the tiles' cost does not grow up to 16 rows), unless the shape cannot run there.
// Two rows with K beyond 8192 also go to the tiles: the register form would take two passes and
// the general GEMV is slower there (measured: 4096 x 11008 13.3 against 9.5 us, 8192 x 28672 48
// against 34; at K = 8192 the GEMV still wins by 5 %).
static int pick_path(int path, int64_t M, int64_t K, bool mfma_ok, bool reg_ok)
{
    if (path != MXFP4_PATH_AUTO)
        return path;
    static int env_path = -1;
    if (env_path < 0) {
        const char* v = getenv("MXFP4_FORCE_PATH");
        env_path = v ? atoi(v) : 0;
    }
    if (env_path > 0)
        return env_path;
    if (M >= 3 && mfma_ok)
        return MXFP4_PATH_MFMA;
    if (reg_ok)
        return MXFP4_PATH_VALU_REG;
    return M == 2 && K > 8192 && mfma_ok ? MXFP4_PATH_MFMA : MXFP4_PATH_VALU_CVT;
}

// Draft verification fused behind the argmax (both product forms): NULL when not asked for.
struct Verify {
    const int32_t* draft;
    int32_t* accept_out;
};

static int check_verify(const Verify* v, int64_t M)
{
    if (!v)
        return MXFP4_OK;
    if (!v->accept_out)
        return fail(MXFP4_ERR_NULL, "accept_out is NULL");
    if (M > 1 && !v->draft)
        return fail(MXFP4_ERR_NULL, "draft_tokens is NULL");
    if (M > kVerifyMaxRows)
        return fail(MXFP4_ERR_SHAPE, "M=%lld rows exceed the %d a verification pass takes", (long long)M,
                    kVerifyMaxRows);
    return MXFP4_OK;
}

static int run_gemm(const void* x, int64_t M, int64_t ldx, const void* q, const void* s, int64_t N, int64_t K,
                    void* y, int64_t ldy, int32_t* argmax_out, float* max_out, void* workspace,
                    size_t workspace_bytes, bool argmax, int path, void* stream, const Verify* verify = nullptr,
                    bool tiled = false, const Epilogue* epi = nullptr)
{
    begin_call();
    int rc = check_verify(verify, M);
    if (rc)
        return rc;
    int64_t C = N;                                  // columns of y
    if (epi) {
        if (epi->act != MXFP4_ACT_NONE && epi->act != MXFP4_ACT_SWIGLU)
            return fail(MXFP4_ERR_ARG, "unknown act %d", epi->act);
        if (epi->act == MXFP4_ACT_SWIGLU) {
            if (N % 2 != 0)
                return fail(MXFP4_ERR_SHAPE, "the gate pairs rows 2c and 2c + 1: N=%lld must be even", (long long)N);
            C = N / 2;
        }
        if (!aligned(epi->bias, 2) || !aligned(epi->residual, 2))
            return fail(MXFP4_ERR_ALIGN, "bias_bf16 and residual_bf16 must be 2-byte aligned");
        if (path == MXFP4_PATH_VALU_BITS || path == MXFP4_PATH_VALU_LUT)
            return fail(MXFP4_ERR_ARG, "path %d has no fused form", path);
    }
    rc = check_weights(q, s, tiled ? (N + 15) / 16 * 16 : N, K);      // tile-major tensors hold whole tiles
    if (rc)
        return rc;
    if (tiled && (K % 128 != 0 || !aligned(s, 16)))
        return K % 128 != 0 ? fail(MXFP4_ERR_SHAPE, "tile-major weights need K %% 128 == 0, K=%lld", (long long)K)
                            : fail(MXFP4_ERR_ALIGN, "s_tiled must be 16-byte aligned");
    rc = check_x(x, M, ldx, K);
    if (rc)
        return rc;
    DeviceInfo dev;
    rc = device_info(&dev);
    if (rc)
        return rc;
    GemmArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.ldx = ldx;
    a.q = static_cast<const uint8_t*>(q);
    a.s = static_cast<const uint8_t*>(s);
    a.m = (int)M;
    a.n = (int)N;
    a.k = (int)K;
    // workspace layout: [argmax partial values][argmax partial indices][split-K partial products]
    const size_t argmax_bytes = argmax ? (size_t)M * gemv_max_parts(dev) * 8 : 0;
    float* splitk_ws = nullptr;
    if (workspace && aligned(workspace, 8)) {
        const size_t sk = mfma_splitk_bytes((int)M, (int)N, (int)K, dev);
        if (sk > 0 && workspace_bytes >= argmax_bytes + sk)
            splitk_ws = reinterpret_cast<float*>(static_cast<char*>(workspace) + argmax_bytes);
    }
    if (argmax) {
        if (!argmax_out)
            return fail(MXFP4_ERR_NULL, "argmax_out is NULL");
        const size_t need = mxfp4_woq_gemm_argmax_workspace_bytes(M, N, K);
        if (!workspace || workspace_bytes < need)
            return fail(MXFP4_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
        if (!aligned(workspace, 8))
            return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
        a.parts = gemv_max_parts(dev);
        a.part_val = static_cast<float*>(workspace);
        a.part_idx = reinterpret_cast<int32_t*>(a.part_val + (size_t)M * a.parts);
    } else {
        if (!y)
            return fail(MXFP4_ERR_NULL, "y_bf16 is NULL");
        if (ldy < C)
            return fail(MXFP4_ERR_SHAPE, "ldy=%lld < %lld columns of y", (long long)ldy, (long long)C);
        a.y = static_cast<uint16_t*>(y);
        a.ldy = ldy;
    }
    const int chosen = tiled ? -1
                             : pick_path(path, M, K, mfma_can_run(a, dev, splitk_ws != nullptr),
                                         gemv_reg_can_run(a, dev) && gemv_reg_single_pass(a));
    hipStream_t st = static_cast<hipStream_t>(stream);
    int parts_used = 0;
    hipError_t e = hipSuccess;
    const bool go = !g_check_only;
    switch (chosen) {
    case -1: {
        // One row: the decode kernel of the tile-major layout (the tiles' matrix-core kernel takes 7 %
        // longer over the four linears of a 7B layer).  Two rows: the tiles where they run (equal or
        // up to 8 % faster on the 7B shapes), else the decode kernel (K = 28672: 28.1 against 29.6 us).
        static const bool tiled_decode = [] {
            const char* e = knob("MXFP4_TILED_DECODE");              // measurement only
            return !e || atoi(e) != 0;
        }();
        if (tiled_decode && !epi && gemv_tile_can_run(a, dev) && (a.m == 1 || !mfma_tile_can_run(a, dev))) {
            if (go)
                e = launch_gemv_tile(a, dev, &parts_used, st);
        } else if (mfma_tile_can_run(a, dev)) {
            if (go)
                e = launch_mfma_tile(a, dev, &parts_used, st, true, epi);
        } else if (!epi && mfma_tile_phased_preferred(a, dev, splitk_ws != nullptr && mfma_tiled_split_can_run(a, dev))) {
            if (go)
                e = launch_mfma_tile_phased(a, dev, st, true);
        } else if (splitk_ws && mfma_tiled_split_can_run(a, dev)) {
            if (go)
                e = launch_mfma(a, dev, splitk_ws, &parts_used, st, false, epi, true);
        } else {
            return fail(MXFP4_ERR_ARG, "the tile-major product needs a pass's activation rows (%lld x K=%lld) to fit "
                                       "the LDS, or a workspace of mxfp4_woq_gemm_workspace_bytes to split K; "
                                       "else use the canonical tensors for this shape",
                        (long long)(M > 16 ? 16 : M), (long long)K);
        }
        break;
    }
    case MXFP4_PATH_VALU_BITS:
    case MXFP4_PATH_VALU_CVT:
    case MXFP4_PATH_VALU_LUT:
        if ((size_t)K * 2 + (chosen == MXFP4_PATH_VALU_LUT ? 32768u : 0u) > (size_t)dev.lds_bytes)
            return fail(MXFP4_ERR_SHAPE, "K=%lld does not fit the LDS copy of one activation row",
                        (long long)K);
        if (go)
            e = launch_gemv(a, chosen, argmax, dev, &parts_used, st, epi);
        break;
    case MXFP4_PATH_VALU_REG:
        if (!gemv_reg_can_run(a, dev))
            return fail(MXFP4_ERR_ARG, "the register-resident GEMV needs K %% 128 == 0, K <= 12288 and N >= %d",
                        dev.cus * 8);
        if (go)
            e = launch_gemv_reg(a, dev, &parts_used, st, epi);
        break;
    case MXFP4_PATH_MFMA:
    case MXFP4_PATH_MFMA_GENERAL:
        if (!mfma_can_run(a, dev, splitk_ws != nullptr))
            return fail(MXFP4_ERR_ARG, "the MFMA path needs K %% 128 == 0 and, without a workspace, four rows of "
                                       "K=%lld elements exceed the LDS", (long long)K);
        if (go)
            e = launch_mfma(a, dev, splitk_ws, &parts_used, st, chosen == MXFP4_PATH_MFMA_GENERAL, epi);
        break;
    default:
        return fail(MXFP4_ERR_ARG, "unknown or unavailable path %d", chosen);
    }
    if (e != hipSuccess)
        return hip_fail(e, "product launch");
    if (argmax && go) {
        e = verify ? launch_verify_finish(a.part_val, a.part_idx, a.parts, parts_used, a.m, verify->draft,
                                          argmax_out, max_out, verify->accept_out, st)
                   : launch_argmax_finish(a.part_val, a.part_idx, a.parts, parts_used, a.m, argmax_out, max_out, st);
        if (e != hipSuccess)
            return hip_fail(e, "argmax finish launch");
    }
    return MXFP4_OK;
}

// ---- BF16-weight product ----------------------------------------------------------------

extern "C" size_t mxfp4_bf16_gemm_argmax_workspace_bytes(int64_t M, int64_t N, int64_t K);

static int run_bf16(const void* x, int64_t M, int64_t ldx, const void* w, int64_t N, int64_t K, int64_t ldw,
                    void* y, int64_t ldy, int32_t* argmax_out, float* max_out, void* workspace,
                    size_t workspace_bytes, bool argmax, void* stream, const Verify* verify = nullptr)
{
    begin_call();
    if (int vrc = check_verify(verify, M))
        return vrc;
    if (!w)
        return fail(MXFP4_ERR_NULL, "w_bf16 is NULL");
    if (N < 1 || N > 0x7FFFFFFF / 8)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 8 || K % 8 != 0 || K > MXFP4_MAX_K)
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a multiple of 8 in [8, %d]", (long long)K, MXFP4_MAX_K);
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (((N - 1) * ldw + K) * 2 > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "%lld bytes of weights exceed 2 GiB - 1", (long long)(((N - 1) * ldw + K) * 2));
    if (ldw % 8 != 0 || !aligned(w, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    int rc = check_x(x, M, ldx, K);
    if (rc)
        return rc;
    DeviceInfo dev;
    rc = device_info(&dev);
    if (rc)
        return rc;
    Bf16Args a{};
    a.x = static_cast<const uint16_t*>(x);
    a.ldx = ldx;
    a.w = static_cast<const uint16_t*>(w);
    a.ldw = ldw;
    a.m = (int)M;
    a.n = (int)N;
    a.k = (int)K;
    if (argmax) {
        if (!argmax_out)
            return fail(MXFP4_ERR_NULL, "argmax_out is NULL");
        const size_t need = mxfp4_bf16_gemm_argmax_workspace_bytes(M, N, K);
        if (!workspace || workspace_bytes < need)
            return fail(MXFP4_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
        if (!aligned(workspace, 8))
            return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
        a.parts = gemv_max_parts(dev);
        a.part_val = static_cast<float*>(workspace);
        a.part_idx = reinterpret_cast<int32_t*>(a.part_val + (size_t)M * a.parts);
    } else {
        if (!y)
            return fail(MXFP4_ERR_NULL, "y_bf16 is NULL");
        if (ldy < N)
            return fail(MXFP4_ERR_SHAPE, "ldy=%lld < N=%lld", (long long)ldy, (long long)N);
        a.y = static_cast<uint16_t*>(y);
        a.ldy = ldy;
    }
    if (!bf16_can_run(a, dev))
        return fail(MXFP4_ERR_SHAPE, "K=%lld does not fit the LDS copy of one activation row", (long long)K);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int parts_used = 0;
    hipError_t e = launch_bf16_gemv(a, dev, &parts_used, st);
    if (e != hipSuccess)
        return hip_fail(e, "BF16 product launch");
    if (argmax) {
        e = verify ? launch_verify_finish(a.part_val, a.part_idx, a.parts, parts_used, a.m, verify->draft,
                                          argmax_out, max_out, verify->accept_out, st)
                   : launch_argmax_finish(a.part_val, a.part_idx, a.parts, parts_used, a.m, argmax_out, max_out, st);
        if (e != hipSuccess)
            return hip_fail(e, "argmax finish launch");
    }
    return MXFP4_OK;
}

// ---- plain streaming kernels ------------------------------------------------------------

// Loads carry the streaming hint, as the product kernels' weight loads do: worth 10 to 25 % on a
// read stream here (5.6 -> 7.0 TB/s over 4 GiB).
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink)
{
    typedef __attribute__((ext_vector_type(4))) unsigned int v4;
    const v4* p = reinterpret_cast<const v4*>(src);
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const v4 a = __builtin_nontemporal_load(p + i), b = __builtin_nontemporal_load(p + i + stride),
                 c = __builtin_nontemporal_load(p + i + 2 * stride), d = __builtin_nontemporal_load(p + i + 3 * stride);
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3] ^ c[0] ^ c[1] ^ c[2] ^ c[3] ^ d[0] ^ d[1] ^ d[2] ^ d[3];
    }
    for (; i < n16; i += stride) {
        const v4 a = __builtin_nontemporal_load(p + i);
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3];
    }
    if (acc == 0x9E3779B9u)                          // practically never: keeps the loads alive
        sink[0] = acc;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src,
                                                          uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, const DeviceInfo& dev,
                              hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    // two workgroups per compute unit: more lowers the rate (measured 7.1 TB/s at 2, 6.1 at 8)
    hipLaunchKernelGGL(stream_read_kernel, dim3(dev.cus * 2), dim3(256), 0, stream,
                       static_cast<const uint4*>(src), n16, static_cast<uint32_t*>(sink));
    return hipGetLastError();
}

hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, const DeviceInfo& dev,
                              hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(dev.cus * 8), dim3(256), 0, stream,
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
    return hipGetLastError();
}

}  // namespace mxfp4

using namespace mxfp4;

extern "C" {

static int cast_impl(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q_packed, void* scales_e8m0,
                     bool integer_rule, void* stream)
{
    begin_call();
    if (N < 0 || N > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > (1 << 24))
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a positive multiple of 32", (long long)K);
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (N == 0)
        return MXFP4_OK;
    if (!w_bf16 || !q_packed || !scales_e8m0)
        return fail(MXFP4_ERR_NULL, "w_bf16, q_packed or scales_e8m0 is NULL");
    if (ldw % 8 != 0 || !aligned(w_bf16, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    if (!aligned(q_packed, 4))
        return fail(MXFP4_ERR_ALIGN, "q_packed must be 4-byte aligned");
    hipError_t e = launch_direct_cast(w_bf16, N, K, ldw, q_packed, scales_e8m0, integer_rule,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "direct cast launch");
}

int mxfp4_direct_cast(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q_packed,
                      void* scales_e8m0, void* stream)
{
    return cast_impl(w_bf16, N, K, ldw, q_packed, scales_e8m0, false, stream);
}

int mxfp4_direct_cast_bits(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q_packed,
                           void* scales_e8m0, void* stream)
{
    return cast_impl(w_bf16, N, K, ldw, q_packed, scales_e8m0, true, stream);
}

static int dequant_impl(const void* q, const void* s, int64_t N, int64_t K, void* w, int64_t ldw, bool hw,
                        void* stream)
{
    begin_call();
    if (N == 0)
        return MXFP4_OK;
    int rc = check_weights(q, s, N, K);
    if (rc)
        return rc;
    if (!w)
        return fail(MXFP4_ERR_NULL, "w_bf16 is NULL");
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (ldw % 8 != 0 || !aligned(w, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    hipError_t e = launch_dequant(q, s, N, K, w, ldw, hw, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "dequant launch");
}

int mxfp4_dequant(const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K, void* w_bf16,
                  int64_t ldw, void* stream)
{
    return dequant_impl(q_packed, scales_e8m0, N, K, w_bf16, ldw, false, stream);
}

int mxfp4_dequant_hwcvt(const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K, void* w_bf16,
                        int64_t ldw, void* stream)
{
    return dequant_impl(q_packed, scales_e8m0, N, K, w_bf16, ldw, true, stream);
}

int mxfp4_woq_gemm(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                   const void* scales_e8m0, int64_t N, int64_t K, void* y_bf16, int64_t ldy, void* stream)
{
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, y_bf16, ldy, nullptr, nullptr, nullptr, 0,
                    false, MXFP4_PATH_AUTO, stream);
}

int mxfp4_woq_gemm_ws(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                      const void* scales_e8m0, int64_t N, int64_t K, void* y_bf16, int64_t ldy,
                      void* workspace, size_t workspace_bytes, int path, void* stream)
{
    if (workspace && !aligned(workspace, 8)) {
        begin_call();
        return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
    }
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, y_bf16, ldy, nullptr, nullptr, workspace,
                    workspace_bytes, false, path, stream);
}

int mxfp4_woq_gemm_fused(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                         const void* scales_e8m0, int64_t N, int64_t K, const void* bias_bf16, int act,
                         const void* residual_bf16, int64_t ldr, void* y_bf16, int64_t ldy, void* workspace,
                         size_t workspace_bytes, int path, void* stream)
{
    begin_call();
    if (workspace && !aligned(workspace, 8))
        return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
    Epilogue epi{static_cast<const uint16_t*>(bias_bf16), static_cast<const uint16_t*>(residual_bf16), 0, act};
    if (residual_bf16) {
        const int64_t C = act == MXFP4_ACT_SWIGLU ? N / 2 : N;
        if (ldr < C || ldr > 0x7FFFFFFF)
            return fail(MXFP4_ERR_SHAPE, "ldr=%lld must be in [%lld, 2^31)", (long long)ldr, (long long)C);
        epi.ldr = (int)ldr;
    }
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, y_bf16, ldy, nullptr, nullptr, workspace,
                    workspace_bytes, false, path, stream, nullptr, false, &epi);
}

// ---- a sequence of products in one call -----------------------------------------------------

static int grouped_one(const mxfp4_gemm_desc& d, void* workspace, size_t workspace_bytes, void* stream)
{
    if ((d.flags & ~(MXFP4_DESC_TILED | MXFP4_DESC_INDEPENDENT)) != 0) {
        begin_call();
        return fail(MXFP4_ERR_ARG, "unknown flags %#x", (unsigned)d.flags);
    }
    const bool tiled = (d.flags & MXFP4_DESC_TILED) != 0;
    if (d.argmax_out) {
        if (d.y_bf16 || d.bias_bf16 || d.residual_bf16 || d.act != MXFP4_ACT_NONE) {
            begin_call();
            return fail(MXFP4_ERR_ARG, "a descriptor with argmax_out takes no y, bias, residual or act");
        }
        if (tiled)
            return mxfp4_woq_gemm_tiled_argmax(d.x_bf16, d.M, d.ldx, d.q_packed, d.scales_e8m0, d.N, d.K,
                                               d.argmax_out, d.max_out, workspace, workspace_bytes, stream);
        return mxfp4_woq_gemm_argmax(d.x_bf16, d.M, d.ldx, d.q_packed, d.scales_e8m0, d.N, d.K, d.argmax_out,
                                     d.max_out, workspace, workspace_bytes, stream);
    }
    if (tiled) {
        if (d.bias_bf16 || d.residual_bf16 || d.act != MXFP4_ACT_NONE)
            return mxfp4_woq_gemm_tiled_fused(d.x_bf16, d.M, d.ldx, d.q_packed, d.scales_e8m0, d.N, d.K, d.bias_bf16,
                                              d.act, d.residual_bf16, d.ldr, d.y_bf16, d.ldy, stream);
        return mxfp4_woq_gemm_tiled_ws(d.x_bf16, d.M, d.ldx, d.q_packed, d.scales_e8m0, d.N, d.K, d.y_bf16, d.ldy,
                                       workspace, workspace_bytes, stream);
    }
    if (d.bias_bf16 || d.residual_bf16 || d.act != MXFP4_ACT_NONE)
        return mxfp4_woq_gemm_fused(d.x_bf16, d.M, d.ldx, d.q_packed, d.scales_e8m0, d.N, d.K, d.bias_bf16, d.act,
                                    d.residual_bf16, d.ldr, d.y_bf16, d.ldy, workspace, workspace_bytes,
                                    MXFP4_PATH_AUTO, stream);
    return mxfp4_woq_gemm_ws(d.x_bf16, d.M, d.ldx, d.q_packed, d.scales_e8m0, d.N, d.K, d.y_bf16, d.ldy, workspace,
                             workspace_bytes, MXFP4_PATH_AUTO, stream);
}

// How many descriptors from descs[0] on can share one launch (0 or 1: none).  Only descriptors that
// have passed the checks of their single call come here.
static int merged_run(const mxfp4_gemm_desc* descs, int64_t left, const DeviceInfo& dev, void* workspace,
                      GemmArgs* items)
{
    int run = 0;
    for (int j = 0; j < kMultiMax && j < left; ++j) {
        const mxfp4_gemm_desc& d = descs[j];
        if (d.flags != MXFP4_DESC_INDEPENDENT || d.M != 1 || d.bias_bf16 || d.residual_bf16 ||
            d.act != MXFP4_ACT_NONE)
            break;
        GemmArgs a{};
        a.x = static_cast<const uint16_t*>(d.x_bf16);
        a.ldx = d.ldx;
        a.q = static_cast<const uint8_t*>(d.q_packed);
        a.s = static_cast<const uint8_t*>(d.scales_e8m0);
        a.m = 1;
        a.n = (int)d.N;
        a.k = (int)d.K;
        if (d.argmax_out) {
            a.parts = gemv_max_parts(dev);
            a.part_val = static_cast<float*>(workspace);
            a.part_idx = reinterpret_cast<int32_t*>(a.part_val + a.parts);
        } else {
            a.y = static_cast<uint16_t*>(d.y_bf16);
            a.ldy = d.ldy;
        }
        items[j] = a;
        if (j > 0 && !gemv_multi_can_run(items, j + 1, dev))
            break;
        run = j + 1;
    }
    return run;
}

size_t mxfp4_woq_gemm_grouped_workspace_bytes(const mxfp4_gemm_desc* descs, int64_t count)
{
    size_t need = 0;
    if (!descs || count < 1 || count > (1 << 20))
        return 0;
    for (int64_t i = 0; i < count; ++i) {
        const size_t b = descs[i].argmax_out
                             ? mxfp4_woq_gemm_argmax_workspace_bytes(descs[i].M, descs[i].N, descs[i].K)
                             : mxfp4_woq_gemm_workspace_bytes(descs[i].M, descs[i].N, descs[i].K);
        need = b > need ? b : need;
    }
    return need;
}

int mxfp4_woq_gemm_grouped(const mxfp4_gemm_desc* descs, int64_t count, void* workspace, size_t workspace_bytes,
                           void* stream)
{
    begin_call();
    if (count < 0 || count > (1 << 20))
        return fail(MXFP4_ERR_SHAPE, "count=%lld out of range", (long long)count);
    if (count == 0)
        return MXFP4_OK;
    if (!descs)
        return fail(MXFP4_ERR_NULL, "descs is NULL");
    // first pass: every check of the single calls and nothing launched; second pass: the launches
    DeviceInfo dev{};
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {                                    // (the checks have asked for the device already)
            const int rc = device_info(&dev);
            if (rc)
                return rc;
        }
        for (int64_t i = 0; i < count; ++i) {
            GemmArgs items[kMultiMax];
            const int run = pass == 1 ? merged_run(descs + i, count - i, dev, workspace, items) : 0;
            if (run >= 2) {
                hipStream_t st = static_cast<hipStream_t>(stream);
                int parts_used = 0;
                hipError_t e = launch_gemv_multi(items, run, dev, &parts_used, st);
                if (e != hipSuccess)
                    return hip_fail(e, "merged product launch");
                for (int j = 0; j < run; ++j)
                    if (descs[i + j].argmax_out) {
                        e = launch_argmax_finish(items[j].part_val, items[j].part_idx, items[j].parts, parts_used, 1,
                                                 descs[i + j].argmax_out, descs[i + j].max_out, st);
                        if (e != hipSuccess)
                            return hip_fail(e, "argmax finish launch");
                    }
                i += run - 1;
                continue;
            }
            g_check_only = pass == 0;
            const int rc = grouped_one(descs[i], workspace, workspace_bytes, stream);
            g_check_only = false;
            if (rc != MXFP4_OK) {
                char text[sizeof g_err];
                snprintf(text, sizeof text, "%s", g_err);
                return fail(rc, "descriptor %lld: %s", (long long)i, text);
            }
        }
    }
    return MXFP4_OK;
}

// ---- a chain of dependent one-token products in one persistent launch ------------------------

size_t mxfp4_woq_gemm_chain_workspace_bytes(void) { return chain_workspace_bytes(); }

int mxfp4_woq_gemm_chain_init(void* chain_ws, size_t chain_ws_bytes, void* stream)
{
    begin_call();
    if (!chain_ws)
        return fail(MXFP4_ERR_NULL, "chain_ws is NULL");
    if (chain_ws_bytes < chain_workspace_bytes())
        return fail(MXFP4_ERR_WORKSPACE, "chain workspace of %zu bytes needed, %zu given", chain_workspace_bytes(),
                    chain_ws_bytes);
    if (!aligned(chain_ws, 256))
        return fail(MXFP4_ERR_ALIGN, "chain_ws must be 256-byte aligned");
    hipError_t e = launch_chain_ws_init(chain_ws, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "chain workspace init launch");
}

int mxfp4_woq_gemm_chain(const mxfp4_gemm_desc* descs, int64_t count, void* chain_ws, size_t chain_ws_bytes,
                         const mxfp4_chain_opts* opts, void* stream)
{
    begin_call();
    if (count < 0 || count > MXFP4_CHAIN_MAX_LINKS)
        return fail(MXFP4_ERR_SHAPE, "count=%lld out of range [0, %d]", (long long)count, MXFP4_CHAIN_MAX_LINKS);
    if (count == 0)
        return MXFP4_OK;
    if (!descs)
        return fail(MXFP4_ERR_NULL, "descs is NULL");
    if (!chain_ws)
        return fail(MXFP4_ERR_NULL, "chain_ws is NULL");
    if (chain_ws_bytes < chain_workspace_bytes())
        return fail(MXFP4_ERR_WORKSPACE, "chain workspace of %zu bytes needed, %zu given", chain_workspace_bytes(),
                    chain_ws_bytes);
    if (!aligned(chain_ws, 256))
        return fail(MXFP4_ERR_ALIGN, "chain_ws must be 256-byte aligned");
    int64_t wait_us = 2000000;
    int phantom = 0, mode = MXFP4_CHAIN_AUTO;
    if (opts) {
        if (opts->wait_us < 0 || opts->wait_us > 20000000 || opts->phantom_workgroups < 0 ||
            opts->phantom_workgroups > 64 || opts->mode < MXFP4_CHAIN_AUTO || opts->mode > MXFP4_CHAIN_SEPARATE)
            return fail(MXFP4_ERR_ARG, "chain options out of range");
        if (opts->wait_us > 0)
            wait_us = opts->wait_us;
        phantom = opts->phantom_workgroups;
        mode = opts->mode;
    }
    std::vector<ChainItem> items((size_t)count);
    for (int64_t i = 0; i < count; ++i) {
        const mxfp4_gemm_desc& d = descs[i];
        auto bad = [&](int code, const char* what) {
            return fail(code, "descriptor %lld: %s", (long long)i, what);
        };
        if (d.flags != 0)
            return bad(MXFP4_ERR_ARG, "a chained product takes no flags (canonical tensors only)");
        if (d.M != 1)
            return bad(MXFP4_ERR_ARG, "a chained product has one activation row (M == 1)");
        int rc = check_weights(d.q_packed, d.scales_e8m0, d.N, d.K);
        if (rc == MXFP4_OK)
            rc = check_x(d.x_bf16, d.M, d.ldx, d.K);
        if (rc != MXFP4_OK) {
            char text[sizeof g_err];
            snprintf(text, sizeof text, "%s", g_err);
            return bad(rc, text);
        }
        if (d.act != MXFP4_ACT_NONE && d.act != MXFP4_ACT_SWIGLU)
            return bad(MXFP4_ERR_ARG, "unknown act");
        if (d.act == MXFP4_ACT_SWIGLU && d.N % 2 != 0)
            return bad(MXFP4_ERR_SHAPE, "the gate pairs rows 2c and 2c + 1: N must be even");
        if (d.argmax_out) {
            if (d.y_bf16 || d.bias_bf16 || d.residual_bf16 || d.act != MXFP4_ACT_NONE)
                return bad(MXFP4_ERR_ARG, "a descriptor with argmax_out takes no y, bias, residual or act");
            if (i != count - 1)
                return bad(MXFP4_ERR_ARG, "only the last product of a chain may carry argmax_out");
            if (!aligned(d.argmax_out, 4) || !aligned(d.max_out, 4))
                return bad(MXFP4_ERR_ALIGN, "argmax_out and max_out must be 4-byte aligned");
        } else {
            if (!d.y_bf16)
                return bad(MXFP4_ERR_NULL, "y_bf16 is NULL");
            if (!aligned(d.y_bf16, 2) || !aligned(d.bias_bf16, 2) || !aligned(d.residual_bf16, 2))
                return bad(MXFP4_ERR_ALIGN, "y_bf16, bias_bf16 and residual_bf16 must be 2-byte aligned");
        }
        ChainItem& it = items[(size_t)i];
        it.x = static_cast<const uint16_t*>(d.x_bf16);
        it.q = static_cast<const uint8_t*>(d.q_packed);
        it.s = static_cast<const uint8_t*>(d.scales_e8m0);
        it.y = static_cast<uint16_t*>(d.y_bf16);
        it.bias = static_cast<const uint16_t*>(d.bias_bf16);
        it.residual = static_cast<const uint16_t*>(d.residual_bf16);
        it.n = (int)d.N;
        it.k = (int)d.K;
        it.act = d.act;
        it.argmax_out = d.argmax_out;
        it.max_out = d.max_out;
    }
    DeviceInfo dev;
    int rc = device_info(&dev);
    if (rc)
        return rc;
    if (!chain_can_run(items.data(), (int)count, dev))
        return fail(MXFP4_ERR_ARG, "not a chain the persistent launch takes: every K %% 128 == 0, at most %d weight "
                                   "rows per compute unit and product, an activation row that fits the LDS",
                    kChainMaxChunk);
    // How many leading products run as launches of their own.  A grid barrier costs more here than
    // a launch does (4 to 5.5 us against 3 to 3.5 us per product, measured on the 7B shapes: the
    // barrier's memory operations queue behind the weight loads of their compute unit), and the LM
    // head with its pick in one persistent launch takes 20 us against 17 for the two ordinary
    // launches (the persistent kernel starts more slowly), so AUTO keeps every product apart.
    const int64_t apart = (phantom == 0 && mode != MXFP4_CHAIN_PERSISTENT) ? count : 0;
    for (int pass = 0; pass < 2 && apart > 0; ++pass) {
        // first every check of the single calls with nothing launched, then the launches
        for (int64_t i = 0; i < apart; ++i) {
            g_check_only = pass == 0;
            const int rc1 = descs[i].argmax_out
                                ? mxfp4_woq_gemm_argmax(descs[i].x_bf16, 1, descs[i].ldx, descs[i].q_packed,
                                                        descs[i].scales_e8m0, descs[i].N, descs[i].K, descs[i].argmax_out,
                                                        descs[i].max_out, static_cast<char*>(chain_ws) + chain_pick_area_offset(),
                                                        chain_workspace_bytes() - chain_pick_area_offset(), stream)
                                : grouped_one(descs[i], nullptr, 0, stream);
            g_check_only = false;
            if (rc1 != MXFP4_OK) {
                char text[sizeof g_err];
                snprintf(text, sizeof text, "%s", g_err);
                return fail(rc1, "descriptor %lld: %s", (long long)i, text);
            }
        }
    }
    if (apart < count) {
        hipError_t e = launch_chain(items.data() + apart, (int)(count - apart), dev, chain_ws, (int)(wait_us * 100),
                                    phantom, static_cast<hipStream_t>(stream));
        if (e != hipSuccess)
            return hip_fail(e, "chained product launch");
    }
    return MXFP4_OK;
}

int mxfp4_woq_gemm_tiled_fused(const void* x_bf16, int64_t M, int64_t ldx, const void* q_tiled,
                               const void* s_tiled, int64_t N, int64_t K, const void* bias_bf16, int act,
                               const void* residual_bf16, int64_t ldr, void* y_bf16, int64_t ldy, void* stream)
{
    begin_call();
    Epilogue epi{static_cast<const uint16_t*>(bias_bf16), static_cast<const uint16_t*>(residual_bf16), 0, act};
    if (residual_bf16) {
        const int64_t C = act == MXFP4_ACT_SWIGLU ? N / 2 : N;
        if (ldr < C || ldr > 0x7FFFFFFF)
            return fail(MXFP4_ERR_SHAPE, "ldr=%lld must be in [%lld, 2^31)", (long long)ldr, (long long)C);
        epi.ldr = (int)ldr;
    }
    return run_gemm(x_bf16, M, ldx, q_tiled, s_tiled, N, K, y_bf16, ldy, nullptr, nullptr, nullptr, 0, false,
                    MXFP4_PATH_AUTO, stream, nullptr, true, &epi);
}

int mxfp4_woq_gemm_path(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                        const void* scales_e8m0, int64_t N, int64_t K, void* y_bf16, int64_t ldy, int path,
                        void* stream)
{
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, y_bf16, ldy, nullptr, nullptr, nullptr, 0,
                    false, path, stream);
}

// Device facts for the size queries, which must also answer without a GPU: the target part.
static DeviceInfo size_query_device()
{
    DeviceInfo dev;
    if (device_info(&dev) != MXFP4_OK) {
        dev.cus = 256;
        dev.lds_bytes = 160 * 1024;
        begin_call();
    }
    return dev;
}

size_t mxfp4_woq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M < 1 || N < 1 || K < 32 || K > MXFP4_MAX_K || M > (1 << 20) || N > 0x7FFFFFFF / 8)
        return 0;
    return mfma_splitk_bytes((int)M, (int)N, (int)K, size_query_device());
}

size_t mxfp4_woq_gemm_argmax_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M < 1)
        return 0;
    // one (value, index) pair per activation row and per workgroup of the product kernel (the
    // bound on workgroups is 8 per compute unit), then the split-K partial products
    const DeviceInfo dev = size_query_device();
    return (size_t)M * gemv_max_parts(dev) * (sizeof(float) + sizeof(int32_t)) +
           mxfp4_woq_gemm_workspace_bytes(M, N, K);
}

// ---- 8-bit draft format ---------------------------------------------------------------------

static int e4m3_check_weights(const void* q8, const void* s, int64_t N, int64_t K)
{
    if (!q8 || !s)
        return fail(MXFP4_ERR_NULL, "q8 or scales_e8m0 is NULL");
    if (N < 1 || N > 0x7FFFFFFF / 8)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > MXFP4_MAX_K)
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a multiple of 32 in [32, %d]", (long long)K, MXFP4_MAX_K);
    if (N * K > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "N*K=%lld bytes of weights exceed 2 GiB - 1", (long long)(N * K));
    if (!aligned(q8, 16))
        return fail(MXFP4_ERR_ALIGN, "q8 must be 16-byte aligned");
    return MXFP4_OK;
}

static int e4m3_cast_impl(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q8, void* scales_e8m0,
                          bool integer_rule, void* stream)
{
    begin_call();
    if (N < 0 || N > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > (1 << 24))
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a positive multiple of 32", (long long)K);
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (N == 0)
        return MXFP4_OK;
    if (!w_bf16 || !q8 || !scales_e8m0)
        return fail(MXFP4_ERR_NULL, "w_bf16, q8 or scales_e8m0 is NULL");
    if (ldw % 8 != 0 || !aligned(w_bf16, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    if (!aligned(q8, 8))
        return fail(MXFP4_ERR_ALIGN, "q8 must be 8-byte aligned");
    hipError_t e = launch_e4m3_cast(w_bf16, N, K, ldw, q8, scales_e8m0, integer_rule,
                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "8-bit cast launch");
}

int mxfp4_e4m3_direct_cast(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q8, void* scales_e8m0,
                           void* stream)
{
    return e4m3_cast_impl(w_bf16, N, K, ldw, q8, scales_e8m0, false, stream);
}

int mxfp4_e4m3_direct_cast_bits(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q8,
                                void* scales_e8m0, void* stream)
{
    return e4m3_cast_impl(w_bf16, N, K, ldw, q8, scales_e8m0, true, stream);
}

int mxfp4_e4m3_dequant(const void* q8, const void* scales_e8m0, int64_t N, int64_t K, void* w_bf16, int64_t ldw,
                       void* stream)
{
    begin_call();
    if (N == 0)
        return MXFP4_OK;
    int rc = e4m3_check_weights(q8, scales_e8m0, N, K);
    if (rc)
        return rc;
    if (!w_bf16)
        return fail(MXFP4_ERR_NULL, "w_bf16 is NULL");
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (ldw % 8 != 0 || !aligned(w_bf16, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    hipError_t e = launch_e4m3_dequant(q8, scales_e8m0, N, K, w_bf16, ldw, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "8-bit dequant launch");
}

static int run_e4m3(const void* x, int64_t M, int64_t ldx, const void* q8, const void* s, int64_t N, int64_t K,
                    void* y, int64_t ldy, int32_t* argmax_out, float* max_out, void* workspace,
                    size_t workspace_bytes, bool argmax, void* stream)
{
    begin_call();
    int rc = e4m3_check_weights(q8, s, N, K);
    if (rc)
        return rc;
    rc = check_x(x, M, ldx, K);
    if (rc)
        return rc;
    DeviceInfo dev;
    rc = device_info(&dev);
    if (rc)
        return rc;
    GemmArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.ldx = ldx;
    a.q = static_cast<const uint8_t*>(q8);
    a.s = static_cast<const uint8_t*>(s);
    a.m = (int)M;
    a.n = (int)N;
    a.k = (int)K;
    if (!e4m3_can_run(a, dev))
        return fail(MXFP4_ERR_SHAPE, "K=%lld does not fit the LDS copy of one activation row", (long long)K);
    if (argmax) {
        if (!argmax_out)
            return fail(MXFP4_ERR_NULL, "argmax_out is NULL");
        const size_t need = (size_t)M * gemv_max_parts(dev) * 8;
        if (!workspace || workspace_bytes < need)
            return fail(MXFP4_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
        if (!aligned(workspace, 8))
            return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
        a.parts = gemv_max_parts(dev);
        a.part_val = static_cast<float*>(workspace);
        a.part_idx = reinterpret_cast<int32_t*>(a.part_val + (size_t)M * a.parts);
    } else {
        if (!y)
            return fail(MXFP4_ERR_NULL, "y_bf16 is NULL");
        if (ldy < N)
            return fail(MXFP4_ERR_SHAPE, "ldy=%lld < N=%lld", (long long)ldy, (long long)N);
        a.y = static_cast<uint16_t*>(y);
        a.ldy = ldy;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    int parts_used = 0;
    // one or two rows in one pass over the weights: the decode-step frame; else the general kernel
    static const bool general_only = [] {
        const char* e = knob("MXFP4_E4M3_GENERAL");              // measurement only
        return e && atoi(e) != 0;
    }();
    const bool reg = !general_only && aligned(s, 4) && gemv_reg_can_run(a, dev) && gemv_reg_single_pass(a);
    // five and more rows: the matrix-core tiles when a pass's activation rows fit the LDS (up to
    // four rows the vector-ALU kernel is faster: 13.5 against 16.8 us on the 7B qkv shape)
    const bool tiles = !general_only && !reg && a.m >= 5 && aligned(s, 4) && aligned(q8, 16) && mfma_tile_fmt_can_run(a, dev);
    hipError_t e = reg     ? launch_gemv_reg(a, dev, &parts_used, st, nullptr, 8)
                   : tiles ? launch_mfma_tile8(a, dev, &parts_used, st)
                           : launch_e4m3_gemv(a, dev, &parts_used, st);
    if (e != hipSuccess)
        return hip_fail(e, "8-bit product launch");
    if (argmax) {
        e = launch_argmax_finish(a.part_val, a.part_idx, a.parts, parts_used, a.m, argmax_out, max_out, st);
        if (e != hipSuccess)
            return hip_fail(e, "argmax finish launch");
    }
    return MXFP4_OK;
}

int mxfp4_e4m3_woq_gemm(const void* x_bf16, int64_t M, int64_t ldx, const void* q8, const void* scales_e8m0,
                        int64_t N, int64_t K, void* y_bf16, int64_t ldy, void* stream)
{
    return run_e4m3(x_bf16, M, ldx, q8, scales_e8m0, N, K, y_bf16, ldy, nullptr, nullptr, nullptr, 0, false, stream);
}

int mxfp4_e4m3_woq_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx, const void* q8,
                               const void* scales_e8m0, int64_t N, int64_t K, int32_t* argmax_out, float* max_out,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    return run_e4m3(x_bf16, M, ldx, q8, scales_e8m0, N, K, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, stream);
}

// ---- 6-bit draft format ---------------------------------------------------------------------

static int e2m3_check_weights(const void* q6, const void* s, int64_t N, int64_t K)
{
    if (!q6 || !s)
        return fail(MXFP4_ERR_NULL, "q6 or scales_e8m0 is NULL");
    if (N < 1 || N > 0x7FFFFFFF / 8)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > MXFP4_MAX_K)
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a multiple of 32 in [32, %d]", (long long)K, MXFP4_MAX_K);
    if (N * (K / 32) * 24 > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "%lld bytes of 6-bit weights exceed 2 GiB - 1", (long long)(N * (K / 32) * 24));
    if (!aligned(q6, 8))
        return fail(MXFP4_ERR_ALIGN, "q6 must be 8-byte aligned");
    return MXFP4_OK;
}

static int e2m3_cast_impl(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q6, void* scales_e8m0,
                          bool integer_rule, void* stream)
{
    begin_call();
    if (N < 0 || N > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > (1 << 24))
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a positive multiple of 32", (long long)K);
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (N == 0)
        return MXFP4_OK;
    if (!w_bf16 || !q6 || !scales_e8m0)
        return fail(MXFP4_ERR_NULL, "w_bf16, q6 or scales_e8m0 is NULL");
    if (ldw % 8 != 0 || !aligned(w_bf16, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    if (!aligned(q6, 8))
        return fail(MXFP4_ERR_ALIGN, "q6 must be 8-byte aligned");
    hipError_t e = launch_e2m3_cast(w_bf16, N, K, ldw, q6, scales_e8m0, integer_rule,
                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "6-bit cast launch");
}

int mxfp4_e2m3_direct_cast(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q6, void* scales_e8m0,
                           void* stream)
{
    return e2m3_cast_impl(w_bf16, N, K, ldw, q6, scales_e8m0, false, stream);
}

int mxfp4_e2m3_direct_cast_bits(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q6,
                                void* scales_e8m0, void* stream)
{
    return e2m3_cast_impl(w_bf16, N, K, ldw, q6, scales_e8m0, true, stream);
}

int mxfp4_e2m3_dequant(const void* q6, const void* scales_e8m0, int64_t N, int64_t K, void* w_bf16, int64_t ldw,
                       void* stream)
{
    begin_call();
    if (N == 0)
        return MXFP4_OK;
    int rc = e2m3_check_weights(q6, scales_e8m0, N, K);
    if (rc)
        return rc;
    if (!w_bf16)
        return fail(MXFP4_ERR_NULL, "w_bf16 is NULL");
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (ldw % 8 != 0 || !aligned(w_bf16, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    hipError_t e = launch_e2m3_dequant(q6, scales_e8m0, N, K, w_bf16, ldw, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "6-bit dequant launch");
}

static int run_e2m3(const void* x, int64_t M, int64_t ldx, const void* q6, const void* s, int64_t N, int64_t K,
                    void* y, int64_t ldy, int32_t* argmax_out, float* max_out, void* workspace,
                    size_t workspace_bytes, bool argmax, void* stream)
{
    begin_call();
    int rc = e2m3_check_weights(q6, s, N, K);
    if (rc)
        return rc;
    if (!aligned(s, 4))
        return fail(MXFP4_ERR_ALIGN, "scales_e8m0 must be 4-byte aligned");
    rc = check_x(x, M, ldx, K);
    if (rc)
        return rc;
    DeviceInfo dev;
    rc = device_info(&dev);
    if (rc)
        return rc;
    GemmArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.ldx = ldx;
    a.q = static_cast<const uint8_t*>(q6);
    a.s = static_cast<const uint8_t*>(s);
    a.m = (int)M;
    a.n = (int)N;
    a.k = (int)K;
    if (argmax) {
        if (!argmax_out)
            return fail(MXFP4_ERR_NULL, "argmax_out is NULL");
        const size_t need = (size_t)M * gemv_max_parts(dev) * 8;
        if (!workspace || workspace_bytes < need)
            return fail(MXFP4_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
        if (!aligned(workspace, 8))
            return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
        a.parts = gemv_max_parts(dev);
        a.part_val = static_cast<float*>(workspace);
        a.part_idx = reinterpret_cast<int32_t*>(a.part_val + (size_t)M * a.parts);
    } else {
        if (!y)
            return fail(MXFP4_ERR_NULL, "y_bf16 is NULL");
        if (ldy < N)
            return fail(MXFP4_ERR_SHAPE, "ldy=%lld < N=%lld", (long long)ldy, (long long)N);
        a.y = static_cast<uint16_t*>(y);
        a.ldy = ldy;
    }
    const bool reg_ok = gemv_reg_can_run(a, dev), tiles_ok = mfma_tile_fmt_can_run(a, dev);
    if (!reg_ok && !tiles_ok)
        return fail(MXFP4_ERR_SHAPE, "the 6-bit product needs K %% 128 == 0 and either four activation rows of K "
                                     "elements within the LDS or K <= 32768 with N >= %d", dev.cus * 8);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int parts_used = 0;
    // Three and more rows: the matrix-core tiles when four activation rows fit the LDS, else
    // passes of the decode kernel over the weights.  One and two rows: the decode kernel; the
    // tiles (any N) for the shapes it does not take.
    const bool tiles = tiles_ok && (a.m >= 3 || !reg_ok);
    hipError_t e = tiles ? launch_mfma_tile8(a, dev, &parts_used, st, 6)
                         : launch_gemv_reg(a, dev, &parts_used, st, nullptr, 6);
    if (e != hipSuccess)
        return hip_fail(e, "6-bit product launch");
    if (argmax) {
        e = launch_argmax_finish(a.part_val, a.part_idx, a.parts, parts_used, a.m, argmax_out, max_out, st);
        if (e != hipSuccess)
            return hip_fail(e, "argmax finish launch");
    }
    return MXFP4_OK;
}

int mxfp4_e2m3_woq_gemm(const void* x_bf16, int64_t M, int64_t ldx, const void* q6, const void* scales_e8m0,
                        int64_t N, int64_t K, void* y_bf16, int64_t ldy, void* stream)
{
    return run_e2m3(x_bf16, M, ldx, q6, scales_e8m0, N, K, y_bf16, ldy, nullptr, nullptr, nullptr, 0, false, stream);
}

int mxfp4_e2m3_woq_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx, const void* q6,
                               const void* scales_e8m0, int64_t N, int64_t K, int32_t* argmax_out, float* max_out,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    return run_e2m3(x_bf16, M, ldx, q6, scales_e8m0, N, K, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, stream);
}

// ---- the product along the rows (value side of attention over a quantised cache) --------------

size_t mxfp4_woq_gemm_t_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M < 1 || M > 64 || N < 1 || N > 0x7FFFFFFF / 8 || !gemm_t_can_run((int)(K > 0x7FFFFFFF ? 0 : K)))
        return 0;
    return gemm_t_workspace_bytes((int)M, (int)N, (int)K, size_query_device());
}

int mxfp4_woq_gemm_t(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed, const void* scales_e8m0,
                     int64_t N, int64_t K, void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                     void* stream)
{
    begin_call();
    int rc = check_weights(q_packed, scales_e8m0, N, K);
    if (rc)
        return rc;
    if (!gemm_t_can_run((int)K))
        return fail(MXFP4_ERR_SHAPE, "K=%lld: the product along the rows takes K up to 2048", (long long)K);
    if (!x_bf16 || !y_bf16)
        return fail(MXFP4_ERR_NULL, "x_bf16 or y_bf16 is NULL");
    if (M < 1 || M > 64)
        return fail(MXFP4_ERR_SHAPE, "M=%lld out of range [1, 64]", (long long)M);
    if (ldx < N)
        return fail(MXFP4_ERR_SHAPE, "ldx=%lld < N=%lld", (long long)ldx, (long long)N);
    if (ldy < K)
        return fail(MXFP4_ERR_SHAPE, "ldy=%lld < K=%lld", (long long)ldy, (long long)K);
    if (!aligned(x_bf16, 2) || !aligned(y_bf16, 2))
        return fail(MXFP4_ERR_ALIGN, "x_bf16 and y_bf16 must be 2-byte aligned");
    DeviceInfo dev;
    rc = device_info(&dev);
    if (rc)
        return rc;
    const size_t need = gemm_t_workspace_bytes((int)M, (int)N, (int)K, dev);
    if (!workspace || workspace_bytes < need)
        return fail(MXFP4_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : (size_t)0);
    if (!aligned(workspace, 4))
        return fail(MXFP4_ERR_ALIGN, "workspace must be 4-byte aligned");
    GemmArgs a{};
    a.x = static_cast<const uint16_t*>(x_bf16);
    a.ldx = ldx;
    a.q = static_cast<const uint8_t*>(q_packed);
    a.s = static_cast<const uint8_t*>(scales_e8m0);
    a.m = (int)M;
    a.n = (int)N;
    a.k = (int)K;
    a.y = static_cast<uint16_t*>(y_bf16);
    a.ldy = ldy;
    hipError_t e = launch_gemm_t(a, dev, static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "product-along-rows launch");
}

// ---- further block formats by id (E5M2, E3M2, 2-bit ternary) ---------------------------------

int mxfp4_fmt_block_bytes(int fmt) { return mxfmt_block_bytes(fmt); }

static int fmt_check_weights(int fmt, const void* q, const void* s, int64_t N, int64_t K)
{
    const int bb = mxfmt_block_bytes(fmt);
    if (bb == 0)
        return fail(MXFP4_ERR_SHAPE, "format id %d is none of MXFP4_FMT_E5M2, _E3M2, _T2", fmt);
    if (!q || !s)
        return fail(MXFP4_ERR_NULL, "q or scales_e8m0 is NULL");
    if (N < 1 || N > 0x7FFFFFFF / 8)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > MXFP4_MAX_K)
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a multiple of 32 in [32, %d]", (long long)K, MXFP4_MAX_K);
    if (N * (K / 32) * bb > 0x7FFFFF00)
        return fail(MXFP4_ERR_SHAPE, "%lld bytes of weights exceed 2 GiB - 256", (long long)(N * (K / 32) * bb));
    if (!aligned(q, 8))
        return fail(MXFP4_ERR_ALIGN, "q must be 8-byte aligned");
    return MXFP4_OK;
}

static int fmt_cast_impl(int fmt, const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q, void* scales_e8m0,
                         bool integer_rule, void* stream)
{
    begin_call();
    if (mxfmt_block_bytes(fmt) == 0)
        return fail(MXFP4_ERR_SHAPE, "format id %d is none of MXFP4_FMT_E5M2, _E3M2, _T2", fmt);
    if (N < 0 || N > 0x7FFFFFFF)
        return fail(MXFP4_ERR_SHAPE, "N=%lld out of range", (long long)N);
    if (K < 32 || K % 32 != 0 || K > (1 << 24))
        return fail(MXFP4_ERR_SHAPE, "K=%lld must be a positive multiple of 32", (long long)K);
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (N == 0)
        return MXFP4_OK;
    if (!w_bf16 || !q || !scales_e8m0)
        return fail(MXFP4_ERR_NULL, "w_bf16, q or scales_e8m0 is NULL");
    if (ldw % 8 != 0 || !aligned(w_bf16, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    if (!aligned(q, 8))
        return fail(MXFP4_ERR_ALIGN, "q must be 8-byte aligned");
    hipError_t e = launch_mxfmt_cast(fmt, w_bf16, N, K, ldw, q, scales_e8m0, integer_rule,
                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "block-format cast launch");
}

int mxfp4_fmt_direct_cast(int fmt, const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q,
                          void* scales_e8m0, void* stream)
{
    return fmt_cast_impl(fmt, w_bf16, N, K, ldw, q, scales_e8m0, false, stream);
}

int mxfp4_fmt_direct_cast_bits(int fmt, const void* w_bf16, int64_t N, int64_t K, int64_t ldw, void* q,
                               void* scales_e8m0, void* stream)
{
    return fmt_cast_impl(fmt, w_bf16, N, K, ldw, q, scales_e8m0, true, stream);
}

int mxfp4_fmt_dequant(int fmt, const void* q, const void* scales_e8m0, int64_t N, int64_t K, void* w_bf16,
                      int64_t ldw, void* stream)
{
    begin_call();
    if (N == 0 && mxfmt_block_bytes(fmt) != 0)
        return MXFP4_OK;
    int rc = fmt_check_weights(fmt, q, scales_e8m0, N, K);
    if (rc)
        return rc;
    if (!w_bf16)
        return fail(MXFP4_ERR_NULL, "w_bf16 is NULL");
    if (ldw < K)
        return fail(MXFP4_ERR_SHAPE, "ldw=%lld < K=%lld", (long long)ldw, (long long)K);
    if (ldw % 8 != 0 || !aligned(w_bf16, 16))
        return fail(MXFP4_ERR_ALIGN, "w_bf16 must be 16-byte aligned with ldw %% 8 == 0");
    hipError_t e = launch_mxfmt_dequant(fmt, q, scales_e8m0, N, K, w_bf16, ldw, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "block-format dequant launch");
}

static int run_fmt(int fmt, const void* x, int64_t M, int64_t ldx, const void* q, const void* s, int64_t N,
                   int64_t K, void* y, int64_t ldy, int32_t* argmax_out, float* max_out, void* workspace,
                   size_t workspace_bytes, bool argmax, void* stream)
{
    begin_call();
    int rc = fmt_check_weights(fmt, q, s, N, K);
    if (rc)
        return rc;
    rc = check_x(x, M, ldx, K);
    if (rc)
        return rc;
    DeviceInfo dev;
    rc = device_info(&dev);
    if (rc)
        return rc;
    GemmArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.ldx = ldx;
    a.q = static_cast<const uint8_t*>(q);
    a.s = static_cast<const uint8_t*>(s);
    a.m = (int)M;
    a.n = (int)N;
    a.k = (int)K;
    if (!mxfmt_can_run(a, dev))
        return fail(MXFP4_ERR_SHAPE, "K=%lld does not fit the LDS copy of one activation row", (long long)K);
    if (argmax) {
        if (!argmax_out)
            return fail(MXFP4_ERR_NULL, "argmax_out is NULL");
        const size_t need = (size_t)M * gemv_max_parts(dev) * 8;
        if (!workspace || workspace_bytes < need)
            return fail(MXFP4_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
        if (!aligned(workspace, 8))
            return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
        a.parts = gemv_max_parts(dev);
        a.part_val = static_cast<float*>(workspace);
        a.part_idx = reinterpret_cast<int32_t*>(a.part_val + (size_t)M * a.parts);
    } else {
        if (!y)
            return fail(MXFP4_ERR_NULL, "y_bf16 is NULL");
        if (ldy < N)
            return fail(MXFP4_ERR_SHAPE, "ldy=%lld < N=%lld", (long long)ldy, (long long)N);
        a.y = static_cast<uint16_t*>(y);
        a.ldy = ldy;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    int parts_used = 0;
    // One or two rows in one pass over the weights: the decode-step frame -- E5M2 and E3M2 that of their
    // sibling formats with the other convert instruction (a lane's 24 bytes of a 6-bit block need the
    // scale bytes 4-byte aligned there), the 2-bit codes with their own decode; everything else: the
    // general kernel
    const bool reg = aligned(s, 4) && aligned(q, 16) && gemv_reg_can_run(a, dev) && gemv_reg_single_pass(a);
    // three and more rows when a pass's activation rows fit the LDS: the matrix-core tiles of the
    // sibling formats (E5M2 at four rows on the 7B qkv shape: 16.8 us there, 20.9 in the general kernel)
    const bool tiles = fmt != MXFP4_FMT_T2 && !reg && a.m >= 3 && a.k % 128 == 0 &&
                       aligned(s, 4) && aligned(q, 16) && mfma_tile_fmt_can_run(a, dev);
    const int code = fmt == MXFP4_FMT_E5M2 ? 24 : (fmt == MXFP4_FMT_E3M2 ? 22 : 2);
    hipError_t e = reg     ? launch_gemv_reg(a, dev, &parts_used, st, nullptr, code)
                   : tiles ? launch_mfma_tile8(a, dev, &parts_used, st, code)
                           : launch_mxfmt_gemv(fmt, a, dev, &parts_used, st);
    if (e != hipSuccess)
        return hip_fail(e, "block-format product launch");
    if (argmax) {
        e = launch_argmax_finish(a.part_val, a.part_idx, a.parts, parts_used, a.m, argmax_out, max_out, st);
        if (e != hipSuccess)
            return hip_fail(e, "argmax finish launch");
    }
    return MXFP4_OK;
}

int mxfp4_fmt_woq_gemm(int fmt, const void* x_bf16, int64_t M, int64_t ldx, const void* q,
                       const void* scales_e8m0, int64_t N, int64_t K, void* y_bf16, int64_t ldy, void* stream)
{
    return run_fmt(fmt, x_bf16, M, ldx, q, scales_e8m0, N, K, y_bf16, ldy, nullptr, nullptr, nullptr, 0, false,
                   stream);
}

int mxfp4_fmt_woq_gemm_argmax(int fmt, const void* x_bf16, int64_t M, int64_t ldx, const void* q,
                              const void* scales_e8m0, int64_t N, int64_t K, int32_t* argmax_out, float* max_out,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    return run_fmt(fmt, x_bf16, M, ldx, q, scales_e8m0, N, K, nullptr, 0, argmax_out, max_out, workspace,
                   workspace_bytes, true, stream);
}

int mxfp4_bf16_gemm(const void* x_bf16, int64_t M, int64_t ldx, const void* w_bf16, int64_t N, int64_t K,
                    int64_t ldw, void* y_bf16, int64_t ldy, void* stream)
{
    return run_bf16(x_bf16, M, ldx, w_bf16, N, K, ldw, y_bf16, ldy, nullptr, nullptr, nullptr, 0, false, stream);
}

size_t mxfp4_bf16_gemm_argmax_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    (void)N;
    (void)K;
    if (M < 1)
        return 0;
    return (size_t)M * gemv_max_parts(size_query_device()) * (sizeof(float) + sizeof(int32_t));
}

int mxfp4_bf16_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx, const void* w_bf16, int64_t N,
                           int64_t K, int64_t ldw, int32_t* argmax_out, float* max_out, void* workspace,
                           size_t workspace_bytes, void* stream)
{
    return run_bf16(x_bf16, M, ldx, w_bf16, N, K, ldw, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, stream);
}

int mxfp4_woq_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                          const void* scales_e8m0, int64_t N, int64_t K, int32_t* argmax_out,
                          float* max_out, void* workspace, size_t workspace_bytes, void* stream)
{
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, MXFP4_PATH_AUTO, stream);
}

// The fused pick for callers that cannot allocate: the scratch of mxfp4_woq_gemm_argmax lives in
// device memory of the library's own, one array per device, which the device holds from the moment
// the library is loaded until the process ends.  In host code the array's name is only a handle for
// the symbol; its address on the current device comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static int static_scratch(void** out)
{
    static void* ptr[64];
    static std::atomic<bool> have[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64)
        return fail(MXFP4_ERR_HIP, "device ordinal %d out of range", dev);
    if (!have[dev].load(std::memory_order_acquire)) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return hip_fail(e, "hipGetSymbolAddress(scratch)");
        ptr[dev] = p;                               // (racing threads store the same address)
        have[dev].store(true, std::memory_order_release);
    }
    *out = ptr[dev];
    return MXFP4_OK;
}

size_t mxfp4_woq_gemm_argmax_noalloc_max_bytes(void) { return kStaticScratchBytes; }

int mxfp4_woq_gemm_argmax_noalloc(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                                  const void* scales_e8m0, int64_t N, int64_t K, int32_t* argmax_out,
                                  float* max_out, void* stream)
{
    begin_call();
    const size_t need = mxfp4_woq_gemm_argmax_workspace_bytes(M, N, K);
    if (need > kStaticScratchBytes)
        return fail(MXFP4_ERR_WORKSPACE, "this shape needs %zu bytes of scratch, the library's own buffer holds %zu: "
                                         "use mxfp4_woq_gemm_argmax with a workspace", need, kStaticScratchBytes);
    void* ws = nullptr;
    if (int rc = static_scratch(&ws))
        return rc;
    // nothing in the buffer has to start at zero: every partial winner that the second stage
    // reads has been written by this call's product kernel
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, nullptr, 0, argmax_out, max_out, ws,
                    kStaticScratchBytes, true, MXFP4_PATH_AUTO, stream);
}

int mxfp4_woq_gemm_argmax_path(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                               const void* scales_e8m0, int64_t N, int64_t K, int32_t* argmax_out,
                               float* max_out, void* workspace, size_t workspace_bytes, int path,
                               void* stream)
{
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, path, stream);
}

size_t mxfp4_tile_repack_q_bytes(int64_t N, int64_t K)
{
    return (N < 1 || K < 128 || K % 128 != 0) ? 0 : tile_repack_q_bytes(N, K);
}

size_t mxfp4_tile_repack_s_bytes(int64_t N, int64_t K)
{
    return (N < 1 || K < 128 || K % 128 != 0) ? 0 : tile_repack_s_bytes(N, K);
}

int mxfp4_tile_repack(const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K, void* q_tiled,
                      void* s_tiled, void* stream)
{
    begin_call();
    int rc = check_weights(q_packed, scales_e8m0, (N + 15) / 16 * 16, K);
    if (rc)
        return rc;
    if (K % 128 != 0)
        return fail(MXFP4_ERR_SHAPE, "tile-major weights need K %% 128 == 0, K=%lld", (long long)K);
    if (!q_tiled || !s_tiled)
        return fail(MXFP4_ERR_NULL, "q_tiled or s_tiled is NULL");
    if (!aligned(q_tiled, 16) || !aligned(s_tiled, 16))
        return fail(MXFP4_ERR_ALIGN, "q_tiled and s_tiled must be 16-byte aligned");
    hipError_t e = launch_tile_repack(q_packed, scales_e8m0, (int)N, (int)K, q_tiled, s_tiled,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "tile repack launch");
}

int mxfp4_woq_gemm_tiled(const void* x_bf16, int64_t M, int64_t ldx, const void* q_tiled, const void* s_tiled,
                         int64_t N, int64_t K, void* y_bf16, int64_t ldy, void* stream)
{
    return run_gemm(x_bf16, M, ldx, q_tiled, s_tiled, N, K, y_bf16, ldy, nullptr, nullptr, nullptr, 0, false,
                    MXFP4_PATH_AUTO, stream, nullptr, true);
}

int mxfp4_woq_gemm_tiled_ws(const void* x_bf16, int64_t M, int64_t ldx, const void* q_tiled, const void* s_tiled,
                            int64_t N, int64_t K, void* y_bf16, int64_t ldy, void* workspace,
                            size_t workspace_bytes, void* stream)
{
    if (workspace && !aligned(workspace, 8)) {
        begin_call();
        return fail(MXFP4_ERR_ALIGN, "workspace must be 8-byte aligned");
    }
    return run_gemm(x_bf16, M, ldx, q_tiled, s_tiled, N, K, y_bf16, ldy, nullptr, nullptr, workspace,
                    workspace_bytes, false, MXFP4_PATH_AUTO, stream, nullptr, true);
}

int mxfp4_woq_gemm_tiled_argmax(const void* x_bf16, int64_t M, int64_t ldx, const void* q_tiled,
                                const void* s_tiled, int64_t N, int64_t K, int32_t* argmax_out, float* max_out,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    return run_gemm(x_bf16, M, ldx, q_tiled, s_tiled, N, K, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, MXFP4_PATH_AUTO, stream, nullptr, true);
}

int mxfp4_woq_gemm_tiled_verify(const void* x_bf16, int64_t M, int64_t ldx, const void* q_tiled,
                                const void* s_tiled, int64_t N, int64_t K, const int32_t* draft_tokens,
                                int32_t* accept_out, int32_t* argmax_out, float* max_out, void* workspace,
                                size_t workspace_bytes, void* stream)
{
    const Verify v{draft_tokens, accept_out};
    return run_gemm(x_bf16, M, ldx, q_tiled, s_tiled, N, K, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, MXFP4_PATH_AUTO, stream, &v, true);
}

int mxfp4_woq_gemm_verify(const void* x_bf16, int64_t M, int64_t ldx, const void* q_packed,
                          const void* scales_e8m0, int64_t N, int64_t K, const int32_t* draft_tokens,
                          int32_t* accept_out, int32_t* argmax_out, float* max_out, void* workspace,
                          size_t workspace_bytes, void* stream)
{
    const Verify v{draft_tokens, accept_out};
    return run_gemm(x_bf16, M, ldx, q_packed, scales_e8m0, N, K, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, MXFP4_PATH_AUTO, stream, &v);
}

int mxfp4_bf16_gemm_verify(const void* x_bf16, int64_t M, int64_t ldx, const void* w_bf16, int64_t N,
                           int64_t K, int64_t ldw, const int32_t* draft_tokens, int32_t* accept_out,
                           int32_t* argmax_out, float* max_out, void* workspace, size_t workspace_bytes,
                           void* stream)
{
    const Verify v{draft_tokens, accept_out};
    return run_bf16(x_bf16, M, ldx, w_bf16, N, K, ldw, nullptr, 0, argmax_out, max_out, workspace,
                    workspace_bytes, true, stream, &v);
}

int mxfp4_diag_stream_read(const void* src, size_t bytes, void* sink4, void* stream)
{
    begin_call();
    if (!src || !sink4)
        return fail(MXFP4_ERR_NULL, "src or sink is NULL");
    if (!aligned(src, 16) || bytes % 16 != 0)
        return fail(MXFP4_ERR_ALIGN, "src must be 16-byte aligned and bytes a multiple of 16");
    DeviceInfo dev;
    int rc = device_info(&dev);
    if (rc)
        return rc;
    hipError_t e = launch_stream_read(src, bytes, sink4, dev, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "stream read launch");
}

int mxfp4_diag_stream_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    begin_call();
    if (!src || !dst)
        return fail(MXFP4_ERR_NULL, "src or dst is NULL");
    if (!aligned(src, 16) || !aligned(dst, 16) || bytes % 16 != 0)
        return fail(MXFP4_ERR_ALIGN, "src/dst must be 16-byte aligned and bytes a multiple of 16");
    DeviceInfo dev;
    int rc = device_info(&dev);
    if (rc)
        return rc;
    hipError_t e = launch_stream_copy(src, dst, bytes, dev, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MXFP4_OK : hip_fail(e, "stream copy launch");
}

const char* mxfp4_last_error(void) { return g_err; }

const char* mxfp4_version(void) { return "mxfp4-gfx950 0.1"; }

}  // extern "C"
