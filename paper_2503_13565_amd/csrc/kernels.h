// Internal launch interface between the C ABI (api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mxfp4 {

// Arguments of one skinny product launch; see include/mxfp4.h for the tensor layouts.
struct GemmArgs {
    const uint16_t* x;   // BF16 [M, K], row stride ldx
    int64_t ldx;
    const uint8_t* q;    // packed nibbles [N, K/2]
    const uint8_t* s;    // scale bytes [N, K/32]
    int m;               // activation rows
    int n;               // output features
    int k;               // reduction length, multiple of 32
    uint16_t* y;         // BF16 [M, N], row stride ldy; unused by the argmax form
    int64_t ldy;
    // argmax form: per-workgroup partial winners [M, parts] written by the product kernel
    float* part_val;
    int32_t* part_idx;
    int parts;           // capacity per row of the two arrays above
    // split-K form of the MFMA path: FP32 partial products [phases, M, N]; the K range is cut
    // into `phases` runs of `phase_steps` steps of 128 elements, one per workgroup row (grid y)
    float* splitk_ws;
    int phases;
    int phase_steps;
};

// What is fused behind the contraction (see mxfp4_woq_gemm_fused in include/mxfp4.h):
// z = product + bias[n]; gated: t[c] = silu(z[2c]) * z[2c + 1] (C = N / 2 outputs per row),
// else t = z; y = t + residual[m][c].  y then has C columns.
struct Epilogue {
    const uint16_t* bias;       // BF16 [N] or null
    const uint16_t* residual;   // BF16 [M, C], row stride ldr, or null; may be y itself
    int ldr;
    int act;                    // MXFP4_ACT_NONE or MXFP4_ACT_SWIGLU
};
struct NoEpilogue {};

struct DeviceInfo {
    int cus;             // compute units
    int lds_bytes;       // LDS per workgroup the device allows
};

// `integer_rule`: round the elements with the integer-only rule instead of the convert instruction.
hipError_t launch_direct_cast(const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q, void* s,
                              bool integer_rule, hipStream_t stream);
hipError_t launch_dequant(const void* q, const void* s, int64_t n_rows, int64_t k, void* w, int64_t ldw,
                          bool hw_convert, hipStream_t stream);

// Wave-per-row-group product on the vector ALUs.  `decode` is one of MXFP4_PATH_VALU_*.
// Handles any M by passing over the weights once per group of activation rows.
// `parts_used` receives the number of partial winners written per row (argmax form).
// `epi`: the fused form (MXFP4_PATH_VALU_CVT only).
hipError_t launch_gemv(const GemmArgs& a, int decode, bool argmax, const DeviceInfo& dev,
                       int* parts_used, hipStream_t stream, const Epilogue* epi = nullptr);
int gemv_max_parts(const DeviceInfo& dev);

// The decode-step form of the same product (converts + dot2, activations in registers, one
// workgroup per compute unit, rows dealt to the waves through an LDS counter); see gemv_reg.hip
// for the shapes it takes.  The argmax form writes one partial winner per workgroup.
bool gemv_reg_can_run(const GemmArgs& a, const DeviceInfo& dev);
bool gemv_reg_single_pass(const GemmArgs& a);     // all activation rows in one pass over the weights
// Several independent one-token products of one K in one launch (y, or part_val/part_idx/parts for
// at most one of them, per item); see gemv_reg.hip.
constexpr int kMultiMax = 8;
bool gemv_multi_can_run(const GemmArgs* items, int count, const DeviceInfo& dev);
hipError_t launch_gemv_multi(const GemmArgs* items, int count, const DeviceInfo& dev, int* parts_used,
                             hipStream_t stream);
// `bits`: 4 (a.q = packed nibbles), 6 (a.q = q6, 24 bytes per block) or 8 (a.q = q8, 32 bytes per
// block); 22 and 24: the same widths with E3M2 and E5M2 elements; 2: the 2-bit ternary codes (8 bytes per
// block); the fused form exists for 4 only.
hipError_t launch_gemv_reg(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream,
                           const Epilogue* epi = nullptr, int bits = 4);

// The 6-bit draft format (E2M3 codes as a 192-bit string per block: a.q is q6 [N, K/32 * 24]); e2m3.hip.
hipError_t launch_e2m3_cast(const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q6, void* s,
                            bool integer_rule, hipStream_t stream);
hipError_t launch_e2m3_dequant(const void* q6, const void* s, int64_t n_rows, int64_t k, void* w, int64_t ldw,
                               hipStream_t stream);

// 16-row MFMA tiles (bf16 16x16x32) for verification batches; passes of up to 16 activation rows.
// When the activation rows of a pass do not fit the LDS whole, K is split: in space over
// workgroups through a workspace of mfma_splitk_bytes() with a second kernel that adds the partial
// products in a fixed order; without a workspace in time inside the kernel when a workgroup's
// tiles are few enough to keep their running sums in LDS; else in narrower passes.
// mfma_can_run: K % 128 == 0 and four activation rows can run in one of these ways.
bool mfma_can_run(const GemmArgs& a, const DeviceInfo& dev, bool have_splitk_ws);
size_t mfma_splitk_bytes(int m, int n, int k, const DeviceInfo& dev);
// `tiled`: a.q / a.s are the tile-major copy and the call is one that mfma_tiled_split_can_run
// accepts (K split in space through the workspace; the whole-K tile-major passes go to
// launch_mfma_tile directly).
hipError_t launch_mfma(const GemmArgs& a, const DeviceInfo& dev, float* splitk_ws, int* parts_used,
                       hipStream_t stream, bool general_only = false, const Epilogue* epi = nullptr,
                       bool tiled = false);
bool mfma_tiled_split_can_run(const GemmArgs& a, const DeviceInfo& dev);

// The same tiles in a leaner kernel for passes whose activation rows fit the LDS whole (no K
// split); launch_mfma uses it whenever it can run unless told `general_only` (or
// MXFP4_MFMA_LEGACY=1 in the environment, for measurements).
bool mfma_tile_can_run(const GemmArgs& a, const DeviceInfo& dev);
hipError_t launch_mfma_tile(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream,
                            bool tiled = false, const Epilogue* epi = nullptr);

// The 8-bit (a.q = q8 [N, K]) and 6-bit (a.q = q6) draft formats on the same tiles; shapes as
// mfma_tile_can_run; `bits` 8 or 6.
bool mfma_tile_fmt_can_run(const GemmArgs& a, const DeviceInfo& dev);   // the same with passes of four rows at least
hipError_t launch_mfma_tile8(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream,
                             int bits = 8);

// The tile kernel with K split in space for passes whose activation rows do not fit the LDS:
// FP32 partial products to ws = float [phases][M][N] (mfma.hip's finish kernel adds them).
bool mfma_tile_split_fits(int phase_steps, int mp, const DeviceInfo& dev);
hipError_t launch_mfma_tile_split(const GemmArgs& a, int m0, int mp, int phases, int phase_steps, float* ws,
                                  const DeviceInfo& dev, hipStream_t stream, bool tiled = false);

// The tile kernel with K in phases inside the workgroup, for passes whose activation rows do not
// fit the LDS: no workspace, no second launch; plain product (no pick, no fused epilogue), passes
// of four or eight rows.  Faster than the split in space where a workgroup has few tiles.
bool mfma_tile_phased_can_run(const GemmArgs& a, const DeviceInfo& dev);
hipError_t launch_mfma_tile_phased(const GemmArgs& a, const DeviceInfo& dev, hipStream_t stream, bool tiled);
// Whether a call whose rows do not fit the LDS should take it: `split_available` says that the
// split in space could run too (the caller gave a workspace).
bool mfma_tile_phased_preferred(const GemmArgs& a, const DeviceInfo& dev, bool split_available);

// Tile-major copy of the weights for the tile kernel (`tiled`: a.q / a.s are that copy): what a
// wave instruction loads is contiguous.  Sizes in bytes; K % 128 == 0.
size_t tile_repack_q_bytes(int64_t n, int64_t k);
size_t tile_repack_s_bytes(int64_t n, int64_t k);
hipError_t launch_tile_repack(const void* q, const void* s, int n, int k, void* qt, void* st, hipStream_t stream);

// The unquantised product with BF16 weights [N, K] (row stride ldw), same conventions otherwise.
struct Bf16Args {
    const uint16_t* x;
    int64_t ldx;
    const uint16_t* w;
    int64_t ldw;
    int m, n, k;
    uint16_t* y;
    int64_t ldy;
    float* part_val;
    int32_t* part_idx;
    int parts;
};
bool bf16_can_run(const Bf16Args& a, const DeviceInfo& dev);
hipError_t launch_bf16_gemv(const Bf16Args& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream);

// The decode step (one or two activation rows) on the tile-major tensors (a.q = q_tiled, a.s =
// s_tiled); gemv_tile.hip.  The argmax form writes one partial winner per workgroup.
bool gemv_tile_can_run(const GemmArgs& a, const DeviceInfo& dev);
hipError_t launch_gemv_tile(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream);

// y[M, K] = x[M, N] * dequant(W)[N, K]: the product along the rows of the stored tensor (gemm_t.hip).
// `part` holds gemm_t_workspace_bytes of FP32 partial sums.
bool gemm_t_can_run(int k);
size_t gemm_t_workspace_bytes(int m, int n, int k, const DeviceInfo& dev);
hipError_t launch_gemm_t(const GemmArgs& a, const DeviceInfo& dev, float* part, hipStream_t stream);

// Further block formats by id (1 E5M2, 2 E3M2, 3 the 2-bit ternary T2; a.q holds 32, 24 or 8 bytes
// per block); mxfmt.hip.  mxfmt_block_bytes is 0 for an unknown id.
int mxfmt_block_bytes(int fmt);
hipError_t launch_mxfmt_cast(int fmt, const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q, void* s,
                             bool integer_rule, hipStream_t stream);
hipError_t launch_mxfmt_dequant(int fmt, const void* q, const void* s, int64_t n_rows, int64_t k, void* w,
                                int64_t ldw, hipStream_t stream);
bool mxfmt_can_run(const GemmArgs& a, const DeviceInfo& dev);
hipError_t launch_mxfmt_gemv(int fmt, const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream);

// The 8-bit draft format (E4M3 elements, one byte each: a.q is q8 [N, K]; a.s as before); e4m3.hip.
hipError_t launch_e4m3_cast(const void* w, int64_t n_rows, int64_t k, int64_t ldw, void* q8, void* s,
                            bool integer_rule, hipStream_t stream);
hipError_t launch_e4m3_dequant(const void* q8, const void* s, int64_t n_rows, int64_t k, void* w, int64_t ldw,
                               hipStream_t stream);
bool e4m3_can_run(const GemmArgs& a, const DeviceInfo& dev);
hipError_t launch_e4m3_gemv(const GemmArgs& a, const DeviceInfo& dev, int* parts_used, hipStream_t stream);

// Second stage of the fused argmax: reduce `parts_used` partial winners per row.
hipError_t launch_argmax_finish(const float* part_val, const int32_t* part_idx, int parts, int parts_used,
                                int m, int32_t* argmax_out, float* max_out, hipStream_t stream);

// The same second stage with the greedy draft verification fused behind it, one workgroup:
// draft[m - 1] tokens are compared with the picks; accept_out[0] = accepted draft tokens,
// accept_out[1] = the pick that follows them.  m <= kVerifyMaxRows.
constexpr int kVerifyMaxRows = 1024;
hipError_t launch_verify_finish(const float* part_val, const int32_t* part_idx, int parts, int parts_used,
                                int m, const int32_t* draft, int32_t* argmax_out, float* max_out,
                                int32_t* accept_out, hipStream_t stream);

// A chain of dependent one-token products in one persistent launch (chain.hip): link i reads what
// the links before it wrote; a grid-wide barrier sits between neighbours and the weights of the
// next link are already streaming while it is crossed.  y == nullptr: the fused pick (last item
// only; argmax_out / max_out).  The workspace holds the barrier's flags (zeroed once by
// launch_chain_ws_init, then only ever advanced by the launches).  `wait_ticks`: bound of one wait
// in 10 ns ticks; `phantom`: workgroups the barrier waits for that do not exist (tests of the
// give-up path only).
constexpr int kChainMaxLinks = 48;       // per launch; longer chains take several launches
constexpr int kChainMaxChunk = 1024;     // weight rows of one link per workgroup
struct ChainItem {
    const uint16_t* x;
    const uint8_t* q;
    const uint8_t* s;
    uint16_t* y;
    const uint16_t* bias;
    const uint16_t* residual;
    int n, k, act;
    int32_t* argmax_out;
    float* max_out;
};
size_t chain_workspace_bytes();
size_t chain_pick_area_offset();       // where the scratch of a pick run as ordinary launches starts
hipError_t launch_chain_ws_init(void* ws, hipStream_t stream);
bool chain_can_run(const ChainItem* items, int count, const DeviceInfo& dev);
hipError_t launch_chain(const ChainItem* items, int count, const DeviceInfo& dev, void* ws, int wait_ticks,
                        int phantom, hipStream_t stream);

// Plain streaming kernels used to measure what the memory system delivers.
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, const DeviceInfo& dev,
                              hipStream_t stream);
hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, const DeviceInfo& dev,
                              hipStream_t stream);

}  // namespace mxfp4
