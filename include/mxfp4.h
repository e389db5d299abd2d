/*
 * mxfp4.h -- C ABI of the MI355X (gfx950) MXFP4 weight-only-quantised linear layer.
 *
 * The operations are those of arXiv 2503.13565 (ML-SpecQD), section 3.4.3: weights are
 * direct-cast once, offline, from BF16 to MXFP4 (an FP4 E2M1 tensor plus one 8-bit E8M0
 * scale per 32 elements), and every draft decode step and every verification pass then
 * multiplies a few BF16 activation rows (1 token when drafting, k+1 when verifying k draft
 * tokens; section 4.4) with the dequantised weights, accumulating in FP32.
 *
 * Conventions shared by all entry points
 *   - Every data pointer is a DEVICE pointer (HBM) unless marked "host".  The caller owns all
 *     buffers and keeps them alive until `stream` has passed the call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work on it and return; they never synchronise, allocate or free device memory.
 *   - BF16 tensors are row-major with an explicit leading dimension in elements.
 *   - Packed weights `q`: uint8 [N, K/2] row-major, byte j of a row holds element 2j in bits
 *     0..3 and element 2j+1 in bits 4..7; a nibble is sign<<3 | eem (magnitudes 0, .5, 1,
 *     1.5, 2, 3, 4, 6).  Scales `s`: uint8 [N, K/32] row-major, value 2^(byte-127), 0xFF marks
 *     a NaN block.  Blocks of 32 run along K, the reduction axis (Eq. 2).
 *   - Return value: MXFP4_OK or an error code; on error nothing was enqueued and
 *     mxfp4_last_error() (host, thread-local) describes it.  No call aborts the process.
 *   - Results are deterministic: the same inputs and shapes give bit-identical outputs.
 *
 * Which calls are what
 *   The contract (the paper's problem statement: cast once, then products per step):
 *     mxfp4_direct_cast, mxfp4_woq_gemm, mxfp4_woq_gemm_argmax (+ _workspace_bytes), mxfp4_last_error.
 *   The same product with more said about it -- one family, pick by what the caller has:
 *     mxfp4_woq_gemm_ws (a workspace), mxfp4_woq_gemm_fused (bias, gate, residual),
 *     mxfp4_woq_gemm_verify (draft acceptance behind the pick), mxfp4_woq_gemm_grouped (a step's
 *     products in one call), mxfp4_woq_gemm_chain (a step's dependent products in one launch),
 *     mxfp4_woq_gemm_argmax_noalloc (no workspace), mxfp4_woq_gemm_tiled* with mxfp4_tile_repack (the
 *     same calls on the tile-major copy of the weights).
 *   Next to the method: mxfp4_bf16_gemm* (the unquantised target's linear), mxfp4_e4m3_*,
 *     mxfp4_e2m3_* and mxfp4_fmt_* (8-, 6- and 2-bit element formats as drafts), mxfp4_woq_gemm_t
 *     (the value side of attention over a cache held in the same format).
 *   Diagnostics, for tests and measurements only: mxfp4_*_path (a kernel family forced),
 *     mxfp4_direct_cast_bits / mxfp4_*_direct_cast_bits (the integer rounding rule in place of the
 *     convert instruction), mxfp4_dequant*, mxfp4_diag_stream_*.
 *   The library reads one environment variable, MXFP4_FORCE_PATH (a MXFP4_PATH_* number in place of
 *   AUTO for every product call; tests only).  The launch-shape switches used while measuring exist
 *   only in builds with -DMXFP4_MEASUREMENT_KNOBS.
 */
#ifndef MXFP4_H
#define MXFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MXFP4_OK = 0,
    MXFP4_ERR_NULL = 1,      /* a required pointer is NULL */
    MXFP4_ERR_SHAPE = 2,     /* K % 32 != 0, a size < 1 (0 rows is allowed and a no-op), ld < K, K too large */
    MXFP4_ERR_ALIGN = 3,     /* a buffer or leading dimension breaks the 16-byte alignment rule */
    MXFP4_ERR_WORKSPACE = 4, /* workspace missing or smaller than *_workspace_bytes() */
    MXFP4_ERR_HIP = 5,       /* the HIP runtime refused a launch */
    MXFP4_ERR_ARG = 6        /* unknown path / option value */
};

/* Kernel families the dispatcher can be forced to (tests and measurements); AUTO picks by M:
 * one or two rows take VALU_REG when the shape allows it, else VALU_CVT; three or more take MFMA. */
enum {
    MXFP4_PATH_AUTO = 0,
    MXFP4_PATH_VALU_BITS = 1, /* wave-per-row GEMV, nibbles decoded with plain integer/FP32 ops  */
    MXFP4_PATH_VALU_CVT = 2,  /* wave-per-row GEMV, gfx950 FP4->BF16 scaled converts + dot2      */
    MXFP4_PATH_VALU_LUT = 3,  /* wave-per-row GEMV, LDS-resident byte -> 2xBF16 lookup table      */
    MXFP4_PATH_MFMA = 4,      /* 16-row MFMA tiles (bf16 16x16x32), for verification batches     */
    MXFP4_PATH_MFMA_GENERAL = 6, /* the general MFMA kernel (K split in time or space) also where the
                                 leaner tile kernel, which MXFP4_PATH_MFMA prefers, could run      */
    MXFP4_PATH_VALU_REG = 5   /* decode-step GEMV: converts + dot2 with the activations in registers,
                                 one or two workgroups per compute unit; K % 128 == 0, K <= 12288 (one row)
                                 or 4096 (two rows at a time), N >= 8 * compute units              */
};

/*
 * Direct cast BF16 -> MXFP4 (section 3.4.3, the two quantisation steps).
 * For every 32-element block along K: scale byte = max(biased_exponent(amax) - 2, 0), i.e.
 * X = 2^(floor(log2 amax) - 2); each element v/X is rounded to the nearest E2M1 value, ties to
 * the even code, saturating at +-6, sign bit preserved (also for zeros).  A block holding NaN
 * or Inf gets scale 0xFF and zero nibbles.  Maximum and scale are integer arithmetic on the BF16
 * bit patterns; the elements are rounded by the gfx950 scaled BF16->FP4 convert.
 *   w_bf16      in  BF16 [N, K], row stride ldw elements (ldw >= K, ldw % 8 == 0, 16-byte aligned)
 *   q_packed    out uint8 [N, K/2]   (4-byte aligned)
 *   scales_e8m0 out uint8 [N, K/32]
 * N may be 0 (no-op).  K must be a positive multiple of 32.
 */
int mxfp4_direct_cast(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                      void* q_packed, void* scales_e8m0, void* stream);

/* The same cast with the elements rounded by the integer-only rule on the bit patterns rather
 * than by the gfx950 scaled BF16->FP4 convert instruction; both give the same bits (kept so that
 * each can be checked against the other and against the CPU definition). */
int mxfp4_direct_cast_bits(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                           void* q_packed, void* scales_e8m0, void* stream);

/*
 * An 8-bit draft on the same path (sections 1, 3.2 and 5 name 8-bit quantisation as a drop-in for
 * the 4-bit draft): the two-step direct cast of section 3.4.3 with the OCP 8-bit element format
 * E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, largest magnitude 448, no
 * infinities, S.1111.111 = NaN) in place of E2M1: X = 2^(floor(log2 amax) - 8), elements rounded
 * to nearest (ties to the even code), magnitudes beyond 448 saturate; zero blocks, tiny scales,
 * non-finite inputs and the sign of zero as in mxfp4_direct_cast.
 *   q8           [N, K] one byte per element (sign << 7 | eeeemmm); 8-byte aligned for the cast,
 *                16-byte aligned for the product and the dequantisation
 *   scales_e8m0  [N, K/32] as for MXFP4
 * mxfp4_e4m3_direct_cast_bits rounds with an integer-only rule instead of the convert instruction
 * (same bits).  mxfp4_e4m3_dequant writes scale * element as BF16 (exact while that is a normal
 * BF16 number).  mxfp4_e4m3_woq_gemm and mxfp4_e4m3_woq_gemm_argmax are mxfp4_woq_gemm and
 * mxfp4_woq_gemm_argmax with q8 in place of q_packed (same arguments, same error codes, same
 * tie rule); N * K stays below 2 GiB; the argmax workspace is M * 8 bytes per workgroup the
 * device can hold, which mxfp4_woq_gemm_argmax_workspace_bytes(M, N, K) covers.
 */
int mxfp4_e4m3_direct_cast(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                           void* q8, void* scales_e8m0, void* stream);
int mxfp4_e4m3_direct_cast_bits(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                                void* q8, void* scales_e8m0, void* stream);
int mxfp4_e4m3_dequant(const void* q8, const void* scales_e8m0, int64_t N, int64_t K,
                       void* w_bf16, int64_t ldw, void* stream);
int mxfp4_e4m3_woq_gemm(const void* x_bf16, int64_t M, int64_t ldx,
                        const void* q8, const void* scales_e8m0, int64_t N, int64_t K,
                        void* y_bf16, int64_t ldy, void* stream);
int mxfp4_e4m3_woq_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx,
                               const void* q8, const void* scales_e8m0, int64_t N, int64_t K,
                               int32_t* argmax_out, float* max_out,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * A 6-bit draft on the same path: the same cast with the OCP 6-bit element format E2M3 (1 sign, 2
 * exponent bits with bias 1, 3 mantissa bits; magnitudes m/8 and (1 + m/8) * 2^(e-1), largest
 * 7.5; no infinities, no NaN): X = 2^(floor(log2 amax) - 2) as for MXFP4, elements rounded to
 * nearest (ties to the even code), beyond 7.5 saturates; zero blocks, tiny scales, non-finite
 * inputs and the sign of zero as in mxfp4_direct_cast.  6.25 bits per weight.
 *   q6           [N, K/32 * 24] bytes: the 32 codes (sign << 5 | eemmm) of a block are a
 *                little-endian bit string of 192 bits, code i in bits 6i .. 6i+5; 8-byte aligned
 *   scales_e8m0  [N, K/32] as for MXFP4 (4-byte aligned for the product)
 * mxfp4_e2m3_direct_cast_bits rounds and packs with integer arithmetic instead of the convert
 * instruction (same bits).  mxfp4_e2m3_woq_gemm and mxfp4_e2m3_woq_gemm_argmax are mxfp4_woq_gemm
 * and mxfp4_woq_gemm_argmax with q6 in place of q_packed, for K % 128 == 0 and any M, when four
 * activation rows of K elements fit the LDS (K up to about 19000; any N: the matrix-core tiles,
 * up to 16 rows per pass) or K <= 32768 and N >= 8 x compute units (the decode kernel, one or two
 * rows per pass); MXFP4_ERR_SHAPE otherwise.  Argmax workspace as for mxfp4_e4m3_woq_gemm_argmax.
 */
int mxfp4_e2m3_direct_cast(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                           void* q6, void* scales_e8m0, void* stream);
int mxfp4_e2m3_direct_cast_bits(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                                void* q6, void* scales_e8m0, void* stream);
int mxfp4_e2m3_dequant(const void* q6, const void* scales_e8m0, int64_t N, int64_t K,
                       void* w_bf16, int64_t ldw, void* stream);
int mxfp4_e2m3_woq_gemm(const void* x_bf16, int64_t M, int64_t ldx,
                        const void* q6, const void* scales_e8m0, int64_t N, int64_t K,
                        void* y_bf16, int64_t ldy, void* stream);
int mxfp4_e2m3_woq_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx,
                               const void* q6, const void* scales_e8m0, int64_t N, int64_t K,
                               int32_t* argmax_out, float* max_out,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Further block formats on the same path, chosen by id (sections 1, 3.2 and 5: 8-bit and lower-bit
 * drafts, down to ternary, as drop-ins for the 4-bit draft; the cast is the two-step rule of
 * section 3.4.3 with the element format named, the product is Eq. 2 with FP32 accumulation):
 *   MXFP4_FMT_E5M2  OCP 8-bit E5M2: 1 sign, 5 exponent bits (bias 15), 2 mantissa bits; largest
 *                   finite magnitude 57344; X = 2^(floor(log2 amax) - 15).  The cast never writes the
 *                   Inf and NaN codes (S.11111.xx); beyond 57344 saturates.  32 bytes per block.
 *   MXFP4_FMT_E3M2  OCP 6-bit E3M2: 1 sign, 3 exponent bits (bias 3), 2 mantissa bits; largest 28, no
 *                   Inf, no NaN; X = 2^(floor(log2 amax) - 4).  24 bytes per block.
 *   MXFP4_FMT_T2    2 bits, sign << 1 | magnitude: values {0, +1, -1} (and -0), a ternary draft;
 *                   X = 2^floor(log2 amax), so |v| / X < 2: up to 1/2 rounds to 0 (the tie goes to the
 *                   even code 0), above it to 1.  8 bytes per block, 2.25 bits per weight.
 * Elements are rounded to nearest, ties to the even code; zero blocks, the clamp of X at 2^-127,
 * non-finite inputs (scale byte 0xFF, zero codes) and the sign of zero as in mxfp4_direct_cast.
 *   q            [N, K/32 * B] bytes, B = mxfp4_fmt_block_bytes(fmt): the 32 codes of a block (sign
 *                in the top bit of a code) are a little-endian bit string, code i in bits b i ..
 *                b i + b - 1 with b the element width; 8-byte aligned; N * K/32 * B below 2 GiB - 256
 *   scales_e8m0  [N, K/32] as for MXFP4
 * mxfp4_fmt_block_bytes is 0 for an unknown id; every other call then returns MXFP4_ERR_SHAPE.
 * mxfp4_fmt_direct_cast_bits rounds by an ALU rule on the bit patterns instead of the convert
 * instructions (same bits; T2 has only that rule).  mxfp4_fmt_dequant writes scale * element as BF16
 * (E5M2, E3M2: exact while that is a normal BF16 number; T2: always exact).  mxfp4_fmt_woq_gemm and
 * mxfp4_fmt_woq_gemm_argmax are mxfp4_woq_gemm and mxfp4_woq_gemm_argmax with q in place of
 * q_packed (same arguments, same error codes, same tie rule) for any M, any N and every K up to
 * MXFP4_MAX_K whose BF16 row fits the LDS (on gfx950 all of them); rows of K <= 1024 with K/32 a power of two (the
 * rows of a quantised attention cache, section 5) are processed 64 / (K/32) at a time per wave.
 * Argmax workspace as for mxfp4_e4m3_woq_gemm_argmax.
 */
enum { MXFP4_FMT_E5M2 = 1, MXFP4_FMT_E3M2 = 2, MXFP4_FMT_T2 = 3 };
int mxfp4_fmt_block_bytes(int fmt);
int mxfp4_fmt_direct_cast(int fmt, const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                          void* q, void* scales_e8m0, void* stream);
int mxfp4_fmt_direct_cast_bits(int fmt, const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                               void* q, void* scales_e8m0, void* stream);
int mxfp4_fmt_dequant(int fmt, const void* q, const void* scales_e8m0, int64_t N, int64_t K,
                      void* w_bf16, int64_t ldw, void* stream);
int mxfp4_fmt_woq_gemm(int fmt, const void* x_bf16, int64_t M, int64_t ldx,
                       const void* q, const void* scales_e8m0, int64_t N, int64_t K,
                       void* y_bf16, int64_t ldy, void* stream);
int mxfp4_fmt_woq_gemm_argmax(int fmt, const void* x_bf16, int64_t M, int64_t ldx,
                              const void* q, const void* scales_e8m0, int64_t N, int64_t K,
                              int32_t* argmax_out, float* max_out,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * The product along the rows of a stored MXFP4 tensor (section 5 names a quantised attention cache
 * as the next step of the method and gives no procedure; the reading taken here: one token per row
 * of q_packed / scales_e8m0, the 32-element blocks of section 3.4.3 along the head dimension K, so
 * that a new token is cast on its own by mxfp4_direct_cast(N = 1) into row T of the cache; the score
 * side  scores[M, T] = query[M, K] * dequant(K-cache)^T  is mxfp4_woq_gemm with N = T; the value side
 * contracts over the rows and is this call):
 *   y[m, k] = sum_n x[m, n] * dequant(W)[n, k],   FP32 accumulation, BF16 result
 *   x_bf16     [M, N] (the attention weights of M query rows that share the cache), row stride ldx
 *              >= N, 2-byte aligned; 1 <= M <= 64
 *   q_packed, scales_e8m0   the stored tensor [N, K/2], [N, K/32] as for mxfp4_woq_gemm; K a multiple
 *              of 32, at most 2048 (a head dimension), else MXFP4_ERR_SHAPE
 *   y_bf16     [M, K], row stride ldy >= K
 *   workspace  mxfp4_woq_gemm_t_workspace_bytes(M, N, K) bytes of device memory (FP32 partial sums
 *              of the workgroups, added in index order: the result is the same on every call),
 *              4-byte aligned; the size query returns 0 for shapes the call refuses
 * A scale byte 0xFF makes the 32 outputs of its block NaN for every row m, also where x[m, n] = 0.
 */
size_t mxfp4_woq_gemm_t_workspace_bytes(int64_t M, int64_t N, int64_t K);
int mxfp4_woq_gemm_t(const void* x_bf16, int64_t M, int64_t ldx,
                     const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                     void* y_bf16, int64_t ldy,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Dequantise to BF16 (exact whenever 2^(scale-127) * 6 is a normal BF16 number): the inverse
 * map of the format in section 3.4.3; used to check the weight decode in isolation.
 *   w_bf16 out BF16 [N, K], row stride ldw elements.
 */
int mxfp4_dequant(const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                  void* w_bf16, int64_t ldw, void* stream);

/*
 * Skinny weight-only-quantised product y = x * dequant(W)^T (section 3.4.3, Eq. 2; the
 * paper's GEMM with 1..8 tokens, section 4.4):
 *   y[m, n] = bf16_rne( sum_k x[m, k] * w_hat[n, k] ),  FP32 accumulation, scale applied per
 *   32-block (late or early scaling are the same number because the scale is a power of two).
 *   x_bf16 in  BF16 [M, K], row stride ldx (ldx >= K, ldx % 8 == 0, base 16-byte aligned)
 *   q_packed, scales_e8m0  in, as written by mxfp4_direct_cast (q 16-byte, scales 4-byte aligned)
 *   y_bf16 out BF16 [M, N], row stride ldy (ldy >= N)
 * M >= 1 (any size; M <= 32 is the designed range), N >= 1, K a positive multiple of 32 and at
 * most MXFP4_MAX_K; the packed weights of one call stay below 2 GiB.  The summation order is fixed per (M, N, K, path), not specified.
 */
#define MXFP4_MAX_K 65536
int mxfp4_woq_gemm(const void* x_bf16, int64_t M, int64_t ldx,
                   const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                   void* y_bf16, int64_t ldy, void* stream);

/* Same, with the kernel family forced (MXFP4_PATH_*); MXFP4_ERR_ARG if the path cannot run
 * the shape. */
int mxfp4_woq_gemm_path(const void* x_bf16, int64_t M, int64_t ldx,
                        const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                        void* y_bf16, int64_t ldy, int path, void* stream);

/*
 * The same product with a caller-provided scratch buffer.  When the activation rows of a pass do
 * not fit the LDS of a compute unit whole (M * K large), the MFMA path cuts K into phases.  With
 * `workspace` the phases run side by side on different compute units and a second kernel adds
 * their FP32 partial products, which live in the workspace, in a fixed order: the fast form.
 * Without it (NULL, or smaller than mxfp4_woq_gemm_workspace_bytes, which is 0 when no split is
 * needed) the call still works: the phases then run one after the other inside the kernel (up to
 * eight rows: about as fast as the split for matrices with one tile of 16 output rows per compute
 * unit, such as a down projection), or, for wider passes over matrices with very many output rows
 * per compute unit, in narrower passes over the weights.
 * workspace: 8-byte aligned, contents unspecified before and after; calls that overlap in time
 * must not share it.  `path` as in mxfp4_woq_gemm_path.
 */
size_t mxfp4_woq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
int mxfp4_woq_gemm_ws(const void* x_bf16, int64_t M, int64_t ldx,
                      const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                      void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                      int path, void* stream);

/*
 * The same product with the operators that surround a linear layer fused behind it (section
 * 3.4: the backend applies bias and residual add to the contraction's output while it is at
 * hand; the gate of the gated MLP of the targets of sections 4.2 and 4.3 is handled the same
 * way).  All of it in FP32 on the accumulators, one rounding to BF16 at the end:
 *   z[m][n] = sum_k x[m][k] * w[n][k] + bias[n]
 *   MXFP4_ACT_NONE:    t[m][c] = z[m][c]                          C = N columns
 *   MXFP4_ACT_SWIGLU:  t[m][c] = silu(z[m][2c]) * z[m][2c + 1]    C = N / 2 columns, N even;
 *                      silu(v) = v / (1 + e^-v); the weight rows are interleaved: row 2c is row
 *                      c of the gate projection, row 2c + 1 row c of the up projection
 *   y[m][c] = bf16(t[m][c] + residual[m][c])
 *   bias_bf16      in  BF16 [N], 2-byte aligned, or NULL (no bias)
 *   residual_bf16  in  BF16 [M, C], row stride ldr >= C, or NULL (none; ldr then ignored).  It
 *                  may be y itself with ldr == ldy (the residual stream updated in place); any
 *                  other overlap with y is not allowed
 *   y_bf16         out BF16 [M, C], row stride ldy >= C
 * x, q, s, workspace and `path` as in mxfp4_woq_gemm_ws (the workspace is optional in the same
 * way; mxfp4_woq_gemm_workspace_bytes(M, N, K) gives its size).  MXFP4_ERR_ARG for an unknown
 * act, MXFP4_ERR_SHAPE for an odd N with the gate.
 */
enum { MXFP4_ACT_NONE = 0, MXFP4_ACT_SWIGLU = 1 };
int mxfp4_woq_gemm_fused(const void* x_bf16, int64_t M, int64_t ldx,
                         const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                         const void* bias_bf16, int act, const void* residual_bf16, int64_t ldr,
                         void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                         int path, void* stream);

/*
 * A sequence of products in one call: the linear layers of a decode or verification step run
 * back to back (sections 3.1 and 3.4: one forward pass is a fixed chain of contractions), and a
 * host that issues them one call at a time spends longer per call than most of these kernels
 * run.  Equivalent to calling, for i = 0 .. count - 1 in this order on `stream`,
 * mxfp4_woq_gemm_ws (descriptor without bias, residual, act and argmax_out),
 * mxfp4_woq_gemm_argmax (argmax_out given: the LM head at the end of the step; y, bias, residual
 * must then be NULL and act MXFP4_ACT_NONE) or mxfp4_woq_gemm_fused (otherwise) with path
 * MXFP4_PATH_AUTO and the one workspace: same kernels, same bits.  A descriptor may read what an
 * earlier one wrote (the stream orders them).
 *   descs      HOST array of `count` descriptors, read during the call only; the fields have
 *              the meaning, layout and alignment rules of the arguments of the same name of
 *              mxfp4_woq_gemm_fused and mxfp4_woq_gemm_argmax; `flags` is 0 or MXFP4_DESC_TILED:
 *              q_packed and scales_e8m0 are then the tile-major pair of mxfp4_tile_repack and the
 *              product is the mxfp4_woq_gemm_tiled_* call of the same kind;
 *              MXFP4_DESC_INDEPENDENT (ignored together with MXFP4_DESC_TILED): the caller states that
 *              this product reads no output of the descriptors next to it that carry the flag too
 *              and that none of them reads or overwrites its outputs; consecutive such
 *              descriptors may then run in one launch, in any order or at once (taken for up to 8
 *              products with M = 1, no bias, act or residual, at most one with argmax_out, each a
 *              shape of the decode kernel -- K % 128 == 0, K <= 32768, N >= 8 x compute units --
 *              whose activation rows fit the LDS together; same bits as the single calls;
 *              otherwise the flag changes nothing).  Other bits: error
 *   workspace  device scratch shared by all products: optional as in mxfp4_woq_gemm_ws when no
 *              descriptor asks for the argmax, required as in mxfp4_woq_gemm_argmax otherwise;
 *              mxfp4_woq_gemm_grouped_workspace_bytes gives the size that serves every
 *              descriptor (the largest single need; 0 for a NULL or invalid array)
 * Every descriptor is checked before anything is launched: on an argument error nothing has
 * run, the code is that of the single call and mxfp4_last_error() names the descriptor's
 * index.  count == 0 is a no-op.
 */
typedef struct mxfp4_gemm_desc {
    const void* x_bf16;
    int64_t M;
    int64_t ldx;
    const void* q_packed;
    const void* scales_e8m0;
    int64_t N;
    int64_t K;
    const void* bias_bf16;
    const void* residual_bf16;
    int64_t ldr;
    void* y_bf16;
    int64_t ldy;
    int32_t* argmax_out;
    float* max_out;
    int32_t act;
    int32_t flags;
} mxfp4_gemm_desc;
enum { MXFP4_DESC_TILED = 1, MXFP4_DESC_INDEPENDENT = 2 };
size_t mxfp4_woq_gemm_grouped_workspace_bytes(const mxfp4_gemm_desc* descs, int64_t count);
int mxfp4_woq_gemm_grouped(const mxfp4_gemm_desc* descs, int64_t count,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * A chain of dependent one-token products, run the fastest way the device allows (section 3.2: a
 * decode step is bound by streaming the model's weights in; sections 3.1 and 3.4: one forward pass
 * is a fixed chain of contractions, each reading what the one before it wrote).  Same results as
 * mxfp4_woq_gemm_grouped on the same descriptors, bit for bit.  Every product is ordered after ALL
 * products before it in the array, so a descriptor may read (x, residual) any earlier output, also
 * in place.
 *
 * The persistent launch.  One workgroup per compute unit stays resident for a run of products; a
 * grid-wide barrier separates neighbours; the weights of the next product are already streaming
 * while the barrier is crossed and the new activation row is fetched; a pick at the end of the
 * chain is finished inside the same launch.  Measured on this device a barrier costs more than a
 * launch (the barrier's own memory operations queue behind the weight loads of their compute
 * unit), so opts.mode decides how much of the chain uses it:
 *   MXFP4_CHAIN_AUTO        (default) the fastest form measured for the shapes at hand; on this device
 *                           that is MXFP4_CHAIN_SEPARATE for every chain tried (7B and 70B shapes)
 *   MXFP4_CHAIN_PERSISTENT  the whole chain in persistent launches (up to 48 products each)
 *   MXFP4_CHAIN_SEPARATE    every product a launch of its own (what mxfp4_woq_gemm_grouped does)
 *
 *   descs     HOST array, read during the call only.  Every descriptor: M == 1, flags == 0,
 *             K % 128 == 0, at most 1024 weight rows per compute unit (N <= 1024 x compute units);
 *             bias, act, residual as in mxfp4_woq_gemm_fused; argmax_out (with optional max_out)
 *             only on the last descriptor.  count <= MXFP4_CHAIN_MAX_LINKS.  Shapes outside this:
 *             MXFP4_ERR_ARG, nothing launched (use mxfp4_woq_gemm_grouped).
 *   chain_ws  device memory of mxfp4_woq_gemm_chain_workspace_bytes() bytes, 256-byte aligned,
 *             prepared ONCE by mxfp4_woq_gemm_chain_init and from then on owned by the chained
 *             calls: it carries the barrier's epoch counters from one call to the next (nothing is
 *             reset between calls, so a call can be captured in a HIP graph and replayed).  One
 *             workspace serves one device and one call at a time: calls that overlap in time on
 *             one workspace corrupt each other's barriers.
 *   opts      NULL, or: wait_us = bound of a single barrier wait in microseconds (0: the default
 *             of 2 s; at most 20 s); phantom_workgroups = number of workgroups the barrier waits
 *             for that do not exist (0 in production; > 0 makes every wait expire and is how the
 *             give-up path is exercised from the host; it implies the persistent kernel for the
 *             whole chain); mode as above.
 * The persistent launch needs all its workgroups resident together (one per compute unit).  Other
 * work on the device only delays it; a wait that outlasts wait_us is given up: every wave then
 * ends normally, the outputs of the call are unspecified, and the 32-bit word at byte offset
 * MXFP4_CHAIN_STATUS_OFFSET of chain_ws becomes non-zero (0x100 + index, within its launch, of the
 * product whose barrier expired).  The status is sticky: later persistent launches on that
 * workspace see it and do nothing, until mxfp4_woq_gemm_chain_init prepares the workspace again.
 * The call itself never synchronises; the caller reads the status word after synchronising the
 * stream.
 */
#define MXFP4_CHAIN_MAX_LINKS 4096
#define MXFP4_CHAIN_STATUS_OFFSET 4224
enum { MXFP4_CHAIN_AUTO = 0, MXFP4_CHAIN_PERSISTENT = 1, MXFP4_CHAIN_SEPARATE = 2 };
typedef struct mxfp4_chain_opts {
    int64_t wait_us;
    int32_t phantom_workgroups;
    int32_t mode;
} mxfp4_chain_opts;
size_t mxfp4_woq_gemm_chain_workspace_bytes(void);
int mxfp4_woq_gemm_chain_init(void* chain_ws, size_t chain_ws_bytes, void* stream);
int mxfp4_woq_gemm_chain(const mxfp4_gemm_desc* descs, int64_t count,
                         void* chain_ws, size_t chain_ws_bytes,
                         const mxfp4_chain_opts* opts, void* stream);

/*
 * The same product with the greedy pick fused (section 3.1: the target's token at each
 * verified position is compared with the draft's; section 4.1: greedy search): for every
 * activation row m, the index n of the largest FP32 accumulator (before any BF16 rounding),
 * the lowest index among equal maxima.  No y is written.
 *   argmax_out out int32 [M]
 *   max_out    out float [M], the winning accumulator; may be NULL
 *   workspace  scratch of at least mxfp4_woq_gemm_argmax_workspace_bytes(M, N, K) bytes,
 *              8-byte aligned; contents before and after the call are unspecified.  Two calls
 *              that overlap in time must not share it.
 * Rows whose accumulators contain NaN give an unspecified index.
 */
size_t mxfp4_woq_gemm_argmax_workspace_bytes(int64_t M, int64_t N, int64_t K);
int mxfp4_woq_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx,
                          const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                          int32_t* argmax_out, float* max_out,
                          void* workspace, size_t workspace_bytes, void* stream);
int mxfp4_woq_gemm_argmax_path(const void* x_bf16, int64_t M, int64_t ldx,
                               const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                               int32_t* argmax_out, float* max_out,
                               void* workspace, size_t workspace_bytes, int path, void* stream);

/*
 * mxfp4_woq_gemm_argmax for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same product,
 * same pick, same bits; the scratch is a buffer of the library's own in device memory
 * (mxfp4_woq_gemm_argmax_noalloc_max_bytes() = 4 MiB per device, held from the time the library is
 * loaded until the process ends).  The call allocates and frees nothing.
 *   - MXFP4_ERR_WORKSPACE when mxfp4_woq_gemm_argmax_workspace_bytes(M, N, K) exceeds that size
 *     (large M with a K that has to be split): use the workspace form then.
 *   - All calls on one device share the one buffer, whose contents are whatever the last call left;
 *     nothing in it needs to start at zero.  Calls that overlap in time on one device (two streams,
 *     two threads) race on it and give unspecified picks: serialise them, or use the workspace form.
 */
size_t mxfp4_woq_gemm_argmax_noalloc_max_bytes(void);
int mxfp4_woq_gemm_argmax_noalloc(const void* x_bf16, int64_t M, int64_t ldx,
                                  const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                                  int32_t* argmax_out, float* max_out, void* stream);

/*
 * The unquantised counterpart, y = x * W^T with BF16 weights: the linear layer as the target
 * model runs it when it verifies draft tokens (section 3.2), and the 2-bytes-per-weight yardstick
 * of the 3.76x in section 3.4.3.  FP32 accumulation, BF16 RNE output, or the fused greedy pick
 * with the same rules and workspace contract as mxfp4_woq_gemm_argmax.
 *   w_bf16 in BF16 [N, K], row stride ldw (ldw >= K, ldw % 8 == 0, base 16-byte aligned);
 *   K a positive multiple of 8, at most MXFP4_MAX_K; the weights of one call stay below 2 GiB.
 * Other arguments as for mxfp4_woq_gemm.  Up to 8 activation rows share one pass over the weights
 * on the vector ALUs (K in phases inside the kernel when the rows do not fit the LDS whole), up
 * to 16 on the matrix cores (M > 8, K % 128 == 0, rows that fit the LDS); more rows take passes.
 */
int mxfp4_bf16_gemm(const void* x_bf16, int64_t M, int64_t ldx,
                    const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                    void* y_bf16, int64_t ldy, void* stream);
size_t mxfp4_bf16_gemm_argmax_workspace_bytes(int64_t M, int64_t N, int64_t K);
int mxfp4_bf16_gemm_argmax(const void* x_bf16, int64_t M, int64_t ldx,
                           const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                           int32_t* argmax_out, float* max_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Verification of a draft in one call (section 3.1): the product with the fused greedy pick, then
 * the comparison with the draft's tokens fused into the pick's last stage.  Row 0 of x belongs
 * to the last accepted token, row m >= 1 to draft token m - 1; the pick of row m is the verifier's
 * token for the position of draft token m.  Draft tokens after the first mismatch are dropped:
 *   draft_tokens in  int32 [M - 1] (device; may be NULL when M == 1)
 *   accept_out   out int32 [2] (device): [0] = G, the number of leading draft tokens that equal
 *                the picks (0 .. M - 1); [1] = the pick at row G, the token the round adds after
 *                them (sections 3.1 and 3.2: G + 1 tokens per verification pass)
 *   argmax_out   out int32 [M], required; max_out may be NULL.
 * M <= 1024.  Workspace as for the matching *_argmax call.  The first form verifies with the
 * MXFP4 weights (the intermediate model of section 3.3 checking the last-level draft), the second
 * with BF16 weights (the target checking the MXFP4 model).
 */
int mxfp4_woq_gemm_verify(const void* x_bf16, int64_t M, int64_t ldx,
                          const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                          const int32_t* draft_tokens, int32_t* accept_out,
                          int32_t* argmax_out, float* max_out,
                          void* workspace, size_t workspace_bytes, void* stream);
int mxfp4_bf16_gemm_verify(const void* x_bf16, int64_t M, int64_t ldx,
                           const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                           const int32_t* draft_tokens, int32_t* accept_out,
                           int32_t* argmax_out, float* max_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Tile-major weights (an internal layout, made once from the canonical tensors; bit-exactness is
 * defined on the canonical ones).  The MFMA tile kernel of the M >= 3 path loads 16 rows x 64 bytes
 * per wave instruction from the row-major tensors; from this copy the same fragment is 1 KiB
 * contiguous, which is worth 10 to 14 % on a verification pass.  The copy serves single rows too
 * (section 3.3: one quantised model drafts and verifies): one row runs a decode kernel of this
 * layout, about 13 % behind the row-major decode kernels over a 7B stack, so a model can keep this
 * copy alone, or both (+0.53 bytes per weight of the 288 GB) for the fastest of each.
 *   q_tiled out uint8, mxfp4_tile_repack_q_bytes(N, K) bytes, 16-byte aligned:
 *           [tile = ceil(N/16)][step = K/128][lane = i + 16 g][16 bytes] = block 4 step + g of row
 *           16 tile + i (rows past N are zero)
 *   s_tiled out uint8, mxfp4_tile_repack_s_bytes(N, K) bytes, 16-byte aligned:
 *           [tile][item = ceil(K/512)][row i][16 scale bytes of blocks 16 item ..] (bytes past K,
 *           rows past N: 0x7F)
 * K % 128 == 0.  The products below take the tile-major pair in place of (q_packed, scales_e8m0)
 * and are otherwise mxfp4_woq_gemm, mxfp4_woq_gemm_ws, mxfp4_woq_gemm_argmax and
 * mxfp4_woq_gemm_verify.  When the activation rows of a pass (min(M, 16) x K BF16) do not fit the
 * LDS of a compute unit next to 8 KB, K is split through the workspace as in mxfp4_woq_gemm_ws
 * (mxfp4_woq_gemm_workspace_bytes(M, N, K) bytes for mxfp4_woq_gemm_tiled_ws; the argmax and
 * verify workspaces of mxfp4_woq_gemm_argmax_workspace_bytes include them); a call of more than
 * eight rows without one (mxfp4_woq_gemm_tiled, a NULL or short workspace) returns MXFP4_ERR_ARG
 * for such a shape, which then goes through the canonical tensors.  Up to eight rows need no
 * workspace at any K (the workgroup walks K in phases); one row (and two, where the tiles cannot
 * run) at any K whose activation rows fit the LDS.
 */
size_t mxfp4_tile_repack_q_bytes(int64_t N, int64_t K);
size_t mxfp4_tile_repack_s_bytes(int64_t N, int64_t K);
int mxfp4_tile_repack(const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                      void* q_tiled, void* s_tiled, void* stream);
int mxfp4_woq_gemm_tiled(const void* x_bf16, int64_t M, int64_t ldx,
                         const void* q_tiled, const void* s_tiled, int64_t N, int64_t K,
                         void* y_bf16, int64_t ldy, void* stream);
int mxfp4_woq_gemm_tiled_ws(const void* x_bf16, int64_t M, int64_t ldx,
                            const void* q_tiled, const void* s_tiled, int64_t N, int64_t K,
                            void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                            void* stream);
int mxfp4_woq_gemm_tiled_argmax(const void* x_bf16, int64_t M, int64_t ldx,
                                const void* q_tiled, const void* s_tiled, int64_t N, int64_t K,
                                int32_t* argmax_out, float* max_out,
                                void* workspace, size_t workspace_bytes, void* stream);
int mxfp4_woq_gemm_tiled_verify(const void* x_bf16, int64_t M, int64_t ldx,
                                const void* q_tiled, const void* s_tiled, int64_t N, int64_t K,
                                const int32_t* draft_tokens, int32_t* accept_out,
                                int32_t* argmax_out, float* max_out,
                                void* workspace, size_t workspace_bytes, void* stream);

/* mxfp4_woq_gemm_fused on the tile-major copy (bias, act, residual, y as there). */
int mxfp4_woq_gemm_tiled_fused(const void* x_bf16, int64_t M, int64_t ldx,
                               const void* q_tiled, const void* s_tiled, int64_t N, int64_t K,
                               const void* bias_bf16, int act, const void* residual_bf16, int64_t ldr,
                               void* y_bf16, int64_t ldy, void* stream);

/* The same decode through the gfx950 scaled FP4->BF16 convert instruction (the one the CVT
 * product path uses), so that its semantics can be checked in isolation. */
int mxfp4_dequant_hwcvt(const void* q_packed, const void* scales_e8m0, int64_t N, int64_t K,
                        void* w_bf16, int64_t ldw, void* stream);

/*
 * Measurement aids, not part of the method: a read-only and a copy kernel over `bytes` bytes
 * (16-byte aligned, multiple of 16) that show what the memory system delivers to plain
 * 128-bit streaming loads.  `sink4` is a 4-byte device scratch word.
 */
int mxfp4_diag_stream_read(const void* src, size_t bytes, void* sink4, void* stream);
int mxfp4_diag_stream_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Host: text of the last error on this thread ("" if none).  Never NULL. */
const char* mxfp4_last_error(void);

/* Host: library version, e.g. "mxfp4-gfx950 0.1". */
const char* mxfp4_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MXFP4_H */
