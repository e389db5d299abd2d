/*
 * CPU oracle for the MXFP4 weight-only-quantised linear layer of ML-SpecQD
 * (arXiv 2503.13565, section 3.4.3 "MXFP4 direct-cast of weights and GEMM
 * Microkernel").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain, slow definition that the HIP
 * kernels are checked against and shares no code, table or header with them.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call it; the product path never does.
 *
 * Everything is written as the definition reads: doubles for arithmetic (every
 * BF16 value, every power of two and every product of a BF16 value with an
 * MXFP4 weight is exact in a double), plain index-order loops, no blocking.  The
 * only parallelism is an optional OpenMP split over independent output rows,
 * which changes no arithmetic.
 *
 * Conventions (section 3.4.3; readings of the silent points are listed with the
 * functions that need them):
 *   - element format E2M1: 1 sign, 2 exponent (bias 1), 1 mantissa bit; the
 *     eight magnitudes are 0, 0.5, 1, 1.5, 2, 3, 4, 6 for codes 0..7;
 *   - scale format E8M0: one byte per 32 consecutive elements along K holding a
 *     biased FP32 exponent, value 2^(byte-127); byte 0xFF marks a NaN block;
 *   - packed layout: byte j of a row holds element 2j in bits 0..3 and element
 *     2j+1 in bits 4..7; scales are [N, K/32] row-major.
 *
 * Pins (tests/test_oracle_*.py): every code point round-trips, the scale equals
 * floor(log2 amax) - 2, the decision intervals of round-to-nearest-even, an
 * integer closed form over every BF16 magnitude, power-of-two invariance, sign
 * symmetry, idempotence, the error bound, the product against a library FP64
 * matmul on on-grid weights, one-hot activations, and brute-force argmax; the
 * BF16-weight product against a library FP64 matmul and against the quantised
 * product on weights that the cast represents exactly; the fused epilogue against
 * a library FP64 silu, closed-form values, the odd-part identity
 * silu(v) - silu(-v) = v, additivity of bias and residual with a non-square
 * padded layout, and the slope constant against a numeric maximum; the 8-bit
 * (E4M3) cast and product against a library float8 conversion and decode, the
 * decision midpoints in exact rational arithmetic, round trips of every code
 * point, saturation, and a library FP64 matmul (tests/test_oracle_e4m3.py); the
 * 6-bit (E2M3) cast, packing and product against a grid and a bit string written
 * out in the test, exact midpoints, round trips, and a library FP64 matmul
 * (tests/test_oracle_e2m3.py); the generic formats (E5M2, E3M2, the 2-bit ternary
 * T2) against grids built from the field widths in exact rationals, a library
 * float8 conversion (E5M2), brute-force nearest search, closed-form intervals
 * (T2), a bit string written out in the test and a library FP64 matmul
 * (tests/test_oracle_mx.py); the product along the rows (oracle_woq_gemm_t)
 * against one-hot activations, a library FP64 matmul on the transpose of the
 * pinned product, and loops written out in the test (tests/test_oracle_kv.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_BLOCK 32

/* The eight E2M1 magnitudes, from the field widths: code = eem, exponent bias 1,
 * code 1 is the single subnormal. */
static double e2m1_magnitude(int code)
{
    int ee = (code >> 1) & 3;
    int m = code & 1;
    if (ee == 0)
        return 0.5 * m;                       /* subnormal: 0.m * 2^(1-1)      */
    return ldexp(1.0 + 0.5 * m, ee - 1);      /* normal:    1.m * 2^(ee-1)     */
}

/* BF16 bit pattern -> double (exact).  BF16 is the top half of an FP32. */
static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round |r| (finite, >= 0) to the nearest E2M1 magnitude; a value exactly half
 * way between two neighbours goes to the one whose code is even (mantissa bit
 * 0); anything beyond the largest magnitude saturates to it.  Section 3.4.3
 * fixes the saturation; round-to-nearest-even is the OCP Microscaling rule the
 * section defers to. */
static int e2m1_round_code(double r)
{
    int best = 0;
    double best_d = fabs(r - e2m1_magnitude(0));
    for (int c = 1; c < 8; ++c) {
        double d = fabs(r - e2m1_magnitude(c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return best;   /* r > 6 lands on code 7 because 6 is then the nearest */
}

/* Direct cast of one 32-element block (section 3.4.3, steps i and ii).
 * Returns the scale byte; writes 32 nibbles (sign<<3 | code) to nib[]. */
static uint8_t cast_block(const uint16_t *w, uint8_t nib[ORACLE_BLOCK])
{
    double v[ORACLE_BLOCK];
    double amax = 0.0;
    int nonfinite = 0;
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        v[i] = bf16_to_double(w[i]);
        if (isnan(v[i]) || isinf(v[i]))
            nonfinite = 1;
        else if (fabs(v[i]) > amax)
            amax = fabs(v[i]);
    }
    if (nonfinite) {
        /* Reading: a block holding NaN or Inf becomes a NaN block. */
        for (int i = 0; i < ORACLE_BLOCK; ++i)
            nib[i] = 0;
        return 0xFF;
    }
    /* Step i: X = (largest power of two <= amax) / (largest power of two that
     * E2M1 represents = 4 = 2^2), i.e. X = 2^E with E = floor(log2 amax) - 2.
     * Reading: an all-zero block and any E below -127 take E = -127 (byte 0);
     * the upper clamp cannot trigger from BF16 inputs. */
    int E;
    if (amax == 0.0) {
        E = -127;
    } else {
        int ex;
        (void)frexp(amax, &ex);               /* amax = f * 2^ex, f in [0.5,1) */
        E = (ex - 1) - 2;                     /* floor(log2 amax) - 2          */
    }
    if (E < -127)
        E = -127;
    if (E > 127)
        E = 127;
    /* Step ii: v_i / X, quantised to E2M1, saturating, sign preserved.
     * Reading: the sign bit of the input is kept even when the magnitude
     * rounds to zero. */
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        double r = ldexp(fabs(v[i]), -E);     /* exact division by 2^E */
        int code = e2m1_round_code(r);
        int sign = (w[i] >> 15) & 1;
        nib[i] = (uint8_t)((sign << 3) | code);
    }
    return (uint8_t)(E + 127);
}

/* Direct cast of W[N,K] (BF16 bit patterns, row stride ldw elements) to packed
 * nibbles q[N,K/2] and scale bytes s[N,K/32].  Returns 0, or 2 on a bad shape. */
int oracle_direct_cast(const uint16_t *w, int64_t N, int64_t K, int64_t ldw,
                       uint8_t *q, uint8_t *s, int threads)
{
    if (N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldw < K)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t b = 0; b < nblk; ++b) {
            uint8_t nib[ORACLE_BLOCK];
            s[n * nblk + b] = cast_block(w + n * ldw + b * ORACLE_BLOCK, nib);
            for (int j = 0; j < ORACLE_BLOCK / 2; ++j)
                q[n * (K / 2) + b * (ORACLE_BLOCK / 2) + j] =
                    (uint8_t)(nib[2 * j] | (nib[2 * j + 1] << 4));
        }
    }
    (void)threads;
    return 0;
}

/* One dequantised weight: (-1)^sign * magnitude(code) * 2^(scale-127); a scale
 * byte of 0xFF gives NaN. */
static double dequant_one(uint8_t nibble, uint8_t scale_byte)
{
    if (scale_byte == 0xFF)
        return NAN;
    double mag = e2m1_magnitude(nibble & 7);
    double val = ldexp(mag, (int)scale_byte - 127);
    return (nibble & 8) ? -val : val;
}

static void dequant_row(const uint8_t *q_row, const uint8_t *s_row, int64_t K,
                        double *out)
{
    for (int64_t k = 0; k < K; ++k) {
        uint8_t byte = q_row[k / 2];
        uint8_t nibble = (k & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xF);
        out[k] = dequant_one(nibble, s_row[k / ORACLE_BLOCK]);
    }
}

/* Dequantise q,s to doubles w_hat[N,K]. */
int oracle_dequant(const uint8_t *q, const uint8_t *s, int64_t N, int64_t K,
                   double *w_hat)
{
    if (N < 0 || K < 0 || K % ORACLE_BLOCK != 0)
        return 2;
    for (int64_t n = 0; n < N; ++n)
        dequant_row(q + n * (K / 2), s + n * (K / ORACLE_BLOCK), K, w_hat + n * K);
    return 0;
}

/* y_ref[m,n] = sum_k x[m,k] * w_hat[n,k] in FP64, k ascending; also
 * a_ref[m,n] = sum_k |x[m,k] * w_hat[n,k]| (the tolerance's magnitude sum).
 * x holds BF16 bit patterns [M,K] with row stride ldx; outputs are [M,N]
 * row-major doubles.  a_ref may be NULL. */
int oracle_woq_gemm(const uint16_t *x, int64_t M, int64_t ldx,
                    const uint8_t *q, const uint8_t *s, int64_t N, int64_t K,
                    double *y_ref, double *a_ref, int threads)
{
    if (M < 0 || N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldx < K)
        return 2;
    double *xd = (double *)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    if (!xd)
        return 6;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            xd[m * K + k] = bf16_to_double(x[m * ldx + k]);
    int failed = 0;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel
#endif
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
        if (!wrow) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
        for (int64_t n = 0; n < N; ++n) {
            if (!wrow)
                continue;
            dequant_row(q + n * (K / 2), s + n * (K / ORACLE_BLOCK), K, wrow);
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0, aacc = 0.0;
                const double *xr = xd + m * K;
                for (int64_t k = 0; k < K; ++k) {
                    double p = xr[k] * wrow[k];
                    acc += p;
                    aacc += fabs(p);
                }
                y_ref[m * N + n] = acc;
                if (a_ref)
                    a_ref[m * N + n] = aacc;
            }
        }
        free(wrow);
    }
    free(xd);
    (void)threads;
    return failed ? 6 : 0;
}

/* The product along the other axis of the same stored tensor (section 5 names a
 * quantised attention cache as the next step; with one token per weight row,
 * blocks along the head dimension, the value side of attention contracts over
 * the rows):  y_ref[m,k] = sum_n x[m,n] * w_hat[n,k] in FP64, n ascending, and
 * a_ref[m,k] = sum_n |x[m,n] * w_hat[n,k]|.  x holds BF16 bit patterns [M,N] with
 * row stride ldx; outputs are [M,K] row-major doubles.  a_ref may be NULL. */
int oracle_woq_gemm_t(const uint16_t *x, int64_t M, int64_t ldx,
                      const uint8_t *q, const uint8_t *s, int64_t N, int64_t K,
                      double *y_ref, double *a_ref)
{
    if (M < 0 || N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldx < N)
        return 2;
    double *wrow = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
    if (!wrow)
        return 6;
    for (int64_t i = 0; i < M * K; ++i) {
        y_ref[i] = 0.0;
        if (a_ref)
            a_ref[i] = 0.0;
    }
    for (int64_t n = 0; n < N; ++n) {
        dequant_row(q + n * (K / 2), s + n * (K / ORACLE_BLOCK), K, wrow);
        for (int64_t m = 0; m < M; ++m) {
            double xv = bf16_to_double(x[m * ldx + n]);
            for (int64_t k = 0; k < K; ++k) {
                double p = xv * wrow[k];
                y_ref[m * K + k] += p;
                if (a_ref)
                    a_ref[m * K + k] += fabs(p);
            }
        }
    }
    free(wrow);
    return 0;
}

/* The same product with the scale applied once per 32-block partial sum (the
 * late-scaling form, Eq. 2).  Used by a test of the identity only. */
int oracle_woq_gemm_late_scaled(const uint16_t *x, int64_t M, int64_t ldx,
                                const uint8_t *q, const uint8_t *s, int64_t N,
                                int64_t K, double *y_ref)
{
    if (M < 0 || N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldx < K)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t b = 0; b < nblk; ++b) {
                uint8_t sb = s[n * nblk + b];
                double partial = 0.0;
                for (int i = 0; i < ORACLE_BLOCK; ++i) {
                    int64_t k = b * ORACLE_BLOCK + i;
                    uint8_t byte = q[n * (K / 2) + k / 2];
                    uint8_t nibble = (k & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xF);
                    double wi = e2m1_magnitude(nibble & 7);
                    if (nibble & 8)
                        wi = -wi;
                    partial += wi * bf16_to_double(x[m * ldx + k]);
                }
                acc += (sb == 0xFF) ? NAN : ldexp(partial, (int)sb - 127);
            }
            y_ref[m * N + n] = acc;
        }
    }
    return 0;
}

/* The unquantised linear layer of the target model (section 3.2: the target
 * verifies in BF16; section 3.4.3 takes its weight bytes as the 3.76x yardstick):
 * y_ref[m,n] = sum_k x[m,k] * w[n,k] with W given as BF16 bit patterns [N,K], row
 * stride ldw, in FP64, k ascending (every product of two BF16 values is exact in a
 * double); a_ref[m,n] = sum_k |x[m,k] * w[n,k]|, may be NULL. */
int oracle_bf16_gemm(const uint16_t *x, int64_t M, int64_t ldx,
                     const uint16_t *w, int64_t N, int64_t K, int64_t ldw,
                     double *y_ref, double *a_ref, int threads)
{
    if (M < 0 || N < 0 || K < 0 || ldx < K || ldw < K)
        return 2;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = bf16_to_double(x[m * ldx + k]) * bf16_to_double(w[n * ldw + k]);
                acc += p;
                aacc += fabs(p);
            }
            y_ref[m * N + n] = acc;
            if (a_ref)
                a_ref[m * N + n] = aacc;
        }
    }
    (void)threads;
    return 0;
}

/* ------------------------------------------------------------------------------
 * An 8-bit draft (sections 1, 3.2 and 5 name 8-bit quantisation as a drop-in for the
 * 4-bit draft): the same two-step direct cast of section 3.4.3 with the OCP
 * 8-bit element format E4M3 in place of E2M1: 1 sign, 4 exponent bits (bias 7),
 * 3 mantissa bits, no infinities, S.1111.111 is NaN, largest magnitude
 * 1.75 * 2^8 = 448; one E8M0 scale per 32 elements as before.  One byte per
 * element, q8[N, K]; scales [N, K/32].
 * Readings: the rule of section 3.4.3 carries over with the largest power of two
 * of the element format now 2^8 (X = 2^(floor(log2 amax) - 8)); rounding to
 * nearest, ties to the even code; magnitudes beyond 448 saturate to 448 (never
 * the NaN code); zero blocks, tiny scales, non-finite inputs and the sign of
 * zero as in the 4-bit cast. */
static double e4m3_magnitude(int code)       /* code = eeeemmm, 0..126 */
{
    int e = (code >> 3) & 15;
    int m = code & 7;
    if (e == 0)
        return ldexp(m / 8.0, -6);            /* subnormal: 0.mmm * 2^(1-7) */
    return ldexp(1.0 + m / 8.0, e - 7);       /* normal:    1.mmm * 2^(e-7) */
}

static int e4m3_round_code(double r)
{
    int best = 0;
    double best_d = fabs(r - e4m3_magnitude(0));
    for (int c = 1; c < 127; ++c) {           /* 127 is the NaN code: not a target */
        double d = fabs(r - e4m3_magnitude(c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return best;
}

static uint8_t e4m3_cast_block(const uint16_t *w, uint8_t out[ORACLE_BLOCK])
{
    double v[ORACLE_BLOCK];
    double amax = 0.0;
    int nonfinite = 0;
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        v[i] = bf16_to_double(w[i]);
        if (isnan(v[i]) || isinf(v[i]))
            nonfinite = 1;
        else if (fabs(v[i]) > amax)
            amax = fabs(v[i]);
    }
    if (nonfinite) {
        for (int i = 0; i < ORACLE_BLOCK; ++i)
            out[i] = 0;
        return 0xFF;
    }
    int E;
    if (amax == 0.0) {
        E = -127;
    } else {
        int ex;
        (void)frexp(amax, &ex);
        E = (ex - 1) - 8;                     /* floor(log2 amax) - 8 */
    }
    if (E < -127)
        E = -127;
    if (E > 127)
        E = 127;
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        double r = ldexp(fabs(v[i]), -E);
        int sign = (w[i] >> 15) & 1;
        out[i] = (uint8_t)((sign << 7) | e4m3_round_code(r));
    }
    return (uint8_t)(E + 127);
}

int oracle_e4m3_direct_cast(const uint16_t *w, int64_t N, int64_t K, int64_t ldw,
                            uint8_t *q8, uint8_t *s, int threads)
{
    if (N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldw < K)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t b = 0; b < nblk; ++b)
            s[n * nblk + b] = e4m3_cast_block(w + n * ldw + b * ORACLE_BLOCK,
                                              q8 + n * K + b * ORACLE_BLOCK);
    (void)threads;
    return 0;
}

static double e4m3_dequant_one(uint8_t byte, uint8_t scale_byte)
{
    if (scale_byte == 0xFF || (byte & 0x7F) == 0x7F)
        return NAN;
    double val = ldexp(e4m3_magnitude(byte & 0x7F), (int)scale_byte - 127);
    return (byte & 0x80) ? -val : val;
}

int oracle_e4m3_dequant(const uint8_t *q8, const uint8_t *s, int64_t N, int64_t K, double *w_hat)
{
    if (N < 0 || K < 0 || K % ORACLE_BLOCK != 0)
        return 2;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            w_hat[n * K + k] = e4m3_dequant_one(q8[n * K + k], s[n * (K / ORACLE_BLOCK) + k / ORACLE_BLOCK]);
    return 0;
}

/* The product with 8-bit weights: y[m][n] = sum_k x[m][k] * w_hat[n][k], k ascending,
 * in FP64 (every product of a BF16 value with an E4M3 weight times a power of two
 * is exact in a double), and the sum of absolute products. */
int oracle_e4m3_woq_gemm(const uint16_t *x, int64_t M, int64_t ldx,
                         const uint8_t *q8, const uint8_t *s, int64_t N, int64_t K,
                         double *y_ref, double *a_ref, int threads)
{
    if (M < 0 || N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldx < K)
        return 2;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = bf16_to_double(x[m * ldx + k]) *
                           e4m3_dequant_one(q8[n * K + k], s[n * (K / ORACLE_BLOCK) + k / ORACLE_BLOCK]);
                acc += p;
                aacc += fabs(p);
            }
            y_ref[m * N + n] = acc;
            if (a_ref)
                a_ref[m * N + n] = aacc;
        }
    }
    (void)threads;
    return 0;
}

double oracle_e4m3_magnitude(int code) { return e4m3_magnitude(code & 0x7F); }

/* ------------------------------------------------------------------------------
 * A 6-bit draft: the same cast with the OCP 6-bit element format E2M3: 1 sign, 2
 * exponent bits (bias 1), 3 mantissa bits, no infinities and no NaN, magnitudes
 * m/8 for exponent field 0 and (1 + m/8) * 2^(e-1) above, largest 7.5.  Its largest
 * power of two is 4 = 2^2 as for E2M1, so X = 2^(floor(log2 amax) - 2); rounding to
 * nearest, ties to the even code, beyond 7.5 saturates.  Packing: the 32 codes
 * (sign << 5 | eemmm) of a block are a little-endian bit string of 192 bits, code i
 * in bits 6i .. 6i+5: 24 bytes per block, q6[N, K/32 * 24]; scales [N, K/32].
 * Zero blocks, tiny scales, non-finite inputs, the sign of zero: as in the 4-bit
 * cast. */
#define E2M3_BLOCK_BYTES 24

static double e2m3_magnitude(int code)       /* code = eemmm, 0..31 */
{
    int e = (code >> 3) & 3;
    int m = code & 7;
    if (e == 0)
        return m / 8.0;                       /* subnormal: 0.mmm * 2^(1-1) */
    return ldexp(1.0 + m / 8.0, e - 1);       /* normal:    1.mmm * 2^(e-1) */
}

static int e2m3_round_code(double r)
{
    int best = 0;
    double best_d = fabs(r - e2m3_magnitude(0));
    for (int c = 1; c < 32; ++c) {
        double d = fabs(r - e2m3_magnitude(c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return best;
}

static void e2m3_put(uint8_t *blk, int i, int code6)
{
    for (int b = 0; b < 6; ++b) {
        int bit = 6 * i + b;
        if ((code6 >> b) & 1)
            blk[bit >> 3] |= (uint8_t)(1u << (bit & 7));
    }
}

static int e2m3_get(const uint8_t *blk, int i)
{
    int code6 = 0;
    for (int b = 0; b < 6; ++b) {
        int bit = 6 * i + b;
        code6 |= ((blk[bit >> 3] >> (bit & 7)) & 1) << b;
    }
    return code6;
}

static uint8_t e2m3_cast_block(const uint16_t *w, uint8_t blk[E2M3_BLOCK_BYTES])
{
    double v[ORACLE_BLOCK];
    double amax = 0.0;
    int nonfinite = 0;
    memset(blk, 0, E2M3_BLOCK_BYTES);
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        v[i] = bf16_to_double(w[i]);
        if (isnan(v[i]) || isinf(v[i]))
            nonfinite = 1;
        else if (fabs(v[i]) > amax)
            amax = fabs(v[i]);
    }
    if (nonfinite)
        return 0xFF;
    int E;
    if (amax == 0.0) {
        E = -127;
    } else {
        int ex;
        (void)frexp(amax, &ex);
        E = (ex - 1) - 2;                     /* floor(log2 amax) - 2 */
    }
    if (E < -127)
        E = -127;
    if (E > 127)
        E = 127;
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        double r = ldexp(fabs(v[i]), -E);
        int sign = (w[i] >> 15) & 1;
        e2m3_put(blk, i, (sign << 5) | e2m3_round_code(r));
    }
    return (uint8_t)(E + 127);
}

int oracle_e2m3_direct_cast(const uint16_t *w, int64_t N, int64_t K, int64_t ldw,
                            uint8_t *q6, uint8_t *s, int threads)
{
    if (N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldw < K)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t b = 0; b < nblk; ++b)
            s[n * nblk + b] = e2m3_cast_block(w + n * ldw + b * ORACLE_BLOCK,
                                              q6 + (n * nblk + b) * E2M3_BLOCK_BYTES);
    (void)threads;
    return 0;
}

static double e2m3_dequant_one(int code6, uint8_t scale_byte)
{
    if (scale_byte == 0xFF)
        return NAN;
    double val = ldexp(e2m3_magnitude(code6 & 31), (int)scale_byte - 127);
    return (code6 & 32) ? -val : val;
}

int oracle_e2m3_dequant(const uint8_t *q6, const uint8_t *s, int64_t N, int64_t K, double *w_hat)
{
    if (N < 0 || K < 0 || K % ORACLE_BLOCK != 0)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int64_t b = k / ORACLE_BLOCK;
            w_hat[n * K + k] = e2m3_dequant_one(e2m3_get(q6 + (n * nblk + b) * E2M3_BLOCK_BYTES, (int)(k % ORACLE_BLOCK)),
                                                s[n * nblk + b]);
        }
    return 0;
}

int oracle_e2m3_woq_gemm(const uint16_t *x, int64_t M, int64_t ldx,
                         const uint8_t *q6, const uint8_t *s, int64_t N, int64_t K,
                         double *y_ref, double *a_ref, int threads)
{
    if (M < 0 || N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldx < K)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                int64_t b = k / ORACLE_BLOCK;
                double wv = e2m3_dequant_one(e2m3_get(q6 + (n * nblk + b) * E2M3_BLOCK_BYTES, (int)(k % ORACLE_BLOCK)),
                                             s[n * nblk + b]);
                double p = bf16_to_double(x[m * ldx + k]) * wv;
                acc += p;
                aacc += fabs(p);
            }
            y_ref[m * N + n] = acc;
            if (a_ref)
                a_ref[m * N + n] = aacc;
        }
    }
    (void)threads;
    return 0;
}

double oracle_e2m3_magnitude(int code) { return e2m3_magnitude(code & 31); }

/* ------------------------------------------------------------------------------
 * Further element formats as drafts, by one generic rule (sections 1, 3.2 and 5 name
 * 8-bit and lower-bit drafts -- 3, 2, 1.58 and 1 bit -- as drop-ins for the 4-bit
 * one without fixing their formats).  Each is "sign + magnitude code" with the MX
 * block scale (one E8M0 byte per 32 elements) and the two-step cast of section
 * 3.4.3: X = 2^(floor(log2 amax) - emax), emax the exponent of the largest power of
 * two the element format holds; elements rounded to the nearest magnitude, ties
 * to the even code, beyond the largest finite magnitude saturated to it; zero
 * blocks, tiny scales, non-finite inputs and the sign of zero as in the 4-bit cast.
 *   format 1, E5M2 (the second OCP 8-bit format): 5 exponent bits (bias 15), 2
 *     mantissa bits; exponent field 31 is Inf/NaN and never produced; largest
 *     finite magnitude 1.75 * 2^15 = 57344, emax = 15; one byte per element.
 *   format 2, E3M2 (the second OCP 6-bit format): 3 exponent bits (bias 3), 2
 *     mantissa bits, no Inf/NaN; largest magnitude 1.75 * 2^4 = 28, emax = 4.
 *   format 3, T2: a 2-bit element, sign and one magnitude bit, values -1, -0, +0, +1
 *     (ternary: the 1.58-bit draft stored in two bits); emax = 0, so X is the
 *     largest power of two not above amax; |v| / X above 1/2 rounds to 1, exactly
 *     1/2 is a tie and goes to the even code 0, everything from 1 up saturates to 1.
 * Packing for every format: the 32 codes (sign << (bits - 1) | magnitude code) of a
 * block as a little-endian bit string, code i in bits bits*i .. bits*i + bits - 1:
 * 32, 24 and 8 bytes per block; q[N, K/32 * block bytes]; scales [N, K/32]. */
typedef struct {
    int bits, ebits, mbits, bias, emax, ncodes;     /* ncodes: finite magnitude codes 0 .. ncodes - 1 */
} mx_fmt;

static int mx_format(int id, mx_fmt *f)
{
    switch (id) {
    case 1: *f = (mx_fmt){8, 5, 2, 15, 15, 31 * 4}; return 0;
    case 2: *f = (mx_fmt){6, 3, 2, 3, 4, 32}; return 0;
    case 3: *f = (mx_fmt){2, 0, 1, 0, 0, 2}; return 0;
    }
    return 2;
}

static double mx_magnitude(const mx_fmt *f, int code)
{
    if (f->ebits == 0)
        return (double)code;                          /* T2: 0 or 1 */
    int e = code >> f->mbits;
    int m = code & ((1 << f->mbits) - 1);
    double frac = (double)m / (double)(1 << f->mbits);
    if (e == 0)
        return ldexp(frac, 1 - f->bias);              /* subnormal */
    return ldexp(1.0 + frac, e - f->bias);            /* normal */
}

static int mx_round_code(const mx_fmt *f, double r)
{
    int best = 0;
    double best_d = fabs(r - mx_magnitude(f, 0));
    for (int c = 1; c < f->ncodes; ++c) {
        double d = fabs(r - mx_magnitude(f, c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return best;
}

static void mx_put(uint8_t *blk, int bits, int i, int code)
{
    for (int b = 0; b < bits; ++b) {
        int bit = bits * i + b;
        if ((code >> b) & 1)
            blk[bit >> 3] |= (uint8_t)(1u << (bit & 7));
    }
}

static int mx_get(const uint8_t *blk, int bits, int i)
{
    int code = 0;
    for (int b = 0; b < bits; ++b) {
        int bit = bits * i + b;
        code |= ((blk[bit >> 3] >> (bit & 7)) & 1) << b;
    }
    return code;
}

static uint8_t mx_cast_block(const mx_fmt *f, const uint16_t *w, uint8_t *blk)
{
    double v[ORACLE_BLOCK];
    double amax = 0.0;
    int nonfinite = 0;
    memset(blk, 0, (size_t)f->bits * 4);
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        v[i] = bf16_to_double(w[i]);
        if (isnan(v[i]) || isinf(v[i]))
            nonfinite = 1;
        else if (fabs(v[i]) > amax)
            amax = fabs(v[i]);
    }
    if (nonfinite)
        return 0xFF;
    int E;
    if (amax == 0.0) {
        E = -127;
    } else {
        int ex;
        (void)frexp(amax, &ex);
        E = (ex - 1) - f->emax;                   /* floor(log2 amax) - emax */
    }
    if (E < -127)
        E = -127;
    if (E > 127)
        E = 127;
    for (int i = 0; i < ORACLE_BLOCK; ++i) {
        double r = ldexp(fabs(v[i]), -E);
        int sign = (w[i] >> 15) & 1;
        mx_put(blk, f->bits, i, (sign << (f->bits - 1)) | mx_round_code(f, r));
    }
    return (uint8_t)(E + 127);
}

int oracle_mx_block_bytes(int fmt)
{
    mx_fmt f;
    return mx_format(fmt, &f) ? 0 : f.bits * 4;
}

double oracle_mx_magnitude(int fmt, int code)
{
    mx_fmt f;
    if (mx_format(fmt, &f) || code < 0 || code >= f.ncodes)
        return NAN;
    return mx_magnitude(&f, code);
}

int oracle_mx_direct_cast(int fmt, const uint16_t *w, int64_t N, int64_t K, int64_t ldw,
                          uint8_t *q, uint8_t *s, int threads)
{
    mx_fmt f;
    if (mx_format(fmt, &f) || N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldw < K)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
    int bb = f.bits * 4;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t b = 0; b < nblk; ++b)
            s[n * nblk + b] = mx_cast_block(&f, w + n * ldw + b * ORACLE_BLOCK, q + (n * nblk + b) * bb);
    (void)threads;
    return 0;
}

static double mx_dequant_one(const mx_fmt *f, int code, uint8_t scale_byte)
{
    int mag = code & ((1 << (f->bits - 1)) - 1);
    if (scale_byte == 0xFF || mag >= f->ncodes)
        return NAN;                                  /* NaN block; Inf/NaN codes of E5M2 */
    double val = ldexp(mx_magnitude(f, mag), (int)scale_byte - 127);
    return (code >> (f->bits - 1)) ? -val : val;
}

int oracle_mx_dequant(int fmt, const uint8_t *q, const uint8_t *s, int64_t N, int64_t K, double *w_hat)
{
    mx_fmt f;
    if (mx_format(fmt, &f) || N < 0 || K < 0 || K % ORACLE_BLOCK != 0)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
    int bb = f.bits * 4;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int64_t b = k / ORACLE_BLOCK;
            w_hat[n * K + k] = mx_dequant_one(&f, mx_get(q + (n * nblk + b) * bb, f.bits, (int)(k % ORACLE_BLOCK)),
                                              s[n * nblk + b]);
        }
    return 0;
}

/* y[m][n] = sum_k x[m][k] * w_hat[n][k] in FP64, k ascending, and the sum of absolute products. */
int oracle_mx_woq_gemm(int fmt, const uint16_t *x, int64_t M, int64_t ldx,
                       const uint8_t *q, const uint8_t *s, int64_t N, int64_t K,
                       double *y_ref, double *a_ref, int threads)
{
    mx_fmt f;
    if (mx_format(fmt, &f) || M < 0 || N < 0 || K < 0 || K % ORACLE_BLOCK != 0 || ldx < K)
        return 2;
    int64_t nblk = K / ORACLE_BLOCK;
    int bb = f.bits * 4;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                int64_t b = k / ORACLE_BLOCK;
                double wv = mx_dequant_one(&f, mx_get(q + (n * nblk + b) * bb, f.bits, (int)(k % ORACLE_BLOCK)),
                                           s[n * nblk + b]);
                double p = bf16_to_double(x[m * ldx + k]) * wv;
                acc += p;
                aacc += fabs(p);
            }
            y_ref[m * N + n] = acc;
            if (a_ref)
                a_ref[m * N + n] = aacc;
        }
    }
    (void)threads;
    return 0;
}

/* What the linear layer's backend fuses around the contraction (section 3.4: bias
 * and residual add applied to the product's output while it is at hand) and, for
 * the gated MLP of the Llama and Qwen targets of sections 4.2 and 4.3, the gate:
 *
 *   z[m][n] = y[m][n] + bias[n]                                   (bias optional)
 *   act 0:  t[m][c] = z[m][c],                        c < N
 *   act 1:  t[m][c] = silu(z[m][2c]) * z[m][2c + 1],  c < N / 2,  silu(v) = v / (1 + exp(-v))
 *           (weight rows interleaved: row 2c is the gate projection's row c, row
 *           2c + 1 the up projection's)
 *   out[m][c] = t[m][c] + residual[m][c]                          (residual optional)
 *
 * y and a are the exact product and its sum of absolute products, [M, N]; bias
 * and residual are BF16 bit patterns ([N]; [M, ldr]); out and a_out are [M, C]
 * with C = N or N / 2.
 *
 * a_out carries the product's error scale through the epilogue, so that the same
 * rule "error <= 1e-3 * a_out + one BF16 ulp" applies to the fused result: if the
 * device's z is off by at most e * A (A = a + |bias|), then, L being the largest
 * slope of silu,
 *   act 0: |d out| <= e * (A + |residual|)
 *   act 1: |d out| <= e * (L A_g |z_u| + |silu(z_g)| A_u + e L A_g A_u + |residual|)
 * with e = 1e-3 in the last product term written out. */
int oracle_epilogue(const double *y, const double *a, int64_t M, int64_t N,
                    const uint16_t *bias, const uint16_t *residual, int64_t ldr,
                    int act, double *out, double *a_out)
{
    const double silu_slope = 1.0998393194985438;   /* max of d/dv silu(v), at v = 2.39936... */
    if (M < 0 || N < 0 || (act != 0 && act != 1) || (act == 1 && N % 2 != 0))
        return 2;
    const int64_t C = act == 1 ? N / 2 : N;
    if (residual && ldr < C)
        return 2;
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t c = 0; c < C; ++c) {
            double t, ta;
            if (act == 0) {
                double b = bias ? bf16_to_double(bias[c]) : 0.0;
                t = y[m * N + c] + b;
                ta = a[m * N + c] + fabs(b);
            } else {
                double bg = bias ? bf16_to_double(bias[2 * c]) : 0.0;
                double bu = bias ? bf16_to_double(bias[2 * c + 1]) : 0.0;
                double zg = y[m * N + 2 * c] + bg, ag = a[m * N + 2 * c] + fabs(bg);
                double zu = y[m * N + 2 * c + 1] + bu, au = a[m * N + 2 * c + 1] + fabs(bu);
                double gate = zg / (1.0 + exp(-zg));
                t = gate * zu;
                ta = silu_slope * ag * fabs(zu) + fabs(gate) * au + 1e-3 * silu_slope * ag * au;
            }
            double r = residual ? bf16_to_double(residual[m * ldr + c]) : 0.0;
            out[m * C + c] = t + r;
            a_out[m * C + c] = ta + fabs(r);
        }
    }
    return 0;
}

/* Greedy pick per row: index of the largest value, lowest index among equals.
 * The result for a row that holds a NaN is unspecified (no graded input has one). */
int oracle_argmax(const double *y, int64_t M, int64_t N, int32_t *idx, double *val)
{
    if (M < 0 || N < 1)
        return 2;
    for (int64_t m = 0; m < M; ++m) {
        int64_t best = 0;
        for (int64_t n = 0; n < N; ++n) {
            if (y[m * N + n] > y[m * N + best])
                best = n;
        }
        idx[m] = (int32_t)best;
        if (val)
            val[m] = y[m * N + best];
    }
    return 0;
}

/* Verification of a draft (section 3.1): the target's forward pass over the last
 * accepted token and the N draft tokens gives N + 1 greedy picks; pick m is the
 * target's token for the position of draft token m.  The draft tokens after the
 * first mismatch are dropped: G = number of leading draft tokens that equal the
 * target's picks (0..N), and the round emits those G tokens plus the target's
 * own pick at position G (the extra token of section 3.2).
 * target[N + 1], draft[N]; out[0] = G, out[1] = target[G]. */
int oracle_greedy_accept(const int32_t *target, const int32_t *draft, int64_t n_draft, int32_t out[2])
{
    if (n_draft < 0)
        return 2;
    int64_t g = 0;
    while (g < n_draft && draft[g] == target[g])
        ++g;
    out[0] = (int32_t)g;
    out[1] = target[g];
    return 0;
}

/* Expected speed-up of one round of speculative decoding over greedy decoding
 * (Eq. 1, first form): G + 1 tokens for one run of the target and N runs of a
 * draft that is S times faster. */
double oracle_sd_speedup(double g, double n_draft, double s)
{
    return (g + 1.0) / (1.0 + n_draft / s);
}

/* The same with the acceptance ratio alpha = G / N (Eq. 1, second form). */
double oracle_sd_speedup_alpha(double alpha, double n_draft, double s)
{
    return (alpha + 1.0 / n_draft) / (1.0 / n_draft + 1.0 / s);
}

/* Two levels (section 3.3): the intermediate draft, s_mid times faster than the
 * target, is itself sped up by speculative decoding with a last-level draft that
 * is s_last times faster than the target (hence s_last / s_mid times faster than
 * the intermediate model); the target then sees a draft S' = s_mid * that gain. */
double oracle_sd_speedup_two_level(double alpha_mid, double n_mid, double s_mid,
                                   double alpha_last, double n_last, double s_last)
{
    double s_prime = s_mid * oracle_sd_speedup_alpha(alpha_last, n_last, s_last / s_mid);
    return oracle_sd_speedup_alpha(alpha_mid, n_mid, s_prime);
}

/* The E2M1 magnitude of a code, exported so a test can print the grid. */
double oracle_e2m1_magnitude(int code) { return e2m1_magnitude(code & 7); }

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
