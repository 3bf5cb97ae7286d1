/*
 * CPU oracle for the fine-grained W4A8 linear layer with integer group scales.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP kernels are checked against.  It shares no code with them and nothing in
 * the product path may call it: only the tests, the smoke check and the
 * benchmark's CPU-baseline leg load this library.
 *
 * What it follows (all citations are to the Integer Scale paper):
 *   - Appendix A.1, symmetric quantisation: s = |X|max / (2^(n-1) - 1),
 *     Q = clamp(round(X / s), -2^(n-1), 2^(n-1) - 1); Appendix A.2 for the
 *     per-token (activations) and group-wise (weights, along K) granularities;
 *     Sec. 5.1 fixes per-token activations and symmetric group-128 weights.
 *   - Eq. (1): O = s_a * sum_g (X_g W_g^T) * s_g            (float group scales)
 *   - Eq. (2): O = s_a * FLOAT( sum_g (X_g W_g^T) * INT(s_g * alpha) ) / alpha
 *   - Table 2, columns "Atom" and "Ours": the per-group recurrences
 *     C_g = A_g W_g ; C' += float(C_g) * s_g     and     C'' += C_g * s_g^INT.
 *   - Sec. 4.1 / Listing 1: the amplifier is the first power of two that lifts
 *     the smallest scale to at least 1.
 *
 * Readings taken where the paper is silent (the same ones the HIP path takes):
 *   - rounding is round-half-to-even, for Q(.) and for INT(.);
 *   - decisions that produce integers (q, xq, IS) are taken in IEEE fp32 with a
 *     true division, because the fp32 quotient decides the integer code;
 *   - alpha is a power of two, given as its log2;
 *   - scale mode RAW: IS = round(s * alpha), channel scale c = 1 (literal Eq. 2);
 *     scale mode NORM: c[n] = max_g s[n,g], IS = round(s / c * alpha), and the
 *     epilogue multiplies by c[n] (scales normalised into (0,1], Sec. 4.1);
 *   - an all-zero group or row has scale 0 and all codes 0;
 *   - the running accumulator is a 32-bit integer that wraps modulo 2^32; the
 *     oracle adds in 64 bits, reports the true sum and the largest |prefix| seen
 *     (Appendix A.5 discusses the overflow risk), and exports the wrapped value.
 *
 * Layouts (row-major, host memory):
 *   w, x       float32 holding fp16-representable values  [N,K] / [M,K]
 *   qweight    uint8 [N, K/2]; byte j of row n holds q[n,2j] in bits 0-3 and
 *              q[n,2j+1] in bits 4-7, each a two's-complement nibble
 *   scale_f32, scale_i32   [N, K/G];   chan_scale [N];   a_scale [M]
 *   xq int8 [M,K];   acc int32 [M,N];   out double [M,N]
 *
 * Parity pins live in tests/test_oracle_*.py (hand-worked examples, brute
 * force, closed forms, invariants).  Accuracy on the paper's datasets is
 * "parity unpinned": neither the datasets nor the model weights are available.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)

static int nibble_to_int(unsigned v) {
    v &= 0xFu;
    return v >= 8u ? (int)v - 16 : (int)v;
}

static int check_shape(int rows, int K, int G) {
    if (rows <= 0 || K <= 0 || G <= 0) return 0;
    if (K % G != 0 || (K & 1) || (G & 1)) return 0;
    return 1;
}

/* Sec. 4.1 / Listing 1: smallest i >= 0 with scale_min * 2^i >= 1, over the
 * non-zero scales; 0 when the smallest scale is already >= 1; capped at 16. */
int oracle_amplifier_log2(const float* scales, long count) {
    float smin = INFINITY;
    for (long i = 0; i < count; ++i)
        if (scales[i] > 0.0f && scales[i] < smin) smin = scales[i];
    if (!isfinite(smin)) return 0;
    int i = 0;
    while (i < 16 && ldexpf(smin, i) < 1.0f) ++i;
    return i;
}

/* Appendix A.1 with n = 4 on every (row, group); then INT(s * alpha) of Eq. (2). */
int oracle_quantize_weights_int4_group(const float* w, int N, int K, int G, int alpha_log2, int scale_mode,
                                       uint8_t* qweight, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                       int* alpha_log2_out) {
    if (!w || !qweight || !scale_f32 || !scale_i32 || !chan_scale) return ORACLE_BAD_ARG;
    if (!check_shape(N, K, G)) return ORACLE_BAD_ARG;
    if (alpha_log2 < -1 || alpha_log2 > 16) return ORACLE_BAD_ARG;
    if (scale_mode != 0 && scale_mode != 1) return ORACLE_BAD_ARG;
    const int NG = K / G;

#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float* wr = w + (size_t)n * K;
        uint8_t* qr = qweight + (size_t)n * (K / 2);
        for (int g = 0; g < NG; ++g) {
            float amax = 0.0f;
            for (int k = g * G; k < (g + 1) * G; ++k) {
                float a = fabsf(wr[k]);
                if (a > amax) amax = a;
            }
            float s = amax / 7.0f;
            scale_f32[(size_t)n * NG + g] = s;
            for (int k = g * G; k < (g + 1) * G; ++k) {
                int q = 0;
                if (s > 0.0f) {
                    float r = rintf(wr[k] / s);
                    if (r < -8.0f) r = -8.0f;
                    if (r > 7.0f) r = 7.0f;
                    q = (int)r;
                }
                unsigned nib = (unsigned)q & 0xFu;
                if (k & 1)
                    qr[k >> 1] = (uint8_t)(qr[k >> 1] | (nib << 4));
                else
                    qr[k >> 1] = (uint8_t)nib;
            }
        }
        float c = 1.0f;
        if (scale_mode == 1) {
            c = 0.0f;
            for (int g = 0; g < NG; ++g)
                if (scale_f32[(size_t)n * NG + g] > c) c = scale_f32[(size_t)n * NG + g];
        }
        chan_scale[n] = c;
    }

    /* The values that get amplified: s itself (RAW) or s / c (NORM). */
    float* amplified = (float*)malloc(sizeof(float) * (size_t)N * NG);
    if (!amplified) return ORACLE_BAD_ARG;
    for (int n = 0; n < N; ++n)
        for (int g = 0; g < NG; ++g) {
            float s = scale_f32[(size_t)n * NG + g];
            float v = s;
            if (scale_mode == 1) v = chan_scale[n] > 0.0f ? s / chan_scale[n] : 0.0f;
            amplified[(size_t)n * NG + g] = v;
        }
    int a = alpha_log2;
    if (a < 0) a = oracle_amplifier_log2(amplified, (long)N * NG);
    if (alpha_log2_out) *alpha_log2_out = a;
    for (size_t i = 0; i < (size_t)N * NG; ++i) scale_i32[i] = (int32_t)rintf(ldexpf(amplified[i], a));
    free(amplified);
    return ORACLE_OK;
}

/* Appendix A.1 with n = 8 on every token row. */
int oracle_quantize_act_int8_token(const float* x, int M, int K, int8_t* xq, float* a_scale) {
    if (!x || !xq || !a_scale || M <= 0 || K <= 0) return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        const float* xr = x + (size_t)m * K;
        float amax = 0.0f;
        for (int k = 0; k < K; ++k) {
            float a = fabsf(xr[k]);
            if (a > amax) amax = a;
        }
        float s = amax / 127.0f;
        a_scale[m] = s;
        for (int k = 0; k < K; ++k) {
            int q = 0;
            if (s > 0.0f) {
                float r = rintf(xr[k] / s);
                if (r < -128.0f) r = -128.0f;
                if (r > 127.0f) r = 127.0f;
                q = (int)r;
            }
            xq[(size_t)m * K + k] = (int8_t)q;
        }
    }
    return ORACLE_OK;
}

static void unpack_row(const uint8_t* qr, int K, int8_t* dst) {
    for (int k = 0; k < K; ++k) {
        unsigned byte = qr[k >> 1];
        dst[k] = (int8_t)nibble_to_int((k & 1) ? (byte >> 4) : byte);
    }
}

/* C_g = A_g W_g of Table 2: the integer partial product of one group. */
static int32_t group_partial(const int8_t* xr, const int8_t* wr, int k0, int G) {
    int32_t p = 0;
    for (int k = k0; k < k0 + G; ++k) p += (int32_t)xr[k] * (int32_t)wr[k];
    return p;
}

/* All group partials P[m,n,g] (int32 [M,N,K/G]); used by tests that need them on their own. */
int oracle_group_partials(const int8_t* xq, const uint8_t* qweight, int M, int N, int K, int G, int32_t* partials) {
    if (!xq || !qweight || !partials || M <= 0 || !check_shape(N, K, G)) return ORACLE_BAD_ARG;
    const int NG = K / G;
#pragma omp parallel
    {
        int8_t* wrow = (int8_t*)malloc((size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            unpack_row(qweight + (size_t)n * (K / 2), K, wrow);
            for (int m = 0; m < M; ++m)
                for (int g = 0; g < NG; ++g)
                    partials[((size_t)m * N + n) * NG + g] = group_partial(xq + (size_t)m * K, wrow, g * G, G);
        }
        free(wrow);
    }
    return ORACLE_OK;
}

/*
 * Eq. (2) with the Table 2 "Ours" recurrence.
 *   acc32       int32 [M,N]  the 32-bit running accumulator after the last group (wrapped modulo 2^32)
 *   out         double [M,N] FLOAT(acc32) * s_a[m] * c[n] / alpha   (not yet rounded to fp16)
 *   acc64       optional int64 [M,N]  the same sum without wrap
 *   max_prefix  optional int64 [M,N]  max over g of |sum of the first g+1 terms| (overflow diagnosis)
 * chan_scale may be NULL (c = 1).
 */
int oracle_gemm_w4a8_intscale(const int8_t* xq, const float* a_scale, const uint8_t* qweight, const int32_t* scale_i32,
                              const float* chan_scale, int M, int N, int K, int G, int alpha_log2, int32_t* acc32,
                              double* out, int64_t* acc64, int64_t* max_prefix) {
    if (!xq || !a_scale || !qweight || !scale_i32 || !acc32 || !out) return ORACLE_BAD_ARG;
    if (M <= 0 || !check_shape(N, K, G)) return ORACLE_BAD_ARG;
    if (alpha_log2 < 0 || alpha_log2 > 30) return ORACLE_BAD_ARG;
    const int NG = K / G;
    const double inv_alpha = ldexp(1.0, -alpha_log2);
#pragma omp parallel
    {
        int8_t* wrow = (int8_t*)malloc((size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            unpack_row(qweight + (size_t)n * (K / 2), K, wrow);
            const double c = chan_scale ? (double)chan_scale[n] : 1.0;
            for (int m = 0; m < M; ++m) {
                int64_t acc = 0, peak = 0;
                for (int g = 0; g < NG; ++g) {
                    int32_t p = group_partial(xq + (size_t)m * K, wrow, g * G, G);
                    acc += (int64_t)p * (int64_t)scale_i32[(size_t)n * NG + g];
                    int64_t mag = acc < 0 ? -acc : acc;
                    if (mag > peak) peak = mag;
                }
                int32_t wrapped = (int32_t)(uint32_t)((uint64_t)acc & 0xFFFFFFFFull);
                size_t o = (size_t)m * N + n;
                acc32[o] = wrapped;
                out[o] = (double)wrapped * (double)a_scale[m] * c * inv_alpha;
                if (acc64) acc64[o] = acc;
                if (max_prefix) max_prefix[o] = peak;
            }
        }
        free(wrow);
    }
    return ORACLE_OK;
}

/*
 * Eq. (1) with the Table 2 "Atom" recurrence, in double.
 *   out      double [M,N]  s_a[m] * sum_g float(P_g) * s_g
 *   abs_sum  optional double [M,N]  s_a[m] * sum_g |P_g| * s_g  (sizes the fp32 summation-order tolerance)
 */
int oracle_gemm_w4a8_floatscale(const int8_t* xq, const float* a_scale, const uint8_t* qweight, const float* scale_f32,
                                int M, int N, int K, int G, double* out, double* abs_sum) {
    if (!xq || !a_scale || !qweight || !scale_f32 || !out) return ORACLE_BAD_ARG;
    if (M <= 0 || !check_shape(N, K, G)) return ORACLE_BAD_ARG;
    const int NG = K / G;
#pragma omp parallel
    {
        int8_t* wrow = (int8_t*)malloc((size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            unpack_row(qweight + (size_t)n * (K / 2), K, wrow);
            for (int m = 0; m < M; ++m) {
                double acc = 0.0, mag = 0.0;
                for (int g = 0; g < NG; ++g) {
                    int32_t p = group_partial(xq + (size_t)m * K, wrow, g * G, G);
                    double t = (double)p * (double)scale_f32[(size_t)n * NG + g];
                    acc += t;
                    mag += fabs(t);
                }
                size_t o = (size_t)m * N + n;
                out[o] = (double)a_scale[m] * acc;
                if (abs_sum) abs_sum[o] = (double)a_scale[m] * mag;
            }
        }
        free(wrow);
    }
    return ORACLE_OK;
}

/* Number of threads the parallel loops above use (reported next to timings). */
int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
