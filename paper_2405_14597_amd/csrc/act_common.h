// Device helpers shared by the activation quantiser and by the kernels that fold it into the operator producing the
// activation: wave and workgroup reductions, and Appendix A.1's code for eight fp16 values at a time.  The quotient
// x / s is a true IEEE fp32 division and rounding is round-half-to-even, because they decide the integer code.
#pragma once
#include "is_common.h"

namespace intscale {

// Maximum over the 64 lanes of a wave, for values that are >= 0 in every lane (an absmax): their bit patterns order
// like unsigned integers.  Four lane-swizzled steps inside each row of 16 lanes (neighbour, pair, mirrored half,
// mirrored row), then the four row results meet in scalar registers.  No trip through the LDS crossbar, whose
// latency would sit six times in a row on the critical path of a one-token kernel.
__device__ __forceinline__ float wave_max(float v) {
    unsigned x = __float_as_uint(v);
    x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, true));  // row_half_mirror
    x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, true));  // row_mirror
    const unsigned r0 = __builtin_amdgcn_readlane((int)x, 0), r1 = __builtin_amdgcn_readlane((int)x, 16);
    const unsigned r2 = __builtin_amdgcn_readlane((int)x, 32), r3 = __builtin_amdgcn_readlane((int)x, 48);
    return __uint_as_float(max(max(r0, r1), max(r2, r3)));
}

__device__ __forceinline__ float absmax8(uint4 v) {
    const __half2* h = reinterpret_cast<const __half2*>(&v);
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 f = __half22float2(h[i]);
        m = fmaxf(m, fmaxf(fabsf(f.x), fabsf(f.y)));
    }
    return m;
}

// e^t and SiLU(g) * u as fixed sequences of separately rounded single-precision operations (no contraction into
// fused multiply-adds): the fp16 result may decide integer codes further on, so every user computes it the same way.
__device__ __forceinline__ float exp_steps(float t) {
#pragma clang fp contract(off)
    t = fminf(fmaxf(t, -87.0f), 88.0f);
    const float n = rintf(t * 1.4426950408889634f);
    const float r = (t - n * 0.693145751953125f) - n * 1.428606765330187e-06f;
    float p = (float)(1.0 / 720.0);
    p = p * r + (float)(1.0 / 120.0);
    p = p * r + (float)(1.0 / 24.0);
    p = p * r + (float)(1.0 / 6.0);
    p = p * r + 0.5f;
    p = p * r + 1.0f;
    p = p * r + 1.0f;
    return ldexpf(p, (int)n);
}

// A single-precision value that is about to be converted to fp16, as the rounded fp32 value it is: without this the
// compiler may merge the last multiply into the conversion (v_fma_mixlo_f16 rounds the exact product once, straight to
// fp16), which differs from "round to fp32, then to fp16" wherever the fp32 result falls on an fp16 tie.
__device__ __forceinline__ float rounded_f32(float v) {
    asm("" : "+v"(v));
    return v;
}

__device__ __forceinline__ float silu_mul(float g, float u) {
#pragma clang fp contract(off)
    const float e = exp_steps(-g);
    return rounded_f32((g / (1.0f + e)) * u);
}


__device__ __forceinline__ int quant_code(float x, float s, float lo, float hi) {
    // s > 0 is checked by the caller
    float r = rintf(x / s);
    r = fminf(fmaxf(r, lo), hi);
    return (int)r;
}

// ---------------------------------------------------------------------------------------------------------
// Activations: one workgroup per token row.  Pass 1 finds the row's absmax (16-byte loads), pass 2 re-reads the
// row (it is at most a few tens of KB, so it comes back from L2) and writes 8 codes per lane as one 8-byte store.
// ---------------------------------------------------------------------------------------------------------
constexpr int kActThreads = 256;

// Appendix A.1 codes of N values of one token row: clamp(rne(x / s)) with the quotient rounded as a true division
// rounds it.  A division costs a dozen instructions, so the codes are first taken from t = x * (1 / s): t and the
// correctly rounded quotient both lie within 1.6e-5 of x / s (|x / s| <= 127, three roundings of 2^-24), so whenever t
// is at least 5e-5 away from the nearest half-integer the two round to the same integer.  If any value of the wave
// comes closer, all N are redone with the division itself (about one chunk of eight in thirty).
// CLAMP = false leaves the range to the caller (quantize8 below, whose packing saturates).
template <int N, bool CLAMP = true>
__device__ __forceinline__ void quant_codes(const float (&x)[N], float s, float (&q)[N]) {
    if (s > 0.0f) {
        const float r = 1.0f / s;
        float far = 0.0f;  // the largest distance of a t from its integer (one running maximum: a flag per value, or-ed
                           // together, is several instructions per value once the compiler has packed the flags into bytes)
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float t = x[i] * r;
            q[i] = rintf(t);
            far = fmaxf(far, fabsf(t - q[i]));
        }
        if (__any(far > 0.49995f)) {
#pragma unroll
            for (int i = 0; i < N; ++i) q[i] = rintf(x[i] / s);
        }
        if constexpr (CLAMP) {
#pragma unroll
            for (int i = 0; i < N; ++i) q[i] = fminf(fmaxf(q[i], -128.0f), 127.0f);
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) q[i] = 0.0f;
    }
}

__device__ __forceinline__ uint2 quantize8(uint4 v, float s) {
    const __half2* h = reinterpret_cast<const __half2*>(&v);
    float x[8], q[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 f = __half22float2(h[i]);
        x[2 * i] = f.x;
        x[2 * i + 1] = f.y;
    }
    quant_codes<8, false>(x, s, q);
    // Codes to bytes: q + 128 (exact: q is an integer) goes through the saturating float -> unsigned byte conversion
    // that also inserts the byte into its word (the clamp to [-128, 127] of Appendix A.1 is that saturation), and
    // flipping the top bit of every byte turns the offset form into two's complement.  Three instructions per code
    // fewer than clamp, convert, mask and shift.
    uint32_t packed[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) packed[i >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(q[i] + 128.0f, i & 3, packed[i >> 2]);
    return make_uint2(packed[0] ^ 0x80808080u, packed[1] ^ 0x80808080u);
}

// NW = waves in the workgroup; `red` holds NW floats
template <int NW = kActThreads / kWave>
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    v = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) v = fmaxf(v, red[i]);
    return v;
}

}  // namespace intscale
