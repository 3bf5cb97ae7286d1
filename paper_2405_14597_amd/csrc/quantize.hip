// Quantisers of the W4A8 layer for gfx950: per-token int8 activations (online) and group-wise int4 weights with
// the integer-scale derivation (offline).  Symmetric quantisation follows Appendix A.1 of the Integer Scale paper
// (s = absmax / (2^(n-1) - 1), Q = clamp(round(x / s))), the integer scale INT(s * alpha) follows Eq. (2) and the
// amplifier search follows Sec. 4.1.  Rounding is round-half-to-even and the quotient x / s is a true IEEE fp32
// division, because that quotient decides the integer code.
#include "act_common.h"
#include "is_common.h"

namespace intscale {
namespace {

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Rows of up to 2048 * CH elements: the row is read once and stays in registers (CH 16-byte chunks per lane) between
// the absmax reduction and the rounding, so a token row costs one trip to memory, not two.  With few rows (a decode
// step) a row is spread over up to 1024 lanes: the chip is far from full and the row's latency is what counts.
template <int CH, int THREADS>
__global__ __launch_bounds__(THREADS) void quantize_act_resident_kernel(const __half* __restrict__ x, int M, int K,
                                                                        int8_t* __restrict__ xq,
                                                                        float* __restrict__ a_scale) {
    __shared__ float red[THREADS / kWave];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const int nchunk = K >> 3;
    const uint4* row = reinterpret_cast<const uint4*>(x + (size_t)m * K);
    uint4 v[CH];
    float amax = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int idx = tid + c * THREADS;
        v[c] = idx < nchunk ? row[idx] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) amax = fmaxf(amax, absmax8(v[c]));
    amax = block_max<THREADS / kWave>(amax, red);
    const float s = amax / 127.0f;
    if (tid == 0) a_scale[m] = s;
    uint2* dst = reinterpret_cast<uint2*>(xq + (size_t)m * K);
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int idx = tid + c * THREADS;
        if (idx < nchunk) dst[idx] = quantize8(v[c], s);
    }
}

// Longer rows: two passes, the second re-reads the row (from L2).
__global__ __launch_bounds__(kActThreads) void quantize_act_kernel(const __half* __restrict__ x, int M, int K,
                                                                   int8_t* __restrict__ xq,
                                                                   float* __restrict__ a_scale) {
    __shared__ float red[kActThreads / kWave];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const int nchunk = K >> 3;
    const uint4* row = reinterpret_cast<const uint4*>(x + (size_t)m * K);
    float amax = 0.0f;
    for (int c = tid; c < nchunk; c += kActThreads) amax = fmaxf(amax, absmax8(row[c]));
    amax = block_max(amax, red);
    const float s = amax / 127.0f;
    if (tid == 0) a_scale[m] = s;
    uint2* dst = reinterpret_cast<uint2*>(xq + (size_t)m * K);
    for (int c = tid; c < nchunk; c += kActThreads) dst[c] = quantize8(row[c], s);
}

// ---------------------------------------------------------------------------------------------------------
// Weights, step 1: one wave per (row, group).  Each lane owns pairs of neighbouring k so that it writes whole
// bytes of the canonical packing (even k in the low nibble).  BITS = 4: codes -8..7, s = absmax / 7, two codes per
// byte; BITS = 8 (the fine-grained W8A8 recipe): codes -128..127, s = absmax / 127, one code per byte, row-major.
// ---------------------------------------------------------------------------------------------------------
constexpr int kWqThreads = 256;

template <int BITS>
__global__ __launch_bounds__(kWqThreads) void quantize_weight_groups_kernel(const __half* __restrict__ w, int N, int K,
                                                                            int G, uint8_t* __restrict__ qweight,
                                                                            float* __restrict__ scale_f32) {
    constexpr float kHi = BITS == 4 ? 7.0f : 127.0f, kLo = -kHi - 1.0f;
    const int NG = K / G;
    const long long unit = (long long)blockIdx.x * (kWqThreads / kWave) + threadIdx.x / kWave;
    if (unit >= (long long)N * NG) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int n = (int)(unit / NG);
    const int g = (int)(unit % NG);
    const size_t base = (size_t)n * K + (size_t)g * G;
    const __half2* src = reinterpret_cast<const __half2*>(w + base);
    const int npairs = G >> 1;

    float amax = 0.0f;
    for (int p = lane; p < npairs; p += kWave) {
        float2 f = __half22float2(src[p]);
        amax = fmaxf(amax, fmaxf(fabsf(f.x), fabsf(f.y)));
    }
    amax = wave_max(amax);
    const float s = amax / kHi;
    if (lane == 0) scale_f32[unit] = s;

    uint8_t* dst = qweight + (BITS == 4 ? base >> 1 : base);
    for (int p = lane; p < npairs; p += kWave) {
        float2 f = __half22float2(src[p]);
        int q0 = 0, q1 = 0;
        if (s > 0.0f) {
            q0 = quant_code(f.x, s, kLo, kHi);
            q1 = quant_code(f.y, s, kLo, kHi);
        }
        if constexpr (BITS == 4) {
            dst[p] = (uint8_t)(((uint32_t)q0 & 0xFu) | (((uint32_t)q1 & 0xFu) << 4));
        } else {
            reinterpret_cast<uint16_t*>(dst)[p] = (uint16_t)(((uint32_t)q0 & 0xFFu) | (((uint32_t)q1 & 0xFFu) << 8));
        }
    }
}

__device__ __forceinline__ float amplified_value(float s, float c, int scale_mode) {
    if (scale_mode == IS_SCALE_NORM) return c > 0.0f ? s / c : 0.0f;
    return s;
}

__device__ __forceinline__ int amplifier_log2_for(float smin) {
    // smallest i >= 0 with smin * 2^i >= 1, capped (Sec. 4.1)
    int i = 0;
    while (i < IS_ALPHA_LOG2_MAX && ldexpf(smin, i) < 1.0f) ++i;
    return i;
}

// Weights, step 2: one wave per row.  Channel scale c[n], then either the integer scales (fixed amplifier) or this
// row's contribution to the amplifier search (the amplifier for the smallest scale is the largest one needed).
__global__ __launch_bounds__(kWqThreads) void derive_int_scales_kernel(const float* __restrict__ scale_f32, int N,
                                                                       int NG, int alpha_log2, int scale_mode,
                                                                       int32_t* __restrict__ scale_i32,
                                                                       float* __restrict__ chan_scale,
                                                                       int* __restrict__ alpha_log2_dev) {
    const int n = blockIdx.x * (kWqThreads / kWave) + threadIdx.x / kWave;
    if (n >= N) return;
    const int lane = threadIdx.x & (kWave - 1);
    const float* srow = scale_f32 + (size_t)n * NG;

    float c = 1.0f;
    if (scale_mode == IS_SCALE_NORM) {
        c = 0.0f;
        for (int g = lane; g < NG; g += kWave) c = fmaxf(c, srow[g]);
        c = wave_max(c);
    }
    if (lane == 0) chan_scale[n] = c;

    if (alpha_log2 >= 0) {
        for (int g = lane; g < NG; g += kWave)
            scale_i32[(size_t)n * NG + g] = (int32_t)rintf(ldexpf(amplified_value(srow[g], c, scale_mode), alpha_log2));
        if (n == 0 && lane == 0 && alpha_log2_dev) *alpha_log2_dev = alpha_log2;
    } else {
        float vmin = INFINITY;
        for (int g = lane; g < NG; g += kWave) {
            float v = amplified_value(srow[g], c, scale_mode);
            if (v > 0.0f) vmin = fminf(vmin, v);
        }
        vmin = wave_min(vmin);
        if (lane == 0 && vmin < INFINITY) atomicMax(alpha_log2_dev, amplifier_log2_for(vmin));
    }
}

__global__ void set_int_kernel(int* p, int v) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = v;
}

// Weights, step 3 (amplifier search only): integer scales with the amplifier found in step 2.
__global__ __launch_bounds__(kWqThreads) void apply_searched_amplifier_kernel(const float* __restrict__ scale_f32,
                                                                              const float* __restrict__ chan_scale,
                                                                              int N, int NG, int scale_mode,
                                                                              const int* __restrict__ alpha_log2_dev,
                                                                              int32_t* __restrict__ scale_i32) {
    const long long i = (long long)blockIdx.x * kWqThreads + threadIdx.x;
    if (i >= (long long)N * NG) return;
    const int a = *alpha_log2_dev;
    const float c = chan_scale[i / NG];
    scale_i32[i] = (int32_t)rintf(ldexpf(amplified_value(scale_f32[i], c, scale_mode), a));
}

}  // namespace

hipError_t launch_quantize_act(const __half* x, int M, int K, int8_t* xq, float* a_scale, hipStream_t stream) {
    const int nchunk = K >> 3;
    const dim3 grid(M);
#define ACT_LAUNCH(CH, T) \
    hipLaunchKernelGGL((quantize_act_resident_kernel<CH, T>), grid, dim3(T), 0, stream, x, M, K, xq, a_scale)
    if (M <= 256 && nchunk > kActThreads && nchunk <= 4096) {  // few rows: one chunk per lane where 1024 lanes reach
        if (nchunk <= 512) ACT_LAUNCH(1, 512);
        else if (nchunk <= 1024) ACT_LAUNCH(1, 1024);
        else if (nchunk <= 2048) ACT_LAUNCH(2, 1024);
        else ACT_LAUNCH(4, 1024);
        return hipGetLastError();
    }
    const int chunks_per_lane = (nchunk + kActThreads - 1) / kActThreads;
    if (chunks_per_lane <= 2) ACT_LAUNCH(2, kActThreads);
    else if (chunks_per_lane <= 8) ACT_LAUNCH(8, kActThreads);
    else if (chunks_per_lane <= 16) ACT_LAUNCH(16, kActThreads);
    else
        hipLaunchKernelGGL(quantize_act_kernel, grid, dim3(kActThreads), 0, stream, x, M, K, xq, a_scale);
#undef ACT_LAUNCH
    return hipGetLastError();
}

hipError_t launch_quantize_weights(const __half* w, int N, int K, int group, int alpha_log2, int scale_mode,
                                   uint8_t* qweight, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                   int* alpha_log2_dev, hipStream_t stream, int bits) {
    const int NG = K / group;
    const long long units = (long long)N * NG;
    const int waves_per_block = kWqThreads / kWave;
    const unsigned blocks1 = (unsigned)((units + waves_per_block - 1) / waves_per_block);
    if (bits == 4)
        hipLaunchKernelGGL(quantize_weight_groups_kernel<4>, dim3(blocks1), dim3(kWqThreads), 0, stream, w, N, K, group,
                           qweight, scale_f32);
    else
        hipLaunchKernelGGL(quantize_weight_groups_kernel<8>, dim3(blocks1), dim3(kWqThreads), 0, stream, w, N, K, group,
                           qweight, scale_f32);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (alpha_log2 < 0) {
        hipLaunchKernelGGL(set_int_kernel, dim3(1), dim3(kWave), 0, stream, alpha_log2_dev, 0);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const unsigned blocks2 = (unsigned)((N + waves_per_block - 1) / waves_per_block);
    hipLaunchKernelGGL(derive_int_scales_kernel, dim3(blocks2), dim3(kWqThreads), 0, stream, scale_f32, N, NG,
                       alpha_log2, scale_mode, scale_i32, chan_scale, alpha_log2_dev);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (alpha_log2 < 0) {
        const unsigned blocks3 = (unsigned)((units + kWqThreads - 1) / kWqThreads);
        hipLaunchKernelGGL(apply_searched_amplifier_kernel, dim3(blocks3), dim3(kWqThreads), 0, stream, scale_f32,
                           chan_scale, N, NG, scale_mode, alpha_log2_dev, scale_i32);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace intscale
