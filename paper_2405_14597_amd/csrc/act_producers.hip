// The activation quantiser folded into the operator that produces the activation (the "kernel fusion" of Sec. 4.3
// and Sec. 5.2): RMSNorm in front of the attention and MLP projections, SiLU(gate) * up in front of the
// down-projection.  Each result is defined as the unfused chain, producer -> fp16 tensor -> Appendix A.1 quantiser
// (n = 8, per token), so folding changes no code; what it saves is the fp16 tensor's round trip through memory
// (7 bytes per element become 3 for the norm, 9 become 5 for SiLU * up).
//
// The producer's fp16 value decides integer codes, so its arithmetic is a fixed sequence of separately rounded
// single-precision operations, with contraction into fused multiply-adds switched off:
//   RMSNorm     sum of squares in double (a squared fp16 value is exact), mean rounded once to single, then
//               r = 1 / sqrt(mean + eps) and y = fp16((x * r) * gamma)
//   SiLU * up   t = clamp(-g, -87, 88), n = rint(t * log2 e), r = (t - n * ln2_hi) - n * ln2_lo, the degree-6 Taylor
//               polynomial of e^r by Horner's rule, e = p * 2^n, h = fp16((g / (1 + e)) * u)
// One workgroup per token row; the row stays in registers between the reductions and the rounding.
#include "act_common.h"
#include "is_common.h"

namespace intscale {
namespace {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

template <int NW = kActThreads / kWave>
__device__ __forceinline__ double block_sum(double v, double* red) {
    v = wave_sum(v);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    v = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) v += red[i];
    return v;
}

__device__ __forceinline__ double sumsq8(uint4 v) {
    const __half2* h = reinterpret_cast<const __half2*>(&v);
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 f = __half22float2(h[i]);
        s += (double)(f.x * f.x);  // 22 significant bits: exact in single precision
        s += (double)(f.y * f.y);
    }
    return s;
}

__device__ __forceinline__ float rms_factor(double sumsq, int K, float eps) {
    const float mean = (float)(sumsq / (double)K);
    return 1.0f / sqrtf(mean + eps);
}

__device__ __forceinline__ uint4 normalize8(uint4 v, uint4 g, float r) {
    const __half2* hv = reinterpret_cast<const __half2*>(&v);
    const __half2* hg = reinterpret_cast<const __half2*>(&g);
    uint4 out;
    __half2* ho = reinterpret_cast<__half2*>(&out);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 f = __half22float2(hv[i]);
        float2 w = __half22float2(hg[i]);
        ho[i] = __floats2half2_rn(rounded_f32((f.x * r) * w.x), rounded_f32((f.y * r) * w.y));
    }
    return out;
}

__device__ __forceinline__ uint4 silu_mul8(uint4 g, uint4 u) {
    const __half2* hg = reinterpret_cast<const __half2*>(&g);
    const __half2* hu = reinterpret_cast<const __half2*>(&u);
    uint4 out;
    __half2* ho = reinterpret_cast<__half2*>(&out);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 a = __half22float2(hg[i]);
        float2 b = __half22float2(hu[i]);
        ho[i] = __floats2half2_rn(silu_mul(a.x, b.x), silu_mul(a.y, b.y));
    }
    return out;
}

// ---------------------------------------------------------------------------------------------------------
// RMSNorm + quantiser.  Rows of up to 2048 * CH elements stay in registers (CH 16-byte chunks per lane): read
// once, normalised in place, written once as codes.  Few rows (a decode step) take 1024 lanes per row instead of 256:
// the chip is far from full then, and a row's arithmetic is spread over four times as many lanes.
// ---------------------------------------------------------------------------------------------------------
template <int CH, int THREADS>
__global__ __launch_bounds__(THREADS) void rmsnorm_quantize_resident_kernel(const __half* __restrict__ x,
                                                                                const __half* __restrict__ gamma,
                                                                                float eps, int M, int K,
                                                                                int8_t* __restrict__ xq,
                                                                                float* __restrict__ a_scale) {
    __shared__ float red[THREADS / kWave];
    __shared__ double dred[THREADS / kWave];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const int nchunk = K >> 3;
    const uint4* row = reinterpret_cast<const uint4*>(x + (size_t)m * K);
    const uint4* grow = reinterpret_cast<const uint4*>(gamma);
    uint4 v[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int idx = tid + c * THREADS;
        v[c] = idx < nchunk ? row[idx] : make_uint4(0u, 0u, 0u, 0u);
    }
    double ss = 0.0;
#pragma unroll
    for (int c = 0; c < CH; ++c) ss += sumsq8(v[c]);
    const float r = rms_factor(block_sum<THREADS / kWave>(ss, dred), K, eps);
    float amax = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int idx = tid + c * THREADS;
        if (idx < nchunk) {
            v[c] = normalize8(v[c], grow[idx], r);
            amax = fmaxf(amax, absmax8(v[c]));
        }
    }
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

// Longer rows: three passes over the row (the later ones come back from L2), the normalised value recomputed.
__global__ __launch_bounds__(kActThreads) void rmsnorm_quantize_kernel(const __half* __restrict__ x,
                                                                       const __half* __restrict__ gamma, float eps,
                                                                       int M, int K, int8_t* __restrict__ xq,
                                                                       float* __restrict__ a_scale) {
    __shared__ float red[kActThreads / kWave];
    __shared__ double dred[kActThreads / kWave];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const int nchunk = K >> 3;
    const uint4* row = reinterpret_cast<const uint4*>(x + (size_t)m * K);
    const uint4* grow = reinterpret_cast<const uint4*>(gamma);
    double ss = 0.0;
    for (int c = tid; c < nchunk; c += kActThreads) ss += sumsq8(row[c]);
    const float r = rms_factor(block_sum(ss, dred), K, eps);
    float amax = 0.0f;
    for (int c = tid; c < nchunk; c += kActThreads) amax = fmaxf(amax, absmax8(normalize8(row[c], grow[c], r)));
    amax = block_max(amax, red);
    const float s = amax / 127.0f;
    if (tid == 0) a_scale[m] = s;
    uint2* dst = reinterpret_cast<uint2*>(xq + (size_t)m * K);
    for (int c = tid; c < nchunk; c += kActThreads) dst[c] = quantize8(normalize8(row[c], grow[c], r), s);
}

// ---------------------------------------------------------------------------------------------------------
// SiLU(gate) * up + quantiser.  gate_up holds the gate half then the up half of each token row (the layout a
// fused gate/up projection writes); a row of `inter` products stays in registers as fp16.
// ---------------------------------------------------------------------------------------------------------
template <int CH, int THREADS>
__global__ __launch_bounds__(THREADS) void silu_mul_quantize_resident_kernel(const __half* __restrict__ gate_up,
                                                                                 int M, int inter,
                                                                                 int8_t* __restrict__ xq,
                                                                                 float* __restrict__ a_scale) {
    __shared__ float red[THREADS / kWave];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const int nchunk = inter >> 3;
    const uint4* grow = reinterpret_cast<const uint4*>(gate_up + (size_t)m * 2 * inter);
    const uint4* urow = grow + nchunk;
    uint4 v[CH];
    float amax = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int idx = tid + c * THREADS;
        v[c] = make_uint4(0u, 0u, 0u, 0u);
        if (idx < nchunk) {
            v[c] = silu_mul8(grow[idx], urow[idx]);
            amax = fmaxf(amax, absmax8(v[c]));
        }
    }
    amax = block_max<THREADS / kWave>(amax, red);
    const float s = amax / 127.0f;
    if (tid == 0) a_scale[m] = s;
    uint2* dst = reinterpret_cast<uint2*>(xq + (size_t)m * inter);
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int idx = tid + c * THREADS;
        if (idx < nchunk) dst[idx] = quantize8(v[c], s);
    }
}

// Longer rows: the product is computed twice, the second time from L2.
__global__ __launch_bounds__(kActThreads) void silu_mul_quantize_kernel(const __half* __restrict__ gate_up, int M,
                                                                        int inter, int8_t* __restrict__ xq,
                                                                        float* __restrict__ a_scale) {
    __shared__ float red[kActThreads / kWave];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const int nchunk = inter >> 3;
    const uint4* grow = reinterpret_cast<const uint4*>(gate_up + (size_t)m * 2 * inter);
    const uint4* urow = grow + nchunk;
    float amax = 0.0f;
    for (int c = tid; c < nchunk; c += kActThreads) amax = fmaxf(amax, absmax8(silu_mul8(grow[c], urow[c])));
    amax = block_max(amax, red);
    const float s = amax / 127.0f;
    if (tid == 0) a_scale[m] = s;
    uint2* dst = reinterpret_cast<uint2*>(xq + (size_t)m * inter);
    for (int c = tid; c < nchunk; c += kActThreads) dst[c] = quantize8(silu_mul8(grow[c], urow[c]), s);
}

}  // namespace

// Few rows: 1024 lanes per row (the chip is not full anyway and the row's latency is what counts).
constexpr int kFewRows = 256;
constexpr int kWideThreads = 1024;

hipError_t launch_rmsnorm_quantize_act(const __half* x, const __half* gamma, float eps, int M, int K, int8_t* xq,
                                       float* a_scale, hipStream_t stream) {
    const int nchunk = K >> 3;
    const dim3 grid(M);
#define RMS_LAUNCH(CH, T) \
    hipLaunchKernelGGL((rmsnorm_quantize_resident_kernel<CH, T>), grid, dim3(T), 0, stream, x, gamma, eps, M, K, xq, a_scale)
    if (M <= kFewRows && nchunk > kActThreads && nchunk <= 4 * kWideThreads) {
        const int cpl = (nchunk + kWideThreads - 1) / kWideThreads;
        if (cpl <= 1) RMS_LAUNCH(1, kWideThreads);
        else if (cpl <= 2) RMS_LAUNCH(2, kWideThreads);
        else RMS_LAUNCH(4, kWideThreads);
        return hipGetLastError();
    }
    const int cpl = (nchunk + kActThreads - 1) / kActThreads;
    if (cpl <= 2) RMS_LAUNCH(2, kActThreads);
    else if (cpl <= 8) RMS_LAUNCH(8, kActThreads);
    else if (cpl <= 16) RMS_LAUNCH(16, kActThreads);
    else
        hipLaunchKernelGGL(rmsnorm_quantize_kernel, grid, dim3(kActThreads), 0, stream, x, gamma, eps, M, K, xq, a_scale);
#undef RMS_LAUNCH
    return hipGetLastError();
}

hipError_t launch_silu_mul_quantize_act(const __half* gate_up, int M, int inter, int8_t* xq, float* a_scale,
                                        hipStream_t stream) {
    const int nchunk = inter >> 3;
    const dim3 grid(M);
#define SILU_LAUNCH(CH, T) \
    hipLaunchKernelGGL((silu_mul_quantize_resident_kernel<CH, T>), grid, dim3(T), 0, stream, gate_up, M, inter, xq, a_scale)
    if (M <= kFewRows && nchunk > kActThreads && nchunk <= 4 * kWideThreads) {
        const int cpl = (nchunk + kWideThreads - 1) / kWideThreads;
        if (cpl <= 1) SILU_LAUNCH(1, kWideThreads);
        else if (cpl <= 2) SILU_LAUNCH(2, kWideThreads);
        else SILU_LAUNCH(4, kWideThreads);
        return hipGetLastError();
    }
    const int cpl = (nchunk + kActThreads - 1) / kActThreads;
    if (cpl <= 2) SILU_LAUNCH(2, kActThreads);
    else if (cpl <= 8) SILU_LAUNCH(8, kActThreads);
    else if (cpl <= 16) SILU_LAUNCH(16, kActThreads);
    else
        hipLaunchKernelGGL(silu_mul_quantize_kernel, grid, dim3(kActThreads), 0, stream, gate_up, M, inter, xq, a_scale);
#undef SILU_LAUNCH
    return hipGetLastError();
}

// The fp16 output of a GEMM whose weight rows alternate gate / up by 16-row tile (is_prepack_w4_gate_up), [M, N]:
// out[m, 16 p + r] = fp16(SiLU(gu[m, 32 p + r]) * gu[m, 32 p + 16 + r]), [M, N / 2].  One thread per 8 outputs.
namespace {
__global__ __launch_bounds__(256) void silu_mul_paired_kernel(const __half* __restrict__ gu, int M, int N,
                                                              __half* __restrict__ out) {
    const int inter = N >> 1, chunks = inter >> 3;
    const size_t at = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (at >= (size_t)M * chunks) return;
    const int m = (int)(at / chunks), c = (int)(at - (size_t)m * chunks);  // outputs 8 c .. 8 c + 7 of row m
    const int p = c >> 1, h = c & 1;
    const __half* row = gu + (size_t)m * N + 32 * p + 8 * h;
    const uint4 g = *reinterpret_cast<const uint4*>(row), u = *reinterpret_cast<const uint4*>(row + 16);
    *reinterpret_cast<uint4*>(out + (size_t)m * inter + 8 * c) = silu_mul8(g, u);
}
}  // namespace

hipError_t launch_silu_mul_paired(const __half* gu, int M, int N, __half* out, hipStream_t stream) {
    const size_t work = (size_t)M * (N >> 4);
    hipLaunchKernelGGL(silu_mul_paired_kernel, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, stream, gu, M, N, out);
    return hipGetLastError();
}

}  // namespace intscale
