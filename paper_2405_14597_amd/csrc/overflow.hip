// Overflow handling around the integer-scale GEMM (the paper's Sec. 5.6, Appendix on maximum activations, and the
// Limitations section): the worst-case accumulator of a layer, and the scales of the overflow-safe ("degraded") form
// in which the amplifier is taken out group by group.
#include "is_common.h"

namespace intscale {
namespace {

constexpr int kThreads = 256;

__global__ void clear_bound_kernel(unsigned long long* bound) { *bound = 0; }

// One wave per weight row: sum_g |IS[n,g]| * group * 128 * 8, the largest |accumulator| any int8 activations and int4
// weights can produce for that row (a group's partial sum is at most group * 128 * 8 in magnitude); the layer's bound
// is the maximum over rows.
__global__ __launch_bounds__(kThreads) void overflow_bound_kernel(const int32_t* __restrict__ scale_i32, int N, int NG,
                                                                  int group, unsigned long long* __restrict__ bound) {
    const int n = blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    if (n >= N) return;
    const int lane = threadIdx.x & (kWave - 1);
    unsigned long long sum = 0;
    for (int g = lane; g < NG; g += kWave) {
        const long long v = scale_i32[(size_t)n * NG + g];
        sum += (unsigned long long)(v < 0 ? -v : v);
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
    if (lane == 0) atomicMax(bound, sum * (unsigned long long)group * 1024ull);
}

// Scales of the overflow-safe form: float(IS[n,g]) * c[n] * 2^-alpha_log2 (the conversion is exact below 2^24, the
// power of two always, so at most the product with c[n] rounds).
__global__ __launch_bounds__(kThreads) void derive_safe_scales_kernel(const int32_t* __restrict__ scale_i32,
                                                                      const float* __restrict__ chan_scale, size_t count,
                                                                      int NG, int alpha_log2, float* __restrict__ out) {
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= count) return;
    const float c = chan_scale ? chan_scale[i / NG] : 1.0f;
    out[i] = ldexpf((float)scale_i32[i] * c, -alpha_log2);
}

}  // namespace

hipError_t launch_overflow_bound(const int32_t* scale_i32, int N, int NG, int group, unsigned long long* bound_dev,
                                 hipStream_t stream) {
    hipLaunchKernelGGL(clear_bound_kernel, dim3(1), dim3(1), 0, stream, bound_dev);
    const int waves_per_block = kThreads / kWave;
    hipLaunchKernelGGL(overflow_bound_kernel, dim3((N + waves_per_block - 1) / waves_per_block), dim3(kThreads), 0, stream,
                       scale_i32, N, NG, group, bound_dev);
    return hipGetLastError();
}

hipError_t launch_derive_safe_scales(const int32_t* scale_i32, const float* chan_scale, size_t rows, int NG,
                                     int alpha_log2, float* out, hipStream_t stream) {
    const size_t count = rows * (size_t)NG;
    hipLaunchKernelGGL(derive_safe_scales_kernel, dim3((unsigned)((count + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       stream, scale_i32, chan_scale, count, NG, alpha_log2, out);
    return hipGetLastError();
}

}  // namespace intscale
