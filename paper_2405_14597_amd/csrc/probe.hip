// Measurement aids, not part of the method: what this chip actually delivers for the two rooflines the GEMMs are
// priced against -- a plain streaming read out of HBM, and a loop of independent int8 MFMAs on registers.
#include "is_common.h"

namespace intscale {
namespace {

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t chunks, int* __restrict__ sink) {
    uint32_t x = 0;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < chunks; i += stride) {
        const uint4 v = src[i];
        x ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (x == 0x9E3779B9u) *sink = (int)x;  // keeps the loads alive; practically never true
}

constexpr int kMfmaPerIter = 16;

__global__ __launch_bounds__(512) void mfma_i8_kernel(int iters, int* __restrict__ sink) {
    v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {4, 5, 6, (int)blockIdx.x};
    v4i acc[kMfmaPerIter];
#pragma unroll
    for (int i = 0; i < kMfmaPerIter; ++i) acc[i] = v4i{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kMfmaPerIter; ++i) acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[i], 0, 0, 0);
    }
    v4i s = acc[0];
#pragma unroll
    for (int i = 1; i < kMfmaPerIter; ++i) s += acc[i];
    if ((s[0] ^ s[1] ^ s[2] ^ s[3]) == 0x5bd1e995) *sink = s[0];
}

// The same loop on operands that change from one MFMA to the next (eight register sets of pseudo-random bytes, used in
// turn): the rate the matrix pipe holds when its inputs toggle, as a GEMM's do.  The chip lowers its clock under that
// load, so this rate, not the one of the loop above, is what a real contraction can reach.
__global__ __launch_bounds__(512) void mfma_i8_random_kernel(int iters, int* __restrict__ sink) {
    v4i a[8], b[8];
    uint32_t h = (uint32_t)(blockIdx.x * 512 + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            h = h * 1664525u + 1013904223u;
            a[i][q] = (int)(h ^ (h >> 15));
            h = h * 1664525u + 1013904223u;
            b[i][q] = (int)((h ^ (h >> 13)) & 0x0F0F0F0Fu);  // weight codes of four bits, as after the unpacking
        }
    v4i acc[kMfmaPerIter];
#pragma unroll
    for (int i = 0; i < kMfmaPerIter; ++i) acc[i] = v4i{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kMfmaPerIter; ++i)
            acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i & 7], b[(i + (i >> 3)) & 7], acc[i], 0, 0, 0);
    }
    v4i s = acc[0];
#pragma unroll
    for (int i = 1; i < kMfmaPerIter; ++i) s += acc[i];
    if ((s[0] ^ s[1] ^ s[2] ^ s[3]) == 0x5bd1e995) *sink = s[0];
}

}  // namespace

int g_cu_count = 0;

int cu_count() {
    if (g_cu_count == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            g_cu_count = n;
        else
            g_cu_count = 256;
    }
    return g_cu_count;
}

hipError_t launch_probe_stream_read(const void* src, size_t bytes, int* sink, hipStream_t stream) {
    const size_t chunks = bytes / 16;
    hipLaunchKernelGGL(stream_read_kernel, dim3(cu_count() * 8), dim3(256), 0, stream, static_cast<const uint4*>(src),
                       chunks, sink);
    return hipGetLastError();
}

hipError_t launch_probe_mfma_i8(int iters, int* sink, double* ops, hipStream_t stream, bool random_operands) {
    const int blocks = cu_count() * 4;  // 512 threads each: 2 waves per SIMD, 4 rounds
    if (random_operands) hipLaunchKernelGGL(mfma_i8_random_kernel, dim3(blocks), dim3(512), 0, stream, iters, sink);
    else hipLaunchKernelGGL(mfma_i8_kernel, dim3(blocks), dim3(512), 0, stream, iters, sink);
    if (ops) *ops = 2.0 * 16 * 16 * 64 * kMfmaPerIter * (double)iters * 8.0 * blocks;
    return hipGetLastError();
}

}  // namespace intscale
