// Offline conversion of a quantised weight matrix from the canonical layouts to the kernel layout described in
// pk_common.h (Sec. 4.2: the amplified scales are converted offline, and the weights go through an "efficient weight
// processing" the paper does not detail).  Same byte count as the canonical tensors up to padding of N to 16.
#include "pk_common.h"

namespace intscale {
namespace {

// Row n of the packed matrix is row source_row(n) of the canonical one.  pair_inter = 0: the same row.  Otherwise the
// canonical matrix is a fused gate/up projection, rows [0, pair_inter) the gate's and [pair_inter, 2 pair_inter) the
// up's, and the packed rows alternate by 16-row tile: tile 2p holds gate rows 16p..16p+15, tile 2p+1 the up rows of
// the same outputs, so that a kernel lane that owns output n of the gate also owns output n of the up projection.
__device__ __forceinline__ int source_row(int n, int pair_inter) {
    if (pair_inter == 0) return n;
    const int t = n >> 4;
    return ((t & 1) ? pair_inter : 0) + ((t >> 1) << 4) + (n & 15);
}

// One thread per 16-byte chunk of the packed weights.
__global__ __launch_bounds__(256) void prepack_weights_kernel(const uint8_t* __restrict__ qw, int N, int K,
                                                              uint4* __restrict__ wpack, int32_t* __restrict__ header,
                                                              int group, int flags, int pair_inter) {
    if (blockIdx.x == 0 && threadIdx.x < 64) {
        int v = 0;
        if (threadIdx.x == 0) v = flags;
        if (threadIdx.x == 1) v = N;
        if (threadIdx.x == 2) v = K;
        if (threadIdx.x == 3) v = group;
        if (threadIdx.x == 4) v = pair_inter;
        header[threadIdx.x] = v;
    }
    const int steps = K >> 7;
    const size_t total = (size_t)((N + 15) / 16) * steps * 64;
    const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= total) return;
    const int lane = (int)(c & 63);
    const size_t blk = c >> 6;
    const int s = (int)(blk % steps);
    const int t = (int)(blk / steps);
    const int kb = lane >> 4, r = lane & 15;
    const int n = 16 * t + r;
    uint4 o = make_uint4(0u, 0u, 0u, 0u);
    if (n < N) {
        const uint8_t* row = qw + (size_t)source_row(n, pair_inter) * (K >> 1);
        // 16 codes k0..k0+15 are 8 canonical bytes (even k in the low nibble)
        const uint2 lo = *reinterpret_cast<const uint2*>(row + ((128 * s + 16 * kb) >> 1));
        const uint2 hi = *reinterpret_cast<const uint2*>(row + ((128 * s + 64 + 16 * kb) >> 1));
        const uint32_t lw[2] = {lo.x, lo.y}, hw[2] = {hi.x, hi.y};
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const uint32_t a = (lw[j >> 3] >> (4 * (j & 7))) & 0xFu;
            const uint32_t b = (hw[j >> 3] >> (4 * (j & 7))) & 0xFu;
            w[j >> 2] |= (a | (b << 4)) << (8 * (j & 3));
        }
        o = make_uint4(w[0], w[1], w[2], w[3]);
    }
    wpack[c] = o;
}

// One thread per packed scale word; integer scales also raise the "wider than 24 bits" flag.
template <bool CHECK>
__global__ __launch_bounds__(256) void prepack_scales_kernel(const int32_t* __restrict__ scale, int N, int NG,
                                                             int32_t* __restrict__ spack, int32_t* __restrict__ header,
                                                             int pair_inter) {
    const size_t total = (size_t)((N + 15) / 16) * NG * 16;
    const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
    bool wide = false;
    if (c < total) {
        const int r = (int)(c & 15);
        const size_t tg = c >> 4;
        const int g = (int)(tg % NG);
        const int n = 16 * (int)(tg / NG) + r;
        const int32_t v = n < N ? scale[(size_t)source_row(n, pair_inter) * NG + g] : 0;
        spack[c] = v;
        if (CHECK) wide = ((uint32_t)(v + (1 << 23)) >> 24) != 0;
    }
    if (CHECK && __any(wide) && (threadIdx.x & (kWave - 1)) == 0) atomicOr(header, kPkFlagWide);
}

__global__ __launch_bounds__(256) void pair_channel_scales_kernel(const float* __restrict__ c, int N, int pair_inter,
                                                                  float* __restrict__ out) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n < N) out[n] = c[source_row(n, pair_inter)];
}

}  // namespace

hipError_t launch_prepack_w4(const uint8_t* qweight, const void* scale, bool float_scales, int N, int K, int group,
                             uint8_t* wpack, uint8_t* spack, hipStream_t stream, int pair_inter, const float* chan_scale,
                             float* chan_scale_packed) {
    if (chan_scale != nullptr)
        hipLaunchKernelGGL(pair_channel_scales_kernel, dim3((N + 255) / 256), dim3(256), 0, stream, chan_scale, N, pair_inter,
                           chan_scale_packed);
    const int NG = K / group;
    const size_t chunks = (size_t)((N + 15) / 16) * (K >> 7) * 64;
    int32_t* header = reinterpret_cast<int32_t*>(spack);
    hipLaunchKernelGGL(prepack_weights_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, stream, qweight, N, K,
                       reinterpret_cast<uint4*>(wpack), header, group,
                       (float_scales ? kPkFlagFloat : 0) | (pair_inter ? kPkFlagPaired : 0), pair_inter);
    const size_t words = (size_t)((N + 15) / 16) * NG * 16;
    int32_t* body = reinterpret_cast<int32_t*>(spack + kPkHeaderBytes);
    const dim3 grid((unsigned)((words + 255) / 256));
    if (float_scales)
        hipLaunchKernelGGL(prepack_scales_kernel<false>, grid, dim3(256), 0, stream, static_cast<const int32_t*>(scale), N,
                           NG, body, header, pair_inter);
    else
        hipLaunchKernelGGL(prepack_scales_kernel<true>, grid, dim3(256), 0, stream, static_cast<const int32_t*>(scale), N,
                           NG, body, header, pair_inter);
    return hipGetLastError();
}

}  // namespace intscale
