// Pieces shared by the MFMA-bound tiled kernels (int4 and int8 weights): buffer descriptors, the buffer-to-LDS load,
// the scale transposition, the row-tile slots of the grouped form.
#ifndef INTSCALE_TILE_COMMON_H_
#define INTSCALE_TILE_COMMON_H_

#include "is_common.h"

namespace intscale {
namespace {

constexpr int kTileRows = 128;  // token rows of a tile (both tiled kernels)

typedef float v4f __attribute__((ext_vector_type(4)));

// Buffer descriptor in four scalar registers: base address, no stride, byte count, raw 32-bit format.  Offsets at or
// past the byte count read as zero.
__device__ __forceinline__ v4i make_desc(const void* base, size_t bytes) {
    const uint64_t p = reinterpret_cast<uint64_t>(base);
    v4i d;
    d[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    d[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((p >> 32) & 0xFFFFu));
    d[2] = __builtin_amdgcn_readfirstlane((int)(bytes > 0x7FFFFFFFull ? 0x7FFFFFFFu : (uint32_t)bytes));
    d[3] = 0x00020000;
    return d;
}

// 64 lanes x 16 bytes from global memory to LDS at lds_base + lds_offset + lane * 16.  Completion is visible through
// the vector memory counter only.
__device__ __forceinline__ void load_to_lds_b128(v4i desc, unsigned lds_base, unsigned lds_offset, int voffset,
                                                 int soffset) {
    asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, %4 offen lds"
                 :
                 : "s"(lds_base), "s"(lds_offset), "v"(voffset), "s"(desc), "s"(soffset)
                 : "memory", "scc");
}
// Preparation of the scales: st[e][g][n] = scale[e][n][g] (32-bit words, integer or float alike), through a 64 x 64
// LDS tile so that both sides are coalesced; CHECK also raises the flag if an integer scale does not fit 24 signed
// bits (the limit of v_mad_i32_i24).
template <bool CHECK>
__global__ __launch_bounds__(256) void prepare_scales_kernel(const int32_t* __restrict__ scale, int N, int NG,
                                                             int32_t* __restrict__ st, int32_t* __restrict__ wide_flag) {
    __shared__ int32_t tile[64][65];
    const size_t e = blockIdx.z;
    const int n0 = blockIdx.x * 64, g0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    bool wide = false;
#pragma unroll
    for (int q = 0; q < 16; ++q) {  // unrolled: the 16 loads of a thread are in flight together
        const int r = ty + 4 * q;
        const int n = n0 + r, g = g0 + tx;
        int32_t v = 0;
        if (n < N && g < NG) v = scale[(e * N + n) * NG + g];
        if (CHECK) wide |= ((uint32_t)(v + (1 << 23)) >> 24) != 0;
        tile[r][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int r = ty + 4 * q;
        const int g = g0 + r, n = n0 + tx;
        if (g < NG && n < N) st[(e * NG + g) * N + n] = tile[tx][r];
    }
    if (CHECK && __any(wide) && (threadIdx.x & (kWave - 1)) == 0) atomicOr(wide_flag, 1);
}

// Row-tile slots of the grouped form (see prepare_activations_kernel).
__host__ __device__ inline int tile_slots(int M, int num_experts) { return (M + kTileRows - 1) / kTileRows + num_experts; }

inline size_t pad256(size_t bytes) { return (bytes + 255) & ~(size_t)255; }

}  // namespace
}  // namespace intscale
#endif
