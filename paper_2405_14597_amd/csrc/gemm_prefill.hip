// MFMA-bound regime (many token rows: prefill, and the per-expert slices of a mixture-of-experts layer) of the
// fine-grained W4A8 GEMM.  Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper; float-scale
// form: Eq. (1) / Table 2 "Atom".  The two differ only in the per-group scale step, which is where the paper's
// saving lives: one v_mad_i32_i24 per partial product against a convert plus a multiply-add.
//
// Tiling.  A workgroup of 4 waves (2 x 2) owns BM = 64*WMS token rows x 256 weight rows; a wave owns 32*WMS x 128,
// as WMS x 4 sub-tiles of v_mfma_i32_32x32x32_i8 (operand A = 32 token rows, operand B = 32 weight rows, so a lane's
// 16 results share one weight row and with it one group scale).  K advances in steps of 128 through double-buffered
// LDS tiles; the global loads of step s+1 are in flight while step s is multiplied.
//
// int4 -> int8 with a zero point instead of a sign extension: the loader stores q + 8 (nibble ^ 8), so a byte is
// unpacked with one AND (even k) or a shift and an AND (odd k), and the product sum comes out as
// P + 8 * sum_k x[m,k].  The correction -8 * sum_k x[m,k] per (token row, K step) is computed once by a small kernel
// into the workspace and enters each MFMA chain as its initial accumulator, so the chain returns P exactly and the
// scale step costs one instruction per element.
//
// LDS layouts.  Activations: row-major 128 B per row and step, 16-byte chunks XOR-swizzled by the row so that the
// 16-byte operand reads of 32 rows spread over all banks; inside a 16-k chunk the bytes are stored as
// [even k of 0..7 | even k of 8..15 | odd k of 0..7 | odd k of 8..15], the order in which the unpacked weights come
// out (a dot product does not care about the order of its terms as long as both operands agree).  Weights: 64 B per
// row and step, 8-byte chunks swizzled the same way.
#include "is_common.h"

namespace intscale {
namespace {

constexpr int kStepK = 128;
constexpr int kOutOfRange = (int)0x80000000u;  // a buffer offset past every descriptor here: the load returns 0
constexpr int kBN = 256;
constexpr int kThreads = 256;

typedef float v16f __attribute__((ext_vector_type(16)));
using rsrc_t = __amdgpu_buffer_rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
    const unsigned n = bytes > 0x7FFFFFFFull ? 0x7FFFFFFFu : (unsigned)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}
__device__ __forceinline__ int pick_even(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u); }
__device__ __forceinline__ int pick_odd(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x07050301u); }

// s8[step][m] = -8 * sum over the 128 k of the step of xq[m,k]: the zero-point correction of the q+8 weight bytes.
// One wave per token row; 8 lanes share a step.
__global__ __launch_bounds__(256) void step_sums_kernel(const int8_t* __restrict__ xq, int M, int K,
                                                        int32_t* __restrict__ s8) {
    const int m = blockIdx.x * 4 + threadIdx.x / kWave;
    if (m >= M) return;
    const int lane = threadIdx.x & (kWave - 1);
    const uint4* row = reinterpret_cast<const uint4*>(xq + (size_t)m * K);
    const int nchunk = K >> 4;
    for (int c0 = 0; c0 < nchunk; c0 += kWave) {
        const int c = c0 + lane;
        int sum = 0;
        if (c < nchunk) {
            const uint4 v = row[c];
            sum = __builtin_amdgcn_sdot4((int)v.x, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)v.y, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)v.z, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)v.w, 0x01010101, sum, false);
        }
        sum += __shfl_xor(sum, 1, kWave);
        sum += __shfl_xor(sum, 2, kWave);
        sum += __shfl_xor(sum, 4, kWave);
        if ((lane & 7) == 0 && c < nchunk) s8[(size_t)(c >> 3) * M + m] = -8 * sum;
    }
}

template <int WMS, bool INT_SCALE>
__global__ __launch_bounds__(kThreads) void gemm_prefill_kernel(GemmArgs a, const int32_t* __restrict__ s8) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int BM = 64 * WMS;
    constexpr int XL = BM * 8 / kThreads;   // 16-byte activation chunks per thread and step
    constexpr int WL = kBN * 4 / kThreads;  // 16-byte weight chunks per thread and step
    constexpr int X_BYTES = BM * 128, W_BYTES = kBN * 64;
    unsigned char* lds_x = smem;                       // [2][BM][128]
    unsigned char* lds_w = smem + 2 * X_BYTES;         // [2][256][64]
    int* lds_sc = reinterpret_cast<int*>(smem + 2 * X_BYTES + 2 * W_BYTES);  // [2][256]
    int* lds_s8 = lds_sc + 2 * kBN;                    // [2][BM]

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    int m_begin = 0, m_end = a.M;
    size_t expert = 0;
    if (a.row_offsets) {
        expert = blockIdx.z;
        m_begin = a.row_offsets[expert];
        m_end = a.row_offsets[expert + 1];
    }
    const int m0 = m_begin + blockIdx.y * BM;
    if (m0 >= m_end) return;  // uniform over the workgroup, before any barrier
    const int m_rows = min(BM, m_end - m0);
    const int n0 = blockIdx.x * kBN;
    const int n_rows = min(kBN, a.N - n0);

    const int NG = a.K / a.group;
    const int spg = a.group / kStepK;
    const int steps = a.K / kStepK;
    const int row_bytes = a.K >> 1;

    const rsrc_t xres = make_rsrc(a.xq + (size_t)m0 * a.K, (size_t)m_rows * a.K);
    const rsrc_t wres = make_rsrc(a.qweight + (expert * (size_t)a.N + n0) * row_bytes, (size_t)n_rows * row_bytes);
    const rsrc_t sres = make_rsrc(reinterpret_cast<const int*>(a.scale) + (expert * (size_t)a.N + n0) * NG,
                                  (size_t)n_rows * NG * 4);
    const rsrc_t zres = make_rsrc(s8, (size_t)steps * a.M * 4);

    // ---- loader roles
    int x_src[XL], x_dst[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        const int c = tid + i * kThreads, row = c >> 3, ch = c & 7;
        x_src[i] = row < m_rows ? row * a.K + ch * 16 : kOutOfRange;
        x_dst[i] = row * 128 + ((ch ^ ((row >> 1) & 7)) << 4);
    }
    int w_src[WL], w_dst[WL];
#pragma unroll
    for (int i = 0; i < WL; ++i) {
        const int c = tid + i * kThreads, row = c >> 2, ch = c & 3;
        w_src[i] = row < n_rows ? row * row_bytes + ch * 16 : kOutOfRange;
        w_dst[i] = row * 64 + (((2 * ch) ^ ((row >> 2) & 7)) << 3);  // second half: chunk index ^ 1
    }
    const int sc_src = tid < n_rows ? tid * NG * 4 : kOutOfRange;
    const int z_src = tid < m_rows ? tid * 4 : kOutOfRange;

    v4i rx[XL], rw[WL];
    int rsc, rz;
    int ld_group = 0, ld_sub = 0;  // group of the next step to load (steps are loaded in order)
    auto load_step = [&](int s) {
#pragma unroll
        for (int i = 0; i < XL; ++i) rx[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, x_src[i], s * kStepK, 0);
#pragma unroll
        for (int i = 0; i < WL; ++i) rw[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, w_src[i], s * (kStepK / 2), 0);
        rsc = __builtin_amdgcn_raw_buffer_load_b32(sres, sc_src, ld_group * 4, 0);
        rz = __builtin_amdgcn_raw_buffer_load_b32(zres, z_src, (s * a.M + m0) * 4, 0);
        if (++ld_sub == spg) {
            ld_sub = 0;
            ++ld_group;
        }
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            v4i p;
            p[0] = pick_even(rx[i][0], rx[i][1]);
            p[1] = pick_even(rx[i][2], rx[i][3]);
            p[2] = pick_odd(rx[i][0], rx[i][1]);
            p[3] = pick_odd(rx[i][2], rx[i][3]);
            *reinterpret_cast<v4i*>(lds_x + buf * X_BYTES + x_dst[i]) = p;
        }
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            // q -> q + 8: flip the top bit of every nibble
            const int2 lo = make_int2(rw[i][0] ^ (int)0x88888888u, rw[i][1] ^ (int)0x88888888u);
            const int2 hi = make_int2(rw[i][2] ^ (int)0x88888888u, rw[i][3] ^ (int)0x88888888u);
            *reinterpret_cast<int2*>(lds_w + buf * W_BYTES + w_dst[i]) = lo;
            *reinterpret_cast<int2*>(lds_w + buf * W_BYTES + (w_dst[i] ^ 8)) = hi;
        }
        lds_sc[buf * kBN + tid] = rsc;
        if (tid < BM) lds_s8[buf * BM + tid] = rz;
    };

    // ---- consumer roles: LDS offsets of this lane's operand reads
    const int a_row = (wm * WMS * 32 + l32) * 128;
    const int b_row = (wn * 128 + l32) * 64;
    int a_off[4], b_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        a_off[kk] = a_row + (((2 * kk + lh) ^ ((l32 >> 1) & 7)) << 4);
        b_off[kk] = b_row + (((2 * kk + lh) ^ ((l32 >> 2) & 7)) << 3);
    }

    using accv = typename std::conditional<INT_SCALE, v16i, v16f>::type;
    accv acc[WMS][4];
#pragma unroll
    for (int ms = 0; ms < WMS; ++ms)
#pragma unroll
        for (int ns = 0; ns < 4; ++ns)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ms][ns][r] = 0;

    load_step(0);
    store_step(0);
    __syncthreads();

    for (int s = 0; s < steps; ++s) {
        const int buf = s & 1;
        if (s + 1 < steps) load_step(s + 1);

        const unsigned char* xs = lds_x + buf * X_BYTES;
        const unsigned char* ws = lds_w + buf * W_BYTES;
        v4i af[WMS][4];
        v16i cinit[WMS];
#pragma unroll
        for (int ms = 0; ms < WMS; ++ms) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) af[ms][kk] = *reinterpret_cast<const v4i*>(xs + ms * 4096 + a_off[kk]);
            // initial accumulator: -8 * sum_k x[m,k] for this lane's 16 token rows (4 runs of 4)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const v4i z = *reinterpret_cast<const v4i*>(lds_s8 + buf * BM + wm * WMS * 32 + ms * 32 + 8 * j + 4 * lh);
#pragma unroll
                for (int q = 0; q < 4; ++q) cinit[ms][4 * j + q] = z[q];
            }
        }
        int scl[4];
#pragma unroll
        for (int ns = 0; ns < 4; ++ns) scl[ns] = lds_sc[buf * kBN + wn * 128 + ns * 32 + l32];
        bool wide = false;
        if constexpr (INT_SCALE) {
#pragma unroll
            for (int ns = 0; ns < 4; ++ns) wide |= ((uint32_t)(scl[ns] + (1 << 23)) >> 24) != 0;
            wide = __any(wide);
        }

#pragma unroll
        for (int ns = 0; ns < 4; ++ns) {
            v4i bf[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int2 p = *reinterpret_cast<const int2*>(ws + ns * 2048 + b_off[kk]);
                bf[kk][0] = p.x & 0x0F0F0F0F;
                bf[kk][1] = p.y & 0x0F0F0F0F;
                bf[kk][2] = (int)(((uint32_t)p.x >> 4) & 0x0F0F0F0Fu);
                bf[kk][3] = (int)(((uint32_t)p.y >> 4) & 0x0F0F0F0Fu);
            }
            const float s_f = __int_as_float(scl[ns]);
#pragma unroll
            for (int ms = 0; ms < WMS; ++ms) {
                v16i part = cinit[ms];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) part = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ms][kk], bf[kk], part, 0, 0, 0);
                // per-group scale step of Table 2
                if constexpr (!INT_SCALE) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[ms][ns][r] = fmaf((float)part[r], s_f, acc[ms][ns][r]);  // C' += float(C_g) * s_g
                } else if (__builtin_expect(wide, 0)) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[ms][ns][r] += part[r] * scl[ns];  // scale wider than 24 bits: full multiply
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[ms][ns][r] += __mul24(part[r], scl[ns]);               // C'' += C_g * s_g^INT
                }
            }
        }

        if (s + 1 < steps) store_step(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue, once per output: FLOAT(acc) * s_a[m] * c[n] / alpha (Eq. (2)), or facc * s_a[m] (Eq. (1))
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);
#pragma unroll
    for (int ns = 0; ns < 4; ++ns) {
        const int nl = wn * 128 + ns * 32 + l32;
        if (nl >= n_rows) continue;
        const int n = n0 + nl;
        float c = 1.0f;
        if constexpr (INT_SCALE) {
            if (a.chan_scale) c = a.chan_scale[expert * (size_t)a.N + n];
            c *= inv_alpha;
        }
#pragma unroll
        for (int ms = 0; ms < WMS; ++ms)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ml = wm * WMS * 32 + ms * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (ml >= m_rows) continue;
                const size_t o = (size_t)(m0 + ml) * a.N + n;
                const float sa = a.a_scale[m0 + ml];
                if constexpr (INT_SCALE) {
                    if (a.acc_out) a.acc_out[o] = acc[ms][ns][r];
                    a.out[o] = __float2half_rn((float)acc[ms][ns][r] * sa * c);
                } else {
                    a.out[o] = __float2half_rn(acc[ms][ns][r] * sa);
                }
            }
    }
}

template <int WMS, bool INT_SCALE>
hipError_t launch_tile(const GemmArgs& a, const int32_t* s8, hipStream_t stream) {
    constexpr int BM = 64 * WMS;
    const size_t smem = 2 * (size_t)BM * 128 + 2 * (size_t)kBN * 64 + 2 * kBN * 4 + 2 * BM * 4;
    auto kern = gemm_prefill_kernel<WMS, INT_SCALE>;
    if (smem > 64 * 1024) {
        static bool raised = false;
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    const int experts = a.row_offsets ? a.num_experts : 1;
    dim3 grid((a.N + kBN - 1) / kBN, (a.M + BM - 1) / BM, experts);
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, stream, a, s8);
    return hipGetLastError();
}

}  // namespace

size_t gemm_prefill_workspace_bytes(int M, int K) { return (size_t)(K / kStepK) * (size_t)M * 4; }

hipError_t launch_gemm_prefill(const GemmArgs& a, bool int_scale, void* workspace, hipStream_t stream) {
    int32_t* s8 = static_cast<int32_t*>(workspace);
    hipLaunchKernelGGL(step_sums_kernel, dim3((a.M + 3) / 4), dim3(256), 0, stream, a.xq, a.M, a.K, s8);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int wms = 2;
    if (int_scale) return wms == 4 ? launch_tile<4, true>(a, s8, stream) : launch_tile<2, true>(a, s8, stream);
    return wms == 4 ? launch_tile<4, false>(a, s8, stream) : launch_tile<2, false>(a, s8, stream);
}

}  // namespace intscale
