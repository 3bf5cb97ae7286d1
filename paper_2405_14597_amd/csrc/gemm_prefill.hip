// MFMA-bound regime (many token rows: prefill, and the per-expert slices of a mixture-of-experts layer) of the
// fine-grained W4A8 GEMM.  Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper; float-scale
// form: Eq. (1) / Table 2 "Atom".  The two differ only in the per-group scale step, which is where the paper's
// saving lives: one v_mad_i32_i24 per partial product against a convert plus a multiply-add.
//
// Tiling.  A workgroup of 8 waves (2 x 4) owns 128 token rows x 256 weight rows; a wave owns 64 x 64, as 4 x 4
// sub-tiles of v_mfma_i32_16x16x64_i8 (operand A = 16 token rows, operand B = 16 weight rows, so a lane's 4 results
// share one weight row and with it one group scale).  A wave stays below 256 registers, so two waves share a SIMD
// and one's scale step overlaps the other's matrix work; inside a wave the three stages of the step (unpack
// sub-tile ns+2, multiply ns+1, scale ns) are software-pipelined for the same reason.  K advances in steps of 128
// through double-buffered LDS tiles; the global loads of step s+1 are in flight while step s is multiplied.
// Workgroups are numbered so that the ones an XCD runs together form an 8 x 4 block of tiles and share their
// operand tiles through that XCD's L2.
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
constexpr int kBM = 128;
constexpr int kBN = 256;
constexpr int kThreads = 512;
constexpr int kXcds = 8;     // workgroup i is dispatched to XCD i % 8
constexpr int kGroupM = 8;   // tile rows of the block of tiles an XCD works on at a time
#ifndef INTSCALE_SWZ_A
#define INTSCALE_SWZ_A 1
#endif
#ifndef INTSCALE_SWZ_B
#define INTSCALE_SWZ_B 1
#endif
constexpr int kSwzA = INTSCALE_SWZ_A;  // activation rows: 16-byte chunk index ^= (row >> kSwzA) & 7
constexpr int kSwzB = INTSCALE_SWZ_B;  // weight rows: 8-byte chunk index ^= (row >> kSwzB) & 7

typedef float v4f __attribute__((ext_vector_type(4)));
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

// WIDE selects the integer scale step: false = v_mad_i32_i24 (exact while every scale fits 24 bits), true = full
// 32-bit multiplies (exact modulo 2^32 for any scale).  Both instantiations are launched; the flag written by
// scan_scales_kernel makes exactly one of them do the work, so neither carries the other's code or registers.
template <bool INT_SCALE, bool WIDE>
__global__ __launch_bounds__(kThreads) void gemm_prefill_kernel(GemmArgs a, const int32_t* __restrict__ s8,
                                                                const int32_t* __restrict__ wide_flag) {
    extern __shared__ __align__(16) unsigned char smem[];
    if constexpr (INT_SCALE) {
        if ((*wide_flag != 0) != WIDE) return;
    }
    constexpr int XL = kBM * 8 / kThreads;  // 16-byte activation chunks per thread and step
    constexpr int WL = kBN * 4 / kThreads;  // 16-byte weight chunks per thread and step
    constexpr int X_BYTES = kBM * 128, W_BYTES = kBN * 64;
    unsigned char* lds_x = smem;                                             // [2][128][128]
    unsigned char* lds_w = smem + 2 * X_BYTES;                               // [2][256][64]
    // every thread stores one scale and one correction word per step (the ones past 256 / 128 are zeros nobody
    // reads): the K loop stays one basic block, which keeps the instruction order chosen below
    int* lds_sc = reinterpret_cast<int*>(smem + 2 * X_BYTES + 2 * W_BYTES);  // [2][512]
    int* lds_s8 = lds_sc + 2 * kThreads;                                     // [2][512]

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int wm = wave >> 2, wn = wave & 3;

    // ---- which tile.  Linear tile numbers are dealt out so that XCD x (workgroups x, x+8, ...) gets one contiguous
    // range of them, and a range walks the output in blocks of kGroupM tile rows, column by column.
    const int tiles_n = (a.N + kBN - 1) / kBN;
    const int tiles_m = (a.M + kBM - 1) / kBM;
    int tile_m, tile_n;
    {
        const int total = tiles_m * tiles_n;
        const int q = total / kXcds, rem = total - q * kXcds;
        const int xcd = blockIdx.x % kXcds, idx = blockIdx.x / kXcds;
        const int lid = xcd * q + min(xcd, rem) + idx;
        const int gsz = kGroupM * tiles_n;
        const int g = lid / gsz, r = lid - g * gsz;
        const int gm = min(kGroupM, tiles_m - g * kGroupM);
        tile_n = r / gm;
        tile_m = g * kGroupM + (r - tile_n * gm);
    }

    int m_begin = 0, m_end = a.M;
    size_t expert = 0;
    if (a.row_offsets) {
        expert = blockIdx.z;
        m_begin = a.row_offsets[expert];
        m_end = a.row_offsets[expert + 1];
    }
    const int m0 = m_begin + tile_m * kBM;
    if (m0 >= m_end) return;  // uniform over the workgroup, before any barrier
    const int m_rows = min(kBM, m_end - m0);
    const int n0 = tile_n * kBN;
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

    // ---- loader roles.  Thread t copies activation chunks t, t+512 (64 rows apart) and weight chunks t, t+512
    // (128 rows apart); rows past the end of the tensors lie outside the descriptors and read as zero.  The XOR
    // swizzles only look at row bits below those strides, so one source and one destination offset do.
    const int x_src0 = (tid >> 3) * a.K + (tid & 7) * 16;
    const int x_dst0 = (tid >> 3) * 128 + (((tid & 7) ^ (((tid >> 3) >> kSwzA) & 7)) << 4);
    const int w_src0 = (tid >> 2) * row_bytes + (tid & 3) * 16;
    const int w_dst0 = (tid >> 2) * 64 + (((2 * (tid & 3)) ^ (((tid >> 2) >> kSwzB) & 7)) << 3);  // second half: chunk index ^ 1
    int sc_src = tid < n_rows ? tid * NG * 4 : kOutOfRange;  // advances by one scale per group
    const int z_src = tid < m_rows ? tid * 4 : kOutOfRange;

    v4i rx[XL], rw[WL];
    int rsc, rz;
    int ld_sub = 0;  // K steps already loaded of the current group (steps are loaded in order)
    auto load_step = [&](int s) {
#pragma unroll
        for (int i = 0; i < XL; ++i) rx[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, x_src0 + i * 64 * a.K, s * kStepK, 0);
#pragma unroll
        for (int i = 0; i < WL; ++i)
            rw[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, w_src0 + i * 128 * row_bytes, s * (kStepK / 2), 0);
        rsc = __builtin_amdgcn_raw_buffer_load_b32(sres, sc_src, 0, 0);
        rz = __builtin_amdgcn_raw_buffer_load_b32(zres, z_src, (s * a.M + m0) * 4, 0);
        if (++ld_sub == spg) {
            ld_sub = 0;
            sc_src += 4;
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
            *reinterpret_cast<v4i*>(lds_x + buf * X_BYTES + x_dst0 + i * 8192) = p;
        }
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            // q -> q + 8: flip the top bit of every nibble
            const int2 lo = make_int2(rw[i][0] ^ (int)0x88888888u, rw[i][1] ^ (int)0x88888888u);
            const int2 hi = make_int2(rw[i][2] ^ (int)0x88888888u, rw[i][3] ^ (int)0x88888888u);
            *reinterpret_cast<int2*>(lds_w + buf * W_BYTES + w_dst0 + i * 8192) = lo;
            *reinterpret_cast<int2*>(lds_w + buf * W_BYTES + (w_dst0 ^ 8) + i * 8192) = hi;
        }
        lds_sc[buf * kThreads + tid] = rsc;
        lds_s8[buf * kThreads + tid] = rz;
    };

    // ---- consumer roles.  MFMA 16x16x64: lane l feeds token row / weight row (l & 15) and the 16-k chunk (l >> 4) of
    // each half step; its 4 results are weight row (l & 15), token rows 4*(l >> 4)..+3.
    constexpr int MS = 4;  // 16-row token sub-tiles per wave
    constexpr int NS = 4;  // 16-row weight sub-tiles per wave
    const int l16 = lane & 15, lq = lane >> 4;
    const int a_row = (wm * 64 + l16) * 128;
    const int b_row = (wn * 64 + l16) * 64;
    int a_off[2], b_off[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        a_off[kk] = a_row + (((4 * kk + lq) ^ ((l16 >> kSwzA) & 7)) << 4);
        b_off[kk] = b_row + (((4 * kk + lq) ^ ((l16 >> kSwzB) & 7)) << 3);
    }

    using acc4 = typename std::conditional<INT_SCALE, v4i, v4f>::type;
    acc4 acc[MS][NS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int ns = 0; ns < NS; ++ns)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[ms][ns][r] = 0;

    // One K step out of LDS buffer `buf`.  The three stages of weight sub-tile ns -- unpack, multiply, scale -- are
    // issued as unpack(ns+2), multiply(ns+1), scale(ns), so that the matrix pipe and the vector ALU work together.
    auto compute_step = [&](int buf) {
        const unsigned char* xs = lds_x + buf * X_BYTES;
        const unsigned char* ws = lds_w + buf * W_BYTES;
        v4i af[MS][2], cinit[MS];
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) af[ms][kk] = *reinterpret_cast<const v4i*>(xs + ms * 2048 + a_off[kk]);
            // initial accumulator: -8 * sum_k x[m,k] for this lane's 4 token rows
            cinit[ms] = *reinterpret_cast<const v4i*>(lds_s8 + buf * kThreads + wm * 64 + ms * 16 + 4 * lq);
        }
        v4i bfu[2][2], part[2][MS];
        int scl[2];
        auto unpack = [&](int ns) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int2 p = *reinterpret_cast<const int2*>(ws + ns * 1024 + b_off[kk]);
                bfu[ns & 1][kk][0] = p.x & 0x0F0F0F0F;
                bfu[ns & 1][kk][1] = p.y & 0x0F0F0F0F;
                bfu[ns & 1][kk][2] = (int)(((uint32_t)p.x >> 4) & 0x0F0F0F0Fu);
                bfu[ns & 1][kk][3] = (int)(((uint32_t)p.y >> 4) & 0x0F0F0F0Fu);
            }
        };
        auto multiply = [&](int ns) {
            scl[ns & 1] = lds_sc[buf * kThreads + wn * 64 + ns * 16 + l16];
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                part[ns & 1][ms] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[ms][0], bfu[ns & 1][0], cinit[ms], 0, 0, 0);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                part[ns & 1][ms] =
                    __builtin_amdgcn_mfma_i32_16x16x64_i8(af[ms][1], bfu[ns & 1][1], part[ns & 1][ms], 0, 0, 0);
        };
        auto scale = [&](int ns) {  // per-group scale step of Table 2
            const int sc_i = scl[ns & 1];
            const float s_f = __int_as_float(sc_i);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int pv = part[ns & 1][ms][r];
                    if constexpr (!INT_SCALE) acc[ms][ns][r] = fmaf((float)pv, s_f, acc[ms][ns][r]);  // C' += float(C_g) * s_g
                    else if constexpr (WIDE) acc[ms][ns][r] += pv * sc_i;
                    else acc[ms][ns][r] += __mul24(pv, sc_i);                                       // C'' += C_g * s_g^INT
                }
        };
        unpack(0);
        multiply(0);
        unpack(1);
#pragma unroll
        for (int ns = 0; ns < NS; ++ns) {
            if (ns + 1 < NS) multiply(ns + 1);
            if (ns + 2 < NS) unpack(ns + 2);
            scale(ns);
            // issue order inside this stage: one MFMA, then a few vector instructions, repeated
#pragma unroll
            for (int i = 0; i < 2 * MS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    load_step(0);
    store_step(0);
    __syncthreads();
    for (int s = 0; s + 1 < steps; ++s) {
        load_step(s + 1);
        compute_step(s & 1);
        store_step((s & 1) ^ 1);
        __syncthreads();
    }
    compute_step((steps - 1) & 1);

    // ---- epilogue, once per output: FLOAT(acc) * s_a[m] * c[n] / alpha (Eq. (2)), or facc * s_a[m] (Eq. (1))
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);
    float sa[MS][4];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ml = wm * 64 + ms * 16 + 4 * lq + r;
            sa[ms][r] = ml < m_rows ? a.a_scale[m0 + ml] : 0.0f;
        }
#pragma unroll
    for (int ns = 0; ns < NS; ++ns) {
        const int nl = wn * 64 + ns * 16 + l16;
        if (nl >= n_rows) continue;
        const int n = n0 + nl;
        float c = 1.0f;
        if constexpr (INT_SCALE) {
            if (a.chan_scale) c = a.chan_scale[expert * (size_t)a.N + n];
            c *= inv_alpha;
        }
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int ml = wm * 64 + ms * 16 + 4 * lq + r;
                if (ml >= m_rows) continue;
                const size_t o = (size_t)(m0 + ml) * a.N + n;
                if constexpr (INT_SCALE) {
                    if (a.acc_out) a.acc_out[o] = acc[ms][ns][r];
                    a.out[o] = __float2half_rn((float)acc[ms][ns][r] * sa[ms][r] * c);
                } else {
                    a.out[o] = __float2half_rn(acc[ms][ns][r] * sa[ms][r]);
                }
            }
    }
}

// flag = 1 if any integer scale does not fit 24 signed bits (the limit of v_mad_i32_i24).
__global__ __launch_bounds__(256) void scan_scales_kernel(const int32_t* __restrict__ scale, size_t count,
                                                          int32_t* __restrict__ flag) {
    bool wide = false;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256)
        wide |= ((uint32_t)(scale[i] + (1 << 23)) >> 24) != 0;
    if (__any(wide) && (threadIdx.x & (kWave - 1)) == 0) atomicOr(flag, 1);
}

__global__ void clear_flag_kernel(int32_t* flag) {
    if (threadIdx.x == 0) *flag = 0;
}

template <bool INT_SCALE>
hipError_t launch_tile(const GemmArgs& a, const int32_t* s8, const int32_t* flag, hipStream_t stream) {
    const size_t smem = 2 * (size_t)kBM * 128 + 2 * (size_t)kBN * 64 + 4 * (size_t)kThreads * 4;
    const int experts = a.row_offsets ? a.num_experts : 1;
    const int tiles = ((a.N + kBN - 1) / kBN) * ((a.M + kBM - 1) / kBM);
    dim3 grid(tiles, 1, experts);
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_prefill_kernel<INT_SCALE, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess && INT_SCALE)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_prefill_kernel<INT_SCALE, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((gemm_prefill_kernel<INT_SCALE, false>), grid, dim3(kThreads), smem, stream, a, s8, flag);
    if (INT_SCALE)
        hipLaunchKernelGGL((gemm_prefill_kernel<INT_SCALE, true>), grid, dim3(kThreads), smem, stream, a, s8, flag);
    return hipGetLastError();
}

}  // namespace

constexpr size_t kHeaderBytes = 256;  // the workspace starts with the wide-scale flag

size_t gemm_prefill_workspace_bytes(int M, int K) { return kHeaderBytes + (size_t)(K / kStepK) * (size_t)M * 4; }

hipError_t launch_gemm_prefill(const GemmArgs& a, bool int_scale, void* workspace, hipStream_t stream) {
    int32_t* flag = static_cast<int32_t*>(workspace);
    int32_t* s8 = reinterpret_cast<int32_t*>(static_cast<unsigned char*>(workspace) + kHeaderBytes);
    hipLaunchKernelGGL(step_sums_kernel, dim3((a.M + 3) / 4), dim3(256), 0, stream, a.xq, a.M, a.K, s8);
    if (int_scale) {
        const int experts = a.row_offsets ? a.num_experts : 1;
        const size_t count = (size_t)experts * a.N * (a.K / a.group);
        hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(kWave), 0, stream, flag);
        hipLaunchKernelGGL(scan_scales_kernel, dim3(512), dim3(256), 0, stream, static_cast<const int32_t*>(a.scale),
                           count, flag);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return int_scale ? launch_tile<true>(a, s8, flag, stream) : launch_tile<false>(a, s8, flag, stream);
}

}  // namespace intscale
