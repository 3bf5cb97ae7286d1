// Fine-grained W4A8 GEMM for groups of 32 and 64 weights (group-wise quantisation, App. A.2, is not tied to the 128 the
// paper measures), on the canonical layouts.  Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper;
// float-scale form: Eq. (1) / Table 2 "Atom".  The other kernels consume K in steps of 128 with one scale step behind
// each; here a step IS a group: one matrix instruction whose K extent is the group (v_mfma_i32_16x16x64_i8 for 64,
// v_mfma_i32_16x16x32_i8 for 32) and the scale step of Table 2 behind it.  This is the covering kernel for these group
// sizes (any M, plain and grouped form), not a tuned one: per weight byte it issues two (four) times the scale steps
// and loads of the 128-wide kernels.
//
// Work split.  A workgroup (4 waves) owns 16 weight rows and up to 16 * MT token rows (of one expert); its waves split
// the groups into contiguous ranges and add their partial accumulators in LDS (int32 adds are order-free; the float
// partials are added in wave order).
//
// MFMA mapping.  Operand A = 16 token rows, B = 16 weight rows: result lane l holds weight row (l & 15), token rows
// 4 (l >> 4) .. + 3.  Lane-group kb = l >> 4 feeds the G / 4 consecutive K-indices [G kb / 4, G (kb + 1) / 4) of the
// group: G / 8 bytes of the canonical int4 row (one 8- or 4-byte load), even indices first, then odd ones (a nibble
// moved to the high half of its byte is 16 q as a signed byte: the MFMA returns 16 P, one shift recovers P); the
// activations' bytes are picked in the same order.
#include "is_common.h"

namespace intscale {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
using rsrc_t = __amdgpu_buffer_rsrc_t;

constexpr int kOutOfRange = (int)0x80000000u;  // a buffer offset past every descriptor here: the load returns 0
constexpr int kWaves = 4;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
    const unsigned n = bytes > 0xFFFFFFFFull ? 0xFFFFFFFFu : (unsigned)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}
// Bytes 0, 2 of lo then bytes 0, 2 of hi (even positions), or bytes 1, 3 (odd positions).
__device__ __forceinline__ int pick_even(int lo, int hi) { return (int)__builtin_amdgcn_perm((uint32_t)hi, (uint32_t)lo, 0x06040200u); }
__device__ __forceinline__ int pick_odd(int lo, int hi) { return (int)__builtin_amdgcn_perm((uint32_t)hi, (uint32_t)lo, 0x07050301u); }

template <int W>
struct Words {
    int v[W];
};
// W dwords at (voff, soff) of a descriptor.
template <int W>
__device__ __forceinline__ Words<W> load_words(rsrc_t r, int voff, int soff) {
    Words<W> o;
    if constexpr (W == 1) {
        o.v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
    } else if constexpr (W == 2) {
        const v2i t = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        o.v[0] = t[0];
        o.v[1] = t[1];
    } else {
        const v4i t = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) o.v[i] = t[i];
    }
    return o;
}

// G: group size (32 or 64).  MT: 16-row token tiles per workgroup.  D: groups in flight per wave.
template <int G, int MT, int D, bool INT_SCALE>
__global__ __launch_bounds__(kWaves* kWave) void gemm_small_group_kernel(GemmArgs a) {
    static_assert(G == 32 || G == 64, "one matrix instruction per group");
    using acc_t = typename std::conditional<INT_SCALE, int, float>::type;
    constexpr int WW = G / 32;  // dwords of weights per lane and group (G / 8 bytes)
    constexpr int XW = G / 16;  // dwords of activations per lane, token tile and group (G / 4 bytes)
    __shared__ v4i slots[kWaves * MT * kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int li = lane & 15, kb = lane >> 4;

    int m_begin = 0, m_end = a.M;
    size_t expert = 0;
    if (a.row_offsets) {
        expert = blockIdx.z;
        m_begin = a.row_offsets[expert];
        m_end = a.row_offsets[expert + 1];
    }
    const int m_base = m_begin + blockIdx.y * (16 * MT);
    if (m_base >= m_end) return;  // uniform over the workgroup, before any barrier
    const int m_rows = min(16 * MT, m_end - m_base);
    const int NG = a.K / G;
    const int row_bytes = a.K >> 1;
    const int n = blockIdx.x * 16 + li;

    const rsrc_t wres = make_rsrc(a.qweight + expert * (size_t)a.N * row_bytes, (size_t)a.N * row_bytes);
    const rsrc_t sres = make_rsrc(reinterpret_cast<const int*>(a.scale) + expert * (size_t)a.N * NG, (size_t)a.N * NG * 4);
    const rsrc_t xres = make_rsrc(a.xq + (size_t)m_base * a.K, (size_t)m_rows * a.K);
    // rows past the end land outside the descriptor and read as zero (every tensor is below 2 GB: no 32-bit wrap)
    const int woff = n < a.N ? n * row_bytes + kb * (G / 8) : kOutOfRange;
    const int soff = n < a.N ? n * NG * 4 : kOutOfRange;
    int xoff[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) xoff[t] = 16 * t + li < m_rows ? (16 * t + li) * a.K + kb * (G / 4) : kOutOfRange;

    // this wave's groups: an even split, the first (NG % waves) waves take one more
    const int gq = NG / kWaves, gr = NG % kWaves;
    const int g_begin = wave * gq + min(wave, gr);
    const int n_groups = gq + (wave < gr ? 1 : 0);
    const int iters = (n_groups + D - 1) / D;  // groups past n_groups are "null": all their loads return zero

    acc_t acc[MT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[t][j] = 0;

    Words<WW> wq[D];
    Words<XW> xa[D][MT];
    int sc[D];
    int nx = g_begin, nx_left = n_groups;
    auto issue = [&](int slot) {
        const bool live = nx_left > 0;
        wq[slot] = load_words<WW>(wres, live ? woff : kOutOfRange, nx * (G / 2));
#pragma unroll
        for (int t = 0; t < MT; ++t) xa[slot][t] = load_words<XW>(xres, live ? xoff[t] : kOutOfRange, nx * G);
        sc[slot] = __builtin_amdgcn_raw_buffer_load_b32(sres, live ? soff : kOutOfRange, nx * 4, 0);
        ++nx;
        --nx_left;
    };
#pragma unroll
    for (int d = 0; d < D; ++d) issue(d);

    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            // operand B: even indices of the lane's slice, then the odd ones
            int wb[2 * WW];
#pragma unroll
            for (int i = 0; i < WW; ++i) {
                const uint32_t p = (uint32_t)wq[d].v[i];
                wb[i] = (int)((p << 4) & 0xF0F0F0F0u);
                wb[WW + i] = (int)(p & 0xF0F0F0F0u);
            }
            int xb[MT][XW];
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int i = 0; i < XW / 2; ++i) {
                    xb[t][i] = pick_even(xa[d][t].v[2 * i], xa[d][t].v[2 * i + 1]);
                    xb[t][XW / 2 + i] = pick_odd(xa[d][t].v[2 * i], xa[d][t].v[2 * i + 1]);
                }
            const int scl = sc[d];
            issue(d);  // refill the slot with the group D ahead
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                v4i part;
                if constexpr (G == 64) {
                    part = __builtin_amdgcn_mfma_i32_16x16x64_i8(v4i{xb[t][0], xb[t][1], xb[t][2], xb[t][3]},
                                                                 v4i{wb[0], wb[1], wb[2], wb[3]}, v4i{0, 0, 0, 0}, 0, 0, 0);
                } else {
                    const long xl = (long)(((unsigned long)(uint32_t)xb[t][1] << 32) | (uint32_t)xb[t][0]);
                    const long wl = (long)(((unsigned long)(uint32_t)wb[1] << 32) | (uint32_t)wb[0]);
                    part = __builtin_amdgcn_mfma_i32_16x16x32_i8(xl, wl, v4i{0, 0, 0, 0}, 0, 0, 0);
                }
                // the per-group scale step of Table 2: C'' += C_g * s_g^INT (exact modulo 2^32), or C' += float(C_g) * s_g
                // (16 P * (s / 16): the power-of-two factor is exact)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if constexpr (INT_SCALE) acc[t][j] += (part[j] >> 4) * scl;
                    else acc[t][j] = fmaf((float)part[j], __int_as_float(scl) * 0.0625f, acc[t][j]);
                }
            }
        }
    }

#pragma unroll
    for (int t = 0; t < MT; ++t) {
        v4i v;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (INT_SCALE) v[j] = acc[t][j];
            else v[j] = __float_as_int(acc[t][j]);
        }
        slots[(wave * MT + t) * kWave + lane] = v;
    }
    __syncthreads();

    // Epilogue, once per output (Eq. (2): the only int -> float conversion).
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);  // 2^-alpha_log2, exact
    for (int unit = threadIdx.x; unit < kWave * MT; unit += kWaves * kWave) {
        const int t = unit / kWave, ul = unit & (kWave - 1);
        acc_t tot[4] = {0, 0, 0, 0};
        for (int w = 0; w < kWaves; ++w) {
            const v4i v = slots[(w * MT + t) * kWave + ul];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (INT_SCALE) tot[j] += v[j];
                else tot[j] += __int_as_float(v[j]);
            }
        }
        const int nn = blockIdx.x * 16 + (ul & 15);
        const int mb = m_base + 16 * t + 4 * (ul >> 4);
        if (nn >= a.N) continue;
        float c = 1.0f;
        if constexpr (INT_SCALE) {
            if (a.chan_scale) c = a.chan_scale[expert * (size_t)a.N + nn];
            c *= inv_alpha;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = mb + j;
            if (m >= m_end) continue;
            const float sa = a.a_scale[m];
            float o;
            if constexpr (INT_SCALE) {
                o = (float)tot[j] * sa * c;
                if (a.acc_out) a.acc_out[(size_t)m * a.N + nn] = tot[j];
            } else {
                o = tot[j] * sa;
            }
            a.out[(size_t)m * a.N + nn] = __float2half_rn(o);
        }
    }
}

template <int G, int MT, int D, bool INT_SCALE>
hipError_t launch_one(const GemmArgs& a, hipStream_t stream) {
    const int experts = a.row_offsets ? a.num_experts : 1;
    const dim3 grid((a.N + 15) / 16, (a.M + 16 * MT - 1) / (16 * MT), experts);
    hipLaunchKernelGGL((gemm_small_group_kernel<G, MT, D, INT_SCALE>), grid, dim3(kWaves * kWave), 0, stream, a);
    return hipGetLastError();
}

template <int G, bool INT_SCALE>
hipError_t launch_rows(const GemmArgs& a, hipStream_t stream) {
    const int experts = a.row_offsets ? a.num_experts : 1;
    // up to 16 token rows (per expert on average): one token tile and a deep ring; more: four tiles share a weight tile
    if (a.M <= 16 * experts) return launch_one<G, 1, 8, INT_SCALE>(a, stream);
    return launch_one<G, 4, 4, INT_SCALE>(a, stream);
}

}  // namespace

bool gemm_small_group_covers(int group) { return group == 32 || group == 64; }

hipError_t launch_gemm_small_group(const GemmArgs& a, bool int_scale, hipStream_t stream) {
    if (a.w_bits != 4 || !gemm_small_group_covers(a.group)) return hipErrorInvalidValue;
    if (a.group == 64) return int_scale ? launch_rows<64, true>(a, stream) : launch_rows<64, false>(a, stream);
    return int_scale ? launch_rows<32, true>(a, stream) : launch_rows<32, false>(a, stream);
}

}  // namespace intscale
