// Bandwidth-bound regime of the fine-grained W4A8 GEMM (few token rows per weight row: decode, and the per-expert
// slices of a mixture-of-experts layer).  Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper;
// float-scale form: Eq. (1) / Table 2 "Atom".  Both share everything except the per-group scale step.
//
// Work split.  A workgroup owns 16*R weight rows (out-features) and up to 16*MT token rows; its waves split K on
// group boundaries and reduce their partial accumulators through LDS (int32 adds are order-free, so the result
// does not depend on the split; the fp32 partials of the float-scale form are summed in a fixed order).
//
// Memory pipeline.  The weights are read exactly once, so the only way to approach the HBM rate is to keep many
// 16-byte loads per lane in flight: every wave runs a D-deep rotating prefetch (weights, activations and group
// scales of step s+D are requested while step s is multiplied).
//
// MFMA mapping (v_mfma_i32_16x16x64_i8).  Operand A = 16 token rows, operand B = 16 weight rows, so lane l of the
// result holds weight row (l & 15) and token rows 4*(l >> 4) .. +3: one group scale per lane and tile.  A lane
// feeds row/column (l & 15) and the K slice chosen by (l >> 4).  Because a dot product does not care about the
// order of its terms, a lane may hold any 16 K-indices as long as A and B agree; here lane-group kb takes the 32
// consecutive K-indices [32*kb, 32*kb+32) of a 128-wide step, the even ones in the first MFMA and the odd ones in
// the second.  That lets each lane fetch its 32 int4 weights with one 16-byte load straight from the canonical
// row-major packing.
//
// Addressing.  All streams go through buffer loads: the descriptor sits in scalar registers, each lane keeps one
// 32-bit row offset per tile and the step offset is a scalar, so the K loop does no address arithmetic in the
// vector ALU, and rows past the end of a tensor read as zero instead of faulting.
//
// int4 -> int8 without sign fix-ups: a nibble moved to the high half of a byte is 16*q as a signed byte
// ((p << 4) & 0xF0F0F0F0 for even k, p & 0xF0F0F0F0 for odd k), so the MFMA chain returns 16*P exactly
// (|16 P| <= 2^21 per 128 indices) and one arithmetic shift recovers P before the scale step.
#include <stdlib.h>

#include "is_common.h"

namespace intscale {
namespace {

constexpr int kStepK = 128;  // K indices consumed per step (one 16-byte weight load per lane and weight-row tile)

// Bytes 0,2 of lo then bytes 0,2 of hi (even positions), or bytes 1,3 (odd positions).
__device__ __forceinline__ int pick_even(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u); }
__device__ __forceinline__ int pick_odd(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x07050301u); }

using rsrc_t = __amdgpu_buffer_rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
    const unsigned n = bytes > 0xFFFFFFFFull ? 0xFFFFFFFFu : (unsigned)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}
__device__ __forceinline__ v4i load16(rsrc_t r, int voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
}
__device__ __forceinline__ int load4(rsrc_t r, int voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
}

// Largest workgroup (in waves) a tile shape may use.  Two limits: the vector registers its prefetch slots,
// accumulators and operands need (a 16-wave workgroup leaves 128 per lane, 8 waves 256, 4 waves 512), and the LDS
// reduction buffer of nwaves * R * MT KB, capped at 64 KB.
constexpr int max_waves(int mt, int r, int d, bool w8 = false) {
    const int regs = 8 * d * mt + (w8 ? 9 : 5) * d * r + 8 * r * mt + 8 * r + 8 * mt + 12;
    const int by_regs = regs <= 120 ? 16 : regs <= 240 ? 8 : 4;
    const int by_lds = 64 / (mt * r);
    return by_regs < by_lds ? by_regs : by_lds;
}

constexpr int kOutOfRange = (int)0x80000000u;  // a buffer offset past every descriptor here: the load returns 0

// SPG1: every group is exactly one 128-wide step (group size 128), the common case, compiled without the
// step-in-group counters.  W8: int8 weights (fine-grained W8A8): a lane's 32 codes of a step are two 16-byte loads,
// used as they are, first half with the first 16 activations of the lane's K slice and second with the rest, and the
// MFMA chain returns P itself.
template <int MT, int R, int D, bool INT_SCALE, bool SPG1, bool W8 = false>
__global__ __launch_bounds__(max_waves(MT, R, D, W8) * kWave) void gemm_skinny_kernel(GemmArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using acc_t = typename std::conditional<INT_SCALE, int, float>::type;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int nwaves = blockDim.x / kWave;
    const int li = lane & 15;   // token row (A) and weight row (B) this lane feeds; weight row of its results
    const int kb = lane >> 4;   // K slice this lane feeds; its results are token rows 4*kb..4*kb+3 of each tile

    // Rows of this workgroup.
    int m_begin = 0, m_end = a.M;
    size_t expert = 0;
    if (a.row_offsets) {
        expert = blockIdx.z;
        m_begin = a.row_offsets[expert];
        m_end = a.row_offsets[expert + 1];
    }
    const int m_base = m_begin + blockIdx.y * (16 * MT);
    if (m_base >= m_end) return;  // uniform over the workgroup, taken before any barrier
    const int m_rows = min(16 * MT, m_end - m_base);

    const int NG = a.K / a.group;
    const int steps_per_group = SPG1 ? 1 : a.group / kStepK;
    const int n0 = blockIdx.x * (16 * R);
    const int row_bytes = W8 ? a.K : a.K >> 1;
    constexpr int kStepBytes = W8 ? kStepK : kStepK / 2;  // weight bytes of a row per step

    // Buffer descriptors: this expert's weights and scales, this workgroup's token rows.
    const rsrc_t wres = make_rsrc(a.qweight + expert * (size_t)a.N * row_bytes, (size_t)a.N * row_bytes);
    const rsrc_t sres = make_rsrc(reinterpret_cast<const int*>(a.scale) + expert * (size_t)a.N * NG,
                                  (size_t)a.N * NG * 4);
    const rsrc_t xres = make_rsrc(a.xq + (size_t)m_base * a.K, (size_t)m_rows * a.K);

    // Per-lane offsets inside the descriptors.  Rows past the end land outside the descriptor and read as zero
    // (the host checks that every tensor is below 2 GB, so the 32-bit offsets cannot wrap).
    int woff[R], soff[R], xoff[MT];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int n = n0 + 16 * r + li;
        woff[r] = n < a.N ? n * row_bytes + kb * (W8 ? 32 : 16) : kOutOfRange;
        soff[r] = n < a.N ? n * NG * 4 : kOutOfRange;
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) xoff[t] = 16 * t + li < m_rows ? (16 * t + li) * a.K + kb * 32 : kOutOfRange;
    // With 48 or 64 token rows the activations are most of what a workgroup reads, and the operand layout (a lane
    // takes 2 x 16 bytes of one of 16 rows a whole row apart) is a poor way to fetch them.  There a step's rows are
    // fetched the coalesced way instead -- request q: lane l takes chunk (l & 7) of row 8 q + (l >> 3), whole 128-byte
    // lines -- and turned into the operand layout through a private piece of LDS when the step is consumed (no
    // barrier: LDS serves one wave's requests in order; chunk index XOR row keeps both sides off each other's banks).
    constexpr bool kStageX = MT >= 3;
    [[maybe_unused]] const int xrow_off = (lane >> 3) * a.K + (lane & 7) * 16;  // rows past m_rows: past the descriptor
    [[maybe_unused]] unsigned char* xstage =
        smem_raw + (size_t)nwaves * R * MT * kWave * sizeof(v4i) + (size_t)wave * (MT * 2048);
    [[maybe_unused]] const int st_wr = (lane >> 3) * 128 + (((lane & 7) ^ ((lane >> 3) & 7)) << 4);
    [[maybe_unused]] const int st_rd0 = li * 128 + (((2 * kb) ^ (li & 7)) << 4);
    [[maybe_unused]] const int st_rd1 = li * 128 + (((2 * kb + 1) ^ (li & 7)) << 4);

    // Groups of this wave: an even split of NG over the waves, the first (NG % nwaves) waves take one more.
    const int gq = NG / nwaves, gr = NG % nwaves;
    const int g_begin = wave * gq + min(wave, gr);
    const int g_end = g_begin + gq + (wave < gr ? 1 : 0);
    const int n_steps = (g_end - g_begin) * steps_per_group;
    const int iters = (n_steps + D - 1) / D;  // steps past n_steps are "null": all their loads return zero

    acc_t acc[R][MT][4];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[r][t][j] = 0;

    // Rotating prefetch slots and the scalar cursor of the next step to request.
    v4i wq[D][R][W8 ? 2 : 1];
    v4i xa[D][MT][2];
    int sc[D][R];
    int nx_w = g_begin * steps_per_group * kStepBytes, nx_x = g_begin * steps_per_group * kStepK, nx_g = g_begin * 4;
    int nx_left = n_steps, nx_sub = 0;

    auto issue = [&](int slot) {
        const bool live = nx_left > 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            wq[slot][r][0] = load16(wres, live ? woff[r] : kOutOfRange, nx_w);
            if constexpr (W8) wq[slot][r][1] = load16(wres, live ? woff[r] : kOutOfRange, nx_w + 16);
        }
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if constexpr (kStageX) {
                // the range check sees the vector offset only: the row term goes there, the step term is scalar
                xa[slot][t][0] = load16(xres, live ? xrow_off + (2 * t) * 8 * a.K : kOutOfRange, nx_x);
                xa[slot][t][1] = load16(xres, live ? xrow_off + (2 * t + 1) * 8 * a.K : kOutOfRange, nx_x);
            } else {
                const int xo = live ? xoff[t] : kOutOfRange;
                xa[slot][t][0] = load16(xres, xo, nx_x);
                xa[slot][t][1] = load16(xres, xo, nx_x + 16);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) sc[slot][r] = load4(sres, live ? soff[r] : kOutOfRange, nx_g);
        nx_w += kStepBytes;
        nx_x += kStepK;
        --nx_left;
        if (SPG1) {
            nx_g += 4;
        } else if (++nx_sub == steps_per_group) {
            nx_sub = 0;
            nx_g += 4;
        }
    };

#pragma unroll
    for (int d = 0; d < D; ++d) issue(d);

    v4i part[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) part[r][t] = v4i{0, 0, 0, 0};
    int cur_sub = 0;
    constexpr int kShift = W8 ? 0 : 4;  // the int4 unpack leaves 16 * P

    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            // Operands of this step out of slot d.
            v4i w_even[R], w_odd[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if constexpr (W8) {
                    w_even[r] = wq[d][r][0];  // ("even" / "odd" read "first" / "second half" for int8 weights)
                    w_odd[r] = wq[d][r][W8 ? 1 : 0];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t p = (uint32_t)wq[d][r][0][i];
                        w_even[r][i] = (int)((p << 4) & 0xF0F0F0F0u);
                        w_odd[r][i] = (int)(p & 0xF0F0F0F0u);
                    }
                }
            }
            v4i x_even[MT], x_odd[MT];
            if constexpr (kStageX) {
#pragma unroll
                for (int q = 0; q < 2 * MT; ++q) *reinterpret_cast<v4i*>(xstage + q * 1024 + st_wr) = xa[d][q >> 1][q & 1];
            }
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                v4i x0, x1;
                if constexpr (kStageX) {
                    x0 = *reinterpret_cast<const v4i*>(xstage + t * 2048 + st_rd0);
                    x1 = *reinterpret_cast<const v4i*>(xstage + t * 2048 + st_rd1);
                } else {
                    x0 = xa[d][t][0];
                    x1 = xa[d][t][1];
                }
                if constexpr (W8) {
                    x_even[t] = x0;
                    x_odd[t] = x1;
                    continue;
                }
                x_even[t][0] = pick_even(x0[0], x0[1]);
                x_even[t][1] = pick_even(x0[2], x0[3]);
                x_even[t][2] = pick_even(x1[0], x1[1]);
                x_even[t][3] = pick_even(x1[2], x1[3]);
                x_odd[t][0] = pick_odd(x0[0], x0[1]);
                x_odd[t][1] = pick_odd(x0[2], x0[3]);
                x_odd[t][2] = pick_odd(x1[0], x1[1]);
                x_odd[t][3] = pick_odd(x1[2], x1[3]);
            }
            int scl[R];
#pragma unroll
            for (int r = 0; r < R; ++r) scl[r] = sc[d][r];

            issue(d);  // refill the slot with the step D ahead

#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    part[r][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(x_even[t], w_even[r], part[r][t], 0, 0, 0);
                    part[r][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(x_odd[t], w_odd[r], part[r][t], 0, 0, 0);
                }

            // Last step of a group: the per-group scale step of Table 2,
            // C'' += C_g * s_g^INT  or  C' += float(C_g) * s_g.
            if (SPG1 || ++cur_sub == steps_per_group) {
                cur_sub = 0;
                if constexpr (INT_SCALE) {
                    // v_mad_i32_i24 multiplies exactly when both factors fit 24 bits (|P| <= 2^18 always does);
                    // scales wider than that take the full 32-bit multiply.  Both are exact modulo 2^32.
                    // (a group's partial sum itself outgrows 24 bits from 8192 int4 or 512 int8 weights on)
                    bool wide = a.group > (W8 ? 256 : 4096);
#pragma unroll
                    for (int r = 0; r < R; ++r) wide |= ((uint32_t)(scl[r] + (1 << 23)) >> 24) != 0;
                    if (__builtin_expect(__any(wide), 0)) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int t = 0; t < MT; ++t)
#pragma unroll
                                for (int j = 0; j < 4; ++j) acc[r][t][j] += (part[r][t][j] >> kShift) * scl[r];
                    } else {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int t = 0; t < MT; ++t)
#pragma unroll
                                for (int j = 0; j < 4; ++j) acc[r][t][j] += __mul24(part[r][t][j] >> kShift, scl[r]);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        // 16*P * (s/16): the power-of-two factor is exact, so this is float(P) * s
                        const float fsc = __int_as_float(scl[r]) * (W8 ? 1.0f : 0.0625f);
#pragma unroll
                        for (int t = 0; t < MT; ++t)
#pragma unroll
                            for (int j = 0; j < 4; ++j) acc[r][t][j] = fmaf((float)part[r][t][j], fsc, acc[r][t][j]);
                    }
                }
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int t = 0; t < MT; ++t) part[r][t] = v4i{0, 0, 0, 0};
            }
        }
    }

    // Cross-wave reduction through LDS: slot [wave][r][t][lane] holds that lane's 4 values of tile (r, t).
    v4i* slots = reinterpret_cast<v4i*>(smem_raw);
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            v4i v;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (INT_SCALE) v[j] = acc[r][t][j];
                else v[j] = __float_as_int(acc[r][t][j]);
            }
            slots[((wave * R + r) * MT + t) * kWave + lane] = v;
        }
    __syncthreads();

    // Epilogue, once per output (Eq. (2): the only int->float conversion): unit = (tile r, tile t, lane position)
    // covers one weight row and 4 consecutive token rows.
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);  // 2^-alpha_log2, exact
    for (int unit = threadIdx.x; unit < kWave * MT * R; unit += blockDim.x) {
        const int rt = unit / kWave, ul = unit & (kWave - 1);
        const int r = rt / MT, t = rt % MT;
        acc_t tot[4] = {0, 0, 0, 0};
        for (int w = 0; w < nwaves; ++w) {
            const v4i v = slots[(w * R * MT + rt) * kWave + ul];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (INT_SCALE) tot[j] += v[j];
                else tot[j] += __int_as_float(v[j]);
            }
        }
        const int n = n0 + 16 * r + (ul & 15);
        const int mb = m_base + 16 * t + 4 * (ul >> 4);
        if (n >= a.N) continue;
        float c = 1.0f;
        if constexpr (INT_SCALE) {
            if (a.chan_scale) c = a.chan_scale[expert * (size_t)a.N + n];
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
                if (a.acc_out) a.acc_out[(size_t)m * a.N + n] = tot[j];
            } else {
                o = tot[j] * sa;
            }
            a.out[(size_t)m * a.N + n] = __float2half_rn(o);
        }
    }
}

struct SkinnyConfig {
    int mt, r, d, nwaves;
};

// Tile shape and wave count for a problem.  Aim: a few thousand waves in flight over 256 CUs, each with D*R KB of
// weight loads outstanding, and at least one workgroup per CU.
SkinnyConfig choose_config(const GemmArgs& a) {
    const int NG = a.K / a.group;
    SkinnyConfig c;
    c.mt = a.M <= 16 ? 1 : a.M <= 32 ? 2 : a.M <= 48 ? 3 : 4;
    const int experts = a.row_offsets ? a.num_experts : 1;
    const long long m_chunks = ((long long)a.M + 16 * c.mt - 1) / (16 * c.mt) * experts;
    c.r = 1;
    if (c.mt >= 2) {
        // more token rows: reuse each activation fragment over more weight-row tiles
        if ((long long)((a.N + 63) / 64) * m_chunks >= 256) c.r = 4;
        else if ((long long)((a.N + 31) / 32) * m_chunks >= 256) c.r = 2;
    } else if ((long long)((a.N + 31) / 32) * m_chunks >= 512) {
        c.r = 2;
    }
    static const int env_r = env_int("INTSCALE_SKINNY_R", 0);  // experiments; read once
    if (env_r) c.r = env_r;
    if (c.r != 1 && c.r != 2 && c.r != 4) c.r = 1;
    // 48 or 64 token rows: the staged activations leave registers for two steps in flight, not four
    c.d = (c.mt >= 3 || c.mt * c.r >= 8) ? 2 : 4;
    static const int env_d = env_int("INTSCALE_SKINNY_D", 0);
    if (env_d) c.d = env_d;
    if (c.d != 2 && c.d != 4) c.d = 2;
    if (a.w_bits == 8) c.d = 2;
    const long long tiles = (long long)((a.N + 16 * c.r - 1) / (16 * c.r)) * m_chunks;
    int nw = 1;
    // LDS: nwaves * R * MT KB for the reduction, at most 64 KB.
    const int cap = max_waves(c.mt, c.r, c.d, a.w_bits == 8);
    while (nw * 2 <= cap && nw * 2 <= NG && tiles * nw < 4096) nw *= 2;
    static const int env_w = env_int("INTSCALE_SKINNY_WAVES", 0);
    if (env_w) nw = env_w;
    if (nw < 1) nw = 1;
    while (nw > 1 && (nw > NG || nw > cap)) nw /= 2;
    c.nwaves = nw;
    return c;
}

template <int MT, int R, int D, bool INT_SCALE, bool W8 = false>
hipError_t launch_one(const GemmArgs& a, const SkinnyConfig& c, hipStream_t stream) {
    const int experts = a.row_offsets ? a.num_experts : 1;
    dim3 grid((a.N + 16 * R - 1) / (16 * R), (a.M + 16 * MT - 1) / (16 * MT), experts);
    // reduction slots, then (48 or 64 token rows) one step of activations per wave
    const size_t smem = (size_t)c.nwaves * R * MT * kWave * sizeof(v4i) + (MT >= 3 ? (size_t)c.nwaves * MT * 2048 : 0);
    auto k1 = gemm_skinny_kernel<MT, R, D, INT_SCALE, true, W8>;
    auto k2 = gemm_skinny_kernel<MT, R, D, INT_SCALE, false, W8>;
    if (smem > 64 * 1024) {
        static LdsLimit limit1, limit2;  // per instantiation
        hipError_t e = limit1.raise(reinterpret_cast<const void*>(k1));
        if (e == hipSuccess) e = limit2.raise(reinterpret_cast<const void*>(k2));
        if (e != hipSuccess) return e;
    }
    if (a.group == kStepK) hipLaunchKernelGGL(k1, grid, dim3(c.nwaves * kWave), smem, stream, a);
    else hipLaunchKernelGGL(k2, grid, dim3(c.nwaves * kWave), smem, stream, a);
    return hipGetLastError();
}

template <int MT, bool INT_SCALE>
hipError_t launch_mt(const GemmArgs& a, const SkinnyConfig& c, hipStream_t stream) {
    if (a.w_bits == 8) {  // int8 weights: two steps in flight (a step's weights take twice the registers)
        switch (c.r) {
            case 1: return launch_one<MT, 1, 2, INT_SCALE, true>(a, c, stream);
            case 2: return launch_one<MT, 2, 2, INT_SCALE, true>(a, c, stream);
            default: return launch_one<MT, 4, 2, INT_SCALE, true>(a, c, stream);
        }
    }
    if (c.d == 2) {
        switch (c.r) {
            case 1: return launch_one<MT, 1, 2, INT_SCALE>(a, c, stream);
            case 2: return launch_one<MT, 2, 2, INT_SCALE>(a, c, stream);
            default: return launch_one<MT, 4, 2, INT_SCALE>(a, c, stream);
        }
    }
    switch (c.r) {
        case 1: return launch_one<MT, 1, 4, INT_SCALE>(a, c, stream);
        case 2: return launch_one<MT, 2, 4, INT_SCALE>(a, c, stream);
        default: return launch_one<MT, 4, 4, INT_SCALE>(a, c, stream);
    }
}

template <bool INT_SCALE>
hipError_t launch_scale(const GemmArgs& a, const SkinnyConfig& c, hipStream_t stream) {
    switch (c.mt) {
        case 1: return launch_mt<1, INT_SCALE>(a, c, stream);
        case 2: return launch_mt<2, INT_SCALE>(a, c, stream);
        case 3: return launch_mt<3, INT_SCALE>(a, c, stream);
        default: return launch_mt<4, INT_SCALE>(a, c, stream);
    }
}

}  // namespace

hipError_t launch_gemm_skinny(const GemmArgs& a, bool int_scale, hipStream_t stream) {
    const SkinnyConfig c = choose_config(a);
    return int_scale ? launch_scale<true>(a, c, stream) : launch_scale<false>(a, c, stream);
}

}  // namespace intscale
