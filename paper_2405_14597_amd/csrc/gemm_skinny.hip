// Bandwidth-bound regime of the fine-grained W4A8 GEMM (few token rows per weight row: decode, and the per-expert
// slices of a mixture-of-experts layer).  Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper;
// float-scale form: Eq. (1) / Table 2 "Atom".  Both share everything except the per-group scale step.
//
// Work split.  A workgroup owns 16 weight rows (out-features) and up to 16*MT token rows; its waves split K on
// group boundaries and reduce their partial accumulators through LDS (int32 adds are order-free, so the result
// does not depend on the split; the fp32 partials of the float-scale form are summed in a fixed order).
//
// MFMA mapping (v_mfma_i32_16x16x64_i8).  Operand A = 16 weight rows, operand B = 16 token rows, so lane l of the
// result holds token row (l & 15) and weight rows 4*(l >> 4) .. +3.  A lane feeds rows/cols (l & 15) and the K
// slice chosen by (l >> 4).  Because a dot product does not care about the order of its terms, a lane may hold any
// 16 K-indices as long as A and B agree; here lane-group kb takes the 32 consecutive K-indices
// [32*kb, 32*kb+32) of a 128-wide step, the even ones in the first MFMA and the odd ones in the second.  That lets
// each lane fetch its 32 int4 weights with one 16-byte load straight from the canonical row-major packing.
//
// int4 -> int8 without sign fix-ups: a nibble moved to the high half of a byte is 16*q as a signed byte
// ((p << 4) & 0xF0F0F0F0 for even k, p & 0xF0F0F0F0 for odd k), so the MFMA chain returns 16*P exactly
// (|16 P| <= 2^21 per 128 indices) and one arithmetic shift recovers P before the scale step.
#include "is_common.h"

namespace intscale {
namespace {

constexpr int kStepK = 128;  // K indices consumed per step (one 16-byte weight load per lane)

// Bytes 0,2 of lo then bytes 0,2 of hi (even positions), or bytes 1,3 (odd positions).
__device__ __forceinline__ int pick_even(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u); }
__device__ __forceinline__ int pick_odd(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x07050301u); }

template <int MT, bool INT_SCALE>
__global__ __launch_bounds__(1024) void gemm_skinny_kernel(GemmArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using acc_t = typename std::conditional<INT_SCALE, int, float>::type;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int nwaves = blockDim.x / kWave;
    const int li = lane & 15;   // row of A / column of B this lane feeds; token row of its results
    const int kb = lane >> 4;   // K slice this lane feeds; its results are weight rows 4*kb..4*kb+3

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

    const int NG = a.K / a.group;
    const int steps_per_group = a.group / kStepK;
    const int n0 = blockIdx.x * 16;
    const size_t row_bytes = (size_t)a.K >> 1;
    const uint8_t* wbase = a.qweight + expert * (size_t)a.N * row_bytes;
    const acc_t* sbase = reinterpret_cast<const acc_t*>(a.scale) + expert * (size_t)a.N * NG;

    const int n_load = min(n0 + li, a.N - 1);  // clamped: rows past N are computed on a valid row and dropped
    const uint8_t* wrow = wbase + (size_t)n_load * row_bytes + kb * 16;

    const int8_t* xrow[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = min(m_base + 16 * t + li, m_end - 1);
        xrow[t] = a.xq + (size_t)m * a.K + kb * 32;
    }
    const acc_t* srow[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) srow[r] = sbase + (size_t)min(n0 + 4 * kb + r, a.N - 1) * NG;

    // Groups of this wave: an even split of NG over the waves, the first (NG % nwaves) waves take one more.
    const int gq = NG / nwaves, gr = NG % nwaves;
    const int g_begin = wave * gq + min(wave, gr);
    const int g_end = g_begin + gq + (wave < gr ? 1 : 0);

    acc_t acc[MT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = 0;

    for (int g = g_begin; g < g_end; ++g) {
        v4i part[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) part[t] = v4i{0, 0, 0, 0};

        for (int s = 0; s < steps_per_group; ++s) {
            const int step = g * steps_per_group + s;
            const uint4 wp = *reinterpret_cast<const uint4*>(wrow + (size_t)step * (kStepK / 2));
            v4i w_even, w_odd;
            w_even[0] = (int)((wp.x << 4) & 0xF0F0F0F0u);
            w_even[1] = (int)((wp.y << 4) & 0xF0F0F0F0u);
            w_even[2] = (int)((wp.z << 4) & 0xF0F0F0F0u);
            w_even[3] = (int)((wp.w << 4) & 0xF0F0F0F0u);
            w_odd[0] = (int)(wp.x & 0xF0F0F0F0u);
            w_odd[1] = (int)(wp.y & 0xF0F0F0F0u);
            w_odd[2] = (int)(wp.z & 0xF0F0F0F0u);
            w_odd[3] = (int)(wp.w & 0xF0F0F0F0u);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const uint4* xp = reinterpret_cast<const uint4*>(xrow[t] + (size_t)step * kStepK);
                const uint4 x0 = xp[0], x1 = xp[1];
                v4i x_even, x_odd;
                x_even[0] = pick_even(x0.x, x0.y);
                x_even[1] = pick_even(x0.z, x0.w);
                x_even[2] = pick_even(x1.x, x1.y);
                x_even[3] = pick_even(x1.z, x1.w);
                x_odd[0] = pick_odd(x0.x, x0.y);
                x_odd[1] = pick_odd(x0.z, x0.w);
                x_odd[2] = pick_odd(x1.x, x1.y);
                x_odd[3] = pick_odd(x1.z, x1.w);
                part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w_even, x_even, part[t], 0, 0, 0);
                part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w_odd, x_odd, part[t], 0, 0, 0);
            }
        }

        // Per-group scale step (Table 2): C'' += C_g * s_g^INT, or C' += float(C_g) * s_g.
        acc_t sc[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) sc[r] = srow[r][g];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (INT_SCALE) {
                    acc[t][r] += (part[t][r] >> 4) * sc[r];
                } else {
                    // 16*P * (s/16): the power-of-two factor is exact, so this is float(P) * s
                    acc[t][r] = fmaf((float)part[t][r], sc[r] * 0.0625f, acc[t][r]);
                }
            }
    }

    // Cross-wave reduction through LDS: slot [wave][t][lane] holds that lane's 4 values of tile t.
    v4i* slots = reinterpret_cast<v4i*>(smem_raw);
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        v4i v;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if constexpr (INT_SCALE) v[r] = acc[t][r];
            else v[r] = __float_as_int(acc[t][r]);
        }
        slots[(wave * MT + t) * kWave + lane] = v;
    }
    __syncthreads();

    // Epilogue, once per output (Eq. (2): the only int->float conversion): unit = (tile t, lane position) covers
    // one token row and 4 consecutive weight rows.
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);  // 2^-alpha_log2, exact
    for (int unit = threadIdx.x; unit < kWave * MT; unit += blockDim.x) {
        const int t = unit / kWave, ul = unit & (kWave - 1);
        acc_t tot[4] = {0, 0, 0, 0};
        for (int w = 0; w < nwaves; ++w) {
            const v4i v = slots[(w * MT + t) * kWave + ul];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (INT_SCALE) tot[r] += v[r];
                else tot[r] += __int_as_float(v[r]);
            }
        }
        const int m = m_base + 16 * t + (ul & 15);
        const int nb = n0 + 4 * (ul >> 4);
        if (m >= m_end) continue;
        const float sa = a.a_scale[m];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = nb + r;
            if (n >= a.N) continue;
            float o;
            if constexpr (INT_SCALE) {
                const float c = a.chan_scale ? a.chan_scale[expert * (size_t)a.N + n] : 1.0f;
                o = (float)tot[r] * sa * c * inv_alpha;
                if (a.acc_out) a.acc_out[(size_t)m * a.N + n] = tot[r];
            } else {
                o = tot[r] * sa;
            }
            a.out[(size_t)m * a.N + n] = __float2half_rn(o);
        }
    }
}

template <int MT, bool INT_SCALE>
hipError_t launch_one(const GemmArgs& a, int nwaves, dim3 grid, hipStream_t stream) {
    const size_t smem = (size_t)nwaves * MT * kWave * sizeof(v4i);
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, INT_SCALE>), grid, dim3(nwaves * kWave), smem, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_skinny(const GemmArgs& a, bool int_scale, hipStream_t stream) {
    const int NG = a.K / a.group;
    const int n_tiles = (a.N + 15) / 16;
    // Token rows per workgroup pass: 16*MT, MT in 1..4; more rows are covered by blockIdx.y (weights re-read).
    const int mt = a.M <= 16 ? 1 : a.M <= 32 ? 2 : a.M <= 48 ? 3 : 4;
    const int m_chunks = (a.M + 16 * mt - 1) / (16 * mt);
    // Waves per workgroup: enough waves in flight to cover HBM latency (about 16 per CU over 256 CUs), never more
    // than there are groups, at most 16.
    int nwaves = 1;
    const long long tiles = (long long)n_tiles * m_chunks * (a.row_offsets ? a.num_experts : 1);
    while (nwaves < 16 && nwaves * 2 <= NG && tiles * nwaves < 4096) nwaves *= 2;
    dim3 grid(n_tiles, m_chunks, a.row_offsets ? a.num_experts : 1);
    if (int_scale) {
        switch (mt) {
            case 1: return launch_one<1, true>(a, nwaves, grid, stream);
            case 2: return launch_one<2, true>(a, nwaves, grid, stream);
            case 3: return launch_one<3, true>(a, nwaves, grid, stream);
            default: return launch_one<4, true>(a, nwaves, grid, stream);
        }
    }
    switch (mt) {
        case 1: return launch_one<1, false>(a, nwaves, grid, stream);
        case 2: return launch_one<2, false>(a, nwaves, grid, stream);
        case 3: return launch_one<3, false>(a, nwaves, grid, stream);
        default: return launch_one<4, false>(a, nwaves, grid, stream);
    }
}

}  // namespace intscale
