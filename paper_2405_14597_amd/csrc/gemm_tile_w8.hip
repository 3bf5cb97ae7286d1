// Fine-grained W8A8 GEMM (int8 weights in groups along K, int8 per-token activations), tiled MFMA kernel for any
// number of token rows.  The paper's LLaMA-3 recipe uses fine-grained W8A8 with integer scales for the
// down-projection layers (Sec. 5.5, Table 5); the arithmetic is that of the W4A8 layer -- Eq. (2) / Table 2 "Ours"
// with integer scales, Eq. (1) / Table 2 "Atom" with float scales -- with nothing to unpack: a group's partial sum
// |P| <= 128 * 128 * 128 = 2^21 still fits the 24-bit multiplier of the integer scale step.
//
// Same tiling as the W4A8 tiled kernel: a workgroup of 8 waves (2 x 4) owns 128 token rows x 256 weight rows, a wave
// 64 x 64 as 4 x 4 sub-tiles of v_mfma_i32_16x16x64_i8.  K advances in steps of 128 through a ring of 3 LDS stages
// (16 KB of activations, 32 KB of weights, 1 KB of scales each) filled by buffer loads that write LDS directly, two
// steps ahead.  Both operands are read in their canonical layouts: rows of 128 bytes per step on both sides, the
// 16-byte chunk index XORed with (row >> 1) & 7 on the way in (applied to the global address each lane fetches), so
// that the operand reads of 16 consecutive rows fall on different banks.  There is no zero point, hence no
// correction and no preparation of the activations; the scales are transposed to [group][weight row] as for W4A8.
#include "tile_common.h"

namespace intscale {
namespace {

constexpr int kStepK = 128;
constexpr int kBM = kTileRows;
constexpr int kBN = 256;
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr int kXcds = 8;
constexpr int kGroupM = 8;
constexpr int kStages = 3;     // LDS ring; tiles are requested kStages - 1 steps ahead
constexpr int kXLoads = 2;     // 1 KB blocks (8 rows x 128 B) of the activation tile a wave requests per step
constexpr int kWLoads = 4;     // ... of the weight tile
constexpr int kTileLoads = kXLoads + kWLoads;  // (+1 on wave 0: the step's 256 scales)
constexpr int kXBytes = kBM * 128, kWBytes = kBN * 128, kAuxBytes = 1024;
constexpr int kStageBytes = kXBytes + kWBytes + kAuxBytes;
static_assert(kStages * kStageBytes <= 160 * 1024, "LDS ring does not fit");

// First of the stream: clears the wide-scale flag and, for the grouped form, lists the row tiles that exist.
__global__ void prepare_w8_kernel(int32_t* __restrict__ wide_flag, const int32_t* __restrict__ row_offsets, int num_experts,
                                  int M, int2* __restrict__ tile_table) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    *wide_flag = 0;
    if (row_offsets == nullptr) return;
    const int slots = tile_slots(M, num_experts);
    int slot = 0;
    for (int e = 0; e < num_experts; ++e) {
        const int rows = row_offsets[e + 1] - row_offsets[e];
        for (int t = 0; t * kBM < rows && slot < slots; ++t) tile_table[slot++] = make_int2(e, t);
    }
    for (; slot < slots; ++slot) tile_table[slot] = make_int2(-1, 0);
}

template <bool INT_SCALE, bool WIDE>
__device__ __forceinline__ void gemm_w8_tile(const GemmArgs& a, const int32_t* __restrict__ scale_t,
                                             const int2* __restrict__ tile_table, unsigned char* smem) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave >> 2, wn = wave & 3;

    // ---- which tile (numbering as in the W4A8 tiled kernel)
    const int tiles_n = (a.N + kBN - 1) / kBN;
    const int tiles_m = a.row_offsets ? tile_slots(a.M, a.num_experts) : (a.M + kBM - 1) / kBM;
    int tile_m, tile_n;
    if (a.row_offsets) {
        tile_m = blockIdx.x / tiles_n;
        tile_n = blockIdx.x - tile_m * tiles_n;
    } else {
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
        const int2 entry = tile_table[tile_m];
        if (entry.x < 0) return;  // an empty slot (uniform over the workgroup, before any barrier)
        expert = entry.x;
        tile_m = entry.y;
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

    // ---- loader roles.  Rows past the end of a tensor lie outside its descriptor and read as zero.  A lane's LDS
    // slot is fixed by the load (block b, lane l: row 8 b + (l >> 3), chunk slot l & 7); the swizzle picks the global
    // chunk that belongs there.
    v4i xdesc = make_desc(a.xq + (size_t)m0 * a.K, (size_t)m_rows * a.K);
    v4i wdesc = make_desc(a.qweight + (expert * (size_t)a.N + n0) * a.K, (size_t)n_rows * a.K);
    v4i adesc = make_desc(nullptr, 0);
    int grp_inc = 0;
    if (wave == 0) {
        adesc = make_desc(scale_t + (expert * NG) * (size_t)a.N + n0, ((size_t)(NG - 1) * a.N + n_rows) * 4);
        grp_inc = a.N * 4;
    }
    const int aux_voff = lane * 16;
    int x_voff[kXLoads], w_voff[kWLoads];
#pragma unroll
    for (int i = 0; i < kXLoads; ++i) {
        const int r = 8 * (wave + kWaves * i) + (lane >> 3);
        x_voff[i] = r * a.K + (((lane & 7) ^ ((r >> 1) & 7)) << 4);
    }
#pragma unroll
    for (int i = 0; i < kWLoads; ++i) {
        const int r = 8 * (wave + kWaves * i) + (lane >> 3);
        w_voff[i] = r * a.K + (((lane & 7) ^ ((r >> 1) & 7)) << 4);
    }
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const unsigned lds_x0 = wave * 1024, lds_w0 = kXBytes + wave * 1024, lds_aux = kXBytes + kWBytes;
    // Steps past the last one request nothing useful: their descriptors are emptied (every offset then lies outside
    // and the load writes zeros into a stage nobody reads), which keeps the counted waits the same to the end.
    const int x_bytes = xdesc[2], w_bytes = wdesc[2], a_bytes = adesc[2];
    unsigned rq_base = lds0;
    int rq_k = 0, aux_soff = 0, ld_sub = 0;
    auto request_step = [&](int t) {
        const bool live = t < steps;
        xdesc[2] = live ? x_bytes : 0;
        wdesc[2] = live ? w_bytes : 0;
        adesc[2] = live ? a_bytes : 0;
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) load_to_lds_b128(xdesc, rq_base, lds_x0 + i * kWaves * 1024, x_voff[i], rq_k);
#pragma unroll
        for (int i = 0; i < kWLoads; ++i) load_to_lds_b128(wdesc, rq_base, lds_w0 + i * kWaves * 1024, w_voff[i], rq_k);
        if (wave == 0) load_to_lds_b128(adesc, rq_base, lds_aux, aux_voff, aux_soff);
        rq_k += kStepK;
        rq_base = rq_base + kStageBytes == lds0 + kStages * kStageBytes ? lds0 : rq_base + kStageBytes;
        const bool group_done = ++ld_sub == spg;
        ld_sub = group_done ? 0 : ld_sub;
        aux_soff += group_done ? grp_inc : 0;
    };

    // ---- consumer roles.  MFMA 16x16x64: lane l feeds token row / weight row (l & 15) and 16 of the 64 k of each half
    // step, chosen by (l >> 4): chunk 4 kk + (l >> 4) of the row's eight; its 4 results are weight row (l & 15), token
    // rows 4 * (l >> 4) .. +3.
    constexpr int MS = 4, NS = 4;
    const int l16 = lane & 15, lq = lane >> 4;
    int a_off[2], b_off[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int ar = wm * 64 + l16, br = wn * 64 + l16;  // + 16 ms / ns: the swizzle bits used are below 16
        a_off[kk] = ar * 128 + (((4 * kk + lq) ^ ((ar >> 1) & 7)) << 4);
        b_off[kk] = kXBytes + br * 128 + (((4 * kk + lq) ^ ((br >> 1) & 7)) << 4);
    }
    const int sc_off = kXBytes + kWBytes + (wn * 64 + l16) * 4;

    using acc4 = typename std::conditional<INT_SCALE, v4i, v4f>::type;
    acc4 acc[MS][NS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int ns = 0; ns < NS; ++ns)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[ms][ns][r] = 0;

    struct Operands {
        v4i af[MS][2];  // activation fragments
        v4i bf[NS][2];  // weight fragments
        int scl[NS];    // group scales
    };
    auto read_fragments = [&](Operands& o, const unsigned char* st) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
            for (int ns = 0; ns < NS; ++ns) o.bf[ns][kk] = *reinterpret_cast<const v4i*>(st + ns * 2048 + b_off[kk]);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) o.af[ms][kk] = *reinterpret_cast<const v4i*>(st + ms * 2048 + a_off[kk]);
        }
    };
    auto read_scales = [&](Operands& o, const unsigned char* st) {
#pragma unroll
        for (int ns = 0; ns < NS; ++ns) o.scl[ns] = *reinterpret_cast<const int*>(st + sc_off + ns * 64);
    };
    // Step t's tile is visible once only this wave's requests of the step after it are outstanding (wave 0 issues one
    // more per step; at the end the wait is for all of them), its own LDS reads are done, and every wave is past the
    // barrier.
    auto wait_tile_and_sync = [&](bool full_flight) {
        if (!full_flight) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else if (wave == 0) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kTileLoads + 1) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kTileLoads) : "memory");
    };

    // One K step: cur holds step s, nxt receives step s+1; multiply(ns+1) is issued ahead of scale(ns) so that the
    // matrix pipe and the vector ALU work together.  Half way, the barrier that publishes step s+1 (everybody has then
    // finished reading step s out of LDS, whose stage is handed to step s+3), then the reads for nxt.
    auto compute_step = [&](Operands& cur, Operands& nxt, int s) {
        v4i part[2][MS];
        auto multiply = [&](int ns) {
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                part[ns & 1][ms] = __builtin_amdgcn_mfma_i32_16x16x64_i8(cur.af[ms][0], cur.bf[ns][0], v4i{0, 0, 0, 0}, 0, 0, 0);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                part[ns & 1][ms] = __builtin_amdgcn_mfma_i32_16x16x64_i8(cur.af[ms][1], cur.bf[ns][1], part[ns & 1][ms], 0, 0, 0);
        };
        auto scale = [&](int ns) {  // per-group scale step of Table 2
            const int sc_i = cur.scl[ns];
            const float s_f = __int_as_float(sc_i);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int pv = part[ns & 1][ms][r];
                    if constexpr (!INT_SCALE) acc[ms][ns][r] = fmaf((float)pv, s_f, acc[ms][ns][r]);  // C' += float(C_g) * s_g
                    else if constexpr (WIDE) {
                        int prod = pv * sc_i;
                        asm volatile("" : "+v"(prod));  // else a 64-bit multiply-add with register pairs
                        acc[ms][ns][r] += prod;
                    }
                    else acc[ms][ns][r] += __mul24(pv, sc_i);                                       // C'' += C_g * s_g^INT
                }
        };
        const unsigned char* next_stage = smem + ((s + 1) % kStages) * kStageBytes;
        multiply(0);
#pragma unroll
        for (int ns = 0; ns < NS; ++ns) {
            if (ns + 1 < NS) multiply(ns + 1);
            if (ns == 2) {  // every fragment of cur has been handed to the matrix pipe by now
                wait_tile_and_sync(s + kStages - 1 < steps);  // step s+2 was requested
                request_step(s + kStages);
                read_fragments(nxt, next_stage);
                read_scales(nxt, next_stage);
            }
            scale(ns);
        }
        asm volatile(""
                     : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[0][2]), "+v"(acc[0][3]), "+v"(acc[1][0]), "+v"(acc[1][1]),
                       "+v"(acc[1][2]), "+v"(acc[1][3]), "+v"(acc[2][0]), "+v"(acc[2][1]), "+v"(acc[2][2]), "+v"(acc[2][3]),
                       "+v"(acc[3][0]), "+v"(acc[3][1]), "+v"(acc[3][2]), "+v"(acc[3][3]));
    };

    Operands ops0, ops1;
#pragma unroll
    for (int t = 0; t < kStages; ++t) request_step(t);
    if (steps < kStages) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    else if (wave == 0) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * (kTileLoads + 1)) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * kTileLoads) : "memory");
    read_fragments(ops0, smem);
    read_scales(ops0, smem);
    for (int s = 0; s < steps; s += 2) {
        compute_step(ops0, ops1, s);
        if (s + 1 < steps) compute_step(ops1, ops0, s + 1);  // uniform over the workgroup (it holds a barrier)
    }

    // ---- epilogue, once per output: FLOAT(acc) * s_a[m] * c[n] / alpha (Eq. (2)), or facc * s_a[m] (Eq. (1))
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);
    float sa[MS][4];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ml = wm * 64 + ms * 16 + 4 * lq + r;
            sa[ms][r] = ml < m_rows ? a.a_scale[m0 + ml] : 0.0f;
        }
    const bool staged = (a.N & 7) == 0 && a.acc_out == nullptr;
    constexpr int kPitch = 264;  // halves per LDS row: 256 + 8, so that rows keep 16-byte alignment
    __half* otile = reinterpret_cast<__half*>(smem);
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
                __half h;
                if constexpr (INT_SCALE) h = __float2half_rn((float)acc[ms][ns][r] * sa[ms][r] * c);
                else h = __float2half_rn(acc[ms][ns][r] * sa[ms][r]);
                if (staged) {
                    otile[ml * kPitch + nl] = h;
                } else if (ml < m_rows) {
                    const size_t o = (size_t)(m0 + ml) * a.N + n;
                    if constexpr (INT_SCALE) {
                        if (a.acc_out) a.acc_out[o] = acc[ms][ns][r];
                    }
                    a.out[o] = h;
                }
            }
    }
    if (staged) {
        __syncthreads();
        const int chunk = tid & 31;  // 8 outputs
        if (chunk * 8 < n_rows) {
#pragma unroll
            for (int pass = 0; pass < kBM / 16; ++pass) {
                const int ml = pass * 16 + (tid >> 5);
                if (ml < m_rows)
                    *reinterpret_cast<uint4*>(a.out + (size_t)(m0 + ml) * a.N + n0 + chunk * 8) =
                        *reinterpret_cast<const uint4*>(otile + ml * kPitch + chunk * 8);
            }
        }
    }
}

template <bool INT_SCALE>
__global__ __launch_bounds__(kThreads) void gemm_w8_kernel(GemmArgs a, const int32_t* __restrict__ scale_t,
                                                           const int32_t* __restrict__ wide_flag,
                                                           const int2* __restrict__ tile_table) {
    extern __shared__ __align__(16) unsigned char smem[];  // [kStages][activations 16 KB | weights 32 KB | scales 1 KB]
    if constexpr (INT_SCALE) {
        if (*wide_flag != 0) gemm_w8_tile<true, true>(a, scale_t, tile_table, smem);
        else gemm_w8_tile<true, false>(a, scale_t, tile_table, smem);
    } else {
        gemm_w8_tile<false, false>(a, scale_t, tile_table, smem);
    }
}

template <bool INT_SCALE>
hipError_t launch_w8_tile(const GemmArgs& a, const int32_t* scale_t, const int32_t* flag, const int2* tile_table,
                          hipStream_t stream) {
    const size_t smem = (size_t)kStages * kStageBytes;
    const int tiles_m = a.row_offsets ? tile_slots(a.M, a.num_experts) : (a.M + kBM - 1) / kBM;
    const int tiles = ((a.N + kBN - 1) / kBN) * tiles_m;
    static LdsLimit limit;  // per instantiation
    const hipError_t e = limit.raise(reinterpret_cast<const void*>(gemm_w8_kernel<INT_SCALE>));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_w8_kernel<INT_SCALE>), dim3(tiles), dim3(kThreads), smem, stream, a, scale_t, flag,
                       tile_table);
    return hipGetLastError();
}

size_t w8_header_bytes(int experts, int M) { return pad256(16 + (size_t)tile_slots(M, experts) * sizeof(int2)); }

}  // namespace

// workspace = [flag and row-tile slots, padded to 256 B | transposed scales: experts x K/group x N words]
size_t gemm_w8_workspace_bytes(int num_experts, int M, int N, int K, int group) {
    return w8_header_bytes(num_experts, M) + pad256((size_t)num_experts * N * (K / group) * 4);
}

// `a.qweight` holds int8 codes [N,K] (one byte per code) here.
hipError_t launch_gemm_w8(const GemmArgs& a, bool int_scale, void* workspace, hipStream_t stream) {
    const int experts = a.row_offsets ? a.num_experts : 1;
    const int NG = a.K / a.group;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int32_t* flag = reinterpret_cast<int32_t*>(ws);
    int2* tile_table = reinterpret_cast<int2*>(ws + 16);
    int32_t* scale_t = reinterpret_cast<int32_t*>(ws + w8_header_bytes(experts, a.M));
    hipLaunchKernelGGL(prepare_w8_kernel, dim3(1), dim3(kWave), 0, stream, flag, a.row_offsets, experts, a.M, tile_table);
    const dim3 sgrid((a.N + 63) / 64, (NG + 63) / 64, experts);
    const int32_t* scale = static_cast<const int32_t*>(a.scale);
    if (int_scale) hipLaunchKernelGGL(prepare_scales_kernel<true>, sgrid, dim3(256), 0, stream, scale, a.N, NG, scale_t, flag);
    else hipLaunchKernelGGL(prepare_scales_kernel<false>, sgrid, dim3(256), 0, stream, scale, a.N, NG, scale_t, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return int_scale ? launch_w8_tile<true>(a, scale_t, flag, tile_table, stream)
                     : launch_w8_tile<false>(a, scale_t, flag, tile_table, stream);
}

}  // namespace intscale
