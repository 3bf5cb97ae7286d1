// Decode regime (at most 64 token rows) of the fine-grained W4A8 GEMM: a persistent, activation-stationary kernel.
// Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper; float-scale form: Eq. (1) / Table 2
// "Atom".
//
// Why this shape.  With so few token rows the layer is a stream of packed int4 weights out of HBM, read once.  At
// 10 us per launch what decides the speed is (1) how many bytes every CU keeps in flight, (2) that all CUs finish
// together and (3) how many dependent memory latencies sit on the critical path.  So:
//   - one workgroup of W waves per CU, launched once ("persistent"); workgroup j owns the 16-row weight tiles
//     j, j+G, j+2G, ... (G = number of workgroups), so the CUs carry equal shares to within one tile;
//   - the W waves of a workgroup split K on group boundaries; a wave keeps the activations of its K range in
//     registers for the whole kernel (MFMA-ready, loaded once), so its only stream is the weights and group scales
//     of its K range, tile after tile, in a rotating prefetch DT tiles deep;
//   - the waves' partial accumulators of a tile meet in LDS (two buffers, one barrier per tile); int32 adds are
//     order-free so the split never changes a bit, and the float-scale partials are added in wave order;
//   - the epilogue (the one int->float conversion of Eq. (2), times s_a[m] * c[n] / alpha) is spread over the
//     workgroup's threads, one output each, with its scalars fetched ahead of time.
//
// MFMA mapping (v_mfma_i32_16x16x64_i8): operand A = 16 token rows, operand B = 16 weight rows; lane l feeds
// row/column (l & 15) and K slice (l >> 4); its 4 results are weight row (l & 15), token rows 4*(l >> 4)..+3.
// A dot product does not care about the order of its terms, so lane-group kb simply takes the 32 consecutive
// K-indices [32*kb, 32*kb+32) of a 128-wide step, even ones in one MFMA and odd ones in the next: each lane gets its
// 32 int4 weights with one 16-byte load from the canonical row-major packing.
//
// int4 -> int8: a nibble in the high half of a byte is 16*q as a signed byte ((p << 4) & 0xF0F0F0F0 for even k,
// p & 0xF0F0F0F0 for odd k).  The MFMA pair returns 16*P exactly (|16 P| <= 2^21), one shift recovers P.  (A zero
// point instead, q + 8 with the correction -8 * sum_k x as the MFMA's initial accumulator, saves that shift but puts
// an LDS read of the correction in front of every MFMA pair; measured here it made every shape 5-15 % slower: what
// bounds this kernel is the chain of dependent latencies per tile, not the count of vector instructions.)
//
// The scale step runs once per 128-wide step with that step's group scale; for groups wider than 128 this is the
// same integer by distributivity ((P1 + P2) * s = P1 * s + P2 * s modulo 2^32).
#include "act_common.h"
#include "is_common.h"

namespace intscale {
namespace {

constexpr int kStepK = 128;
constexpr int kOutOfRange = (int)0x80000000u;  // a buffer offset past every descriptor here: the load returns 0

using rsrc_t = __amdgpu_buffer_rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
    const unsigned n = bytes > 0x7FFFFFFFull ? 0x7FFFFFFFu : (unsigned)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}

__device__ __forceinline__ int pick_even(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u); }
__device__ __forceinline__ int pick_odd(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x07050301u); }

// Workgroup barrier that only waits for this wave's LDS traffic.  __syncthreads() would also drain every global
// load in flight (s_waitcnt vmcnt(0)) and with it the prefetch that this kernel lives on.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// MT: 16-row token tiles.  XS: steps of K a wave owns at most (its activations stay in 8*XS*MT registers).
// DT: weight tiles in flight per wave.
// WAVES: waves per workgroup (16 leaves 128 vector registers per lane, 8 leaves 256).
// FUSEQ: one fp16 token (M = 1) instead of quantised activations: the per-token quantiser of Appendix A.1 runs in the
// prologue (every wave covers its own K slice, the absmax meets in LDS behind the barrier that is there anyway).
// XLDS: one token (M = 1) whose K slice per wave is too long to keep its operand registers for the whole kernel
// (K from 12288 to 20480): the token's codes stay in LDS, one copy per workgroup, and every step reads its two operand
// registers from there.
template <int MT, int XS, int DT, int WAVES, bool INT_SCALE, bool FUSEQ = false, bool XLDS = false>
__global__ __launch_bounds__(WAVES * kWave) void gemm_decode_kernel(GemmArgs a, DecodePlan p) {
    static_assert(!FUSEQ || MT == 1, "the fused quantiser handles one token");
    static_assert(!XLDS || MT == 1, "operands from LDS: one token");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using acc_t = typename std::conditional<INT_SCALE, int, float>::type;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    constexpr int W = WAVES;
    constexpr int T = W * kWave;
    constexpr int OPT = (256 * MT + T - 1) / T;  // outputs of a tile each thread finishes
    const int li = lane & 15, kb = lane >> 4;
    const int NG = p.num_groups;
    const int row_bytes = a.K >> 1;
    const int G = gridDim.x;
    const int tile0 = blockIdx.x;
    const int my_tiles = p.tiles_q + ((int)blockIdx.x < p.tiles_r ? 1 : 0);  // >= 1: at most `tiles` workgroups run

    // K range of this wave: whole groups, the first p.gr waves take one more.
    const int g0 = wave * p.gq + min(wave, p.gr);
    const int ng = p.gq + (wave < p.gr ? 1 : 0);
    const int s0 = g0 * p.spg;
    const int ns = ng * p.spg;  // <= XS by construction of the plan

    const rsrc_t wres = make_rsrc(a.qweight, (size_t)a.N * row_bytes);
    const rsrc_t sres = make_rsrc(a.scale, (size_t)a.N * NG * 4);
    const rsrc_t xres = FUSEQ ? make_rsrc(a.x_fp16, (size_t)a.K * 2) : make_rsrc(a.xq, (size_t)a.M * a.K);
    const rsrc_t cres = make_rsrc(a.chan_scale, a.chan_scale ? (size_t)a.N * 4 : 0);

    // LDS: two buffers of partial accumulators [W][MT][64 lanes][4], then two buffers of one tile's group scales
    // (16 rows x NG, rows padded by one word so that the 16 rows a wave reads fall into different banks).
    int* lds = reinterpret_cast<int*>(smem_raw);
    const int part_ints = W * MT * kWave * 4;
    const int srow_ints = NG + 1;
    int* lds_scale = lds + 2 * part_ints;
    const int scale_ints = 16 * srow_ints;
    // then, per scale buffer, one word per wave: "a scale staged by this wave does not fit 24 bits"; then (64 token
    // rows) the activation staging
    int* lds_wide = lds_scale + 2 * scale_ints;

    // ---- cheap parts of this thread's roles, needed to start the stream (the rest is set up while it is in flight)
    const int n_out = threadIdx.x & 15;
    const bool writer0 = threadIdx.x < 256 * MT && (int)(threadIdx.x >> 4) < a.M;
    // Byte offsets inside a tile; a tile's base is added per request.  The whole offset travels in the vector offset,
    // which is what the descriptor's range check sees: rows and columns past N read as zero without a compare, and an
    // offset that starts out of range (0x80000000 + anything below 2 GB) stays there.
    const int woff = li * row_bytes + s0 * (kStepK / 2) + kb * 16;  // step i: + 64 i (scalar, or out of range past ns)
    const int cs_off = writer0 ? n_out * 4 : kOutOfRange;
    const int tile_w_bytes = 16 * row_bytes, tile_s_bytes = 16 * NG * 4;

    // The group scales of a tile go through LDS and are needed one tile before its weights, so they travel in slots
    // of their own, at least two deep (with one weight slot the next tile's scales must already be on their way
    // while the current tile is multiplied).
    constexpr int SD = DT > 1 ? DT : 2;
    // Where the "some scale needs more than 24 bits" test of the integer scale step is made: once per tile while its
    // scales are staged (one word of LDS per wave and tile; pays with several token tiles, where it keeps the branch
    // out of every step), else per step on the scales just read (one token tile: an LDS read more per tile would
    // lengthen the chain of dependent latencies that bounds those shapes).
    constexpr bool kTileFlag = MT >= 2;
    constexpr bool kStepRefill = DT == 1 && (WAVES == 8 || XLDS);
    v4i wq[DT][XS];
    // words of a tile's 16 x NG block of scales each thread copies: NG <= XS * WAVES by construction of the plan
    constexpr int SJ = (16 * XS * WAVES + T - 1) / T;
    int scv[SD][SJ];
    float cs[DT];

    // (The tile number is made opaque to the optimiser in these requests: it would otherwise keep one precomputed
    // vector offset per unrolled position of the tile loop for the whole kernel, and spill.)
    auto issue_scales = [&](int slot, int tile) {
        asm volatile("" : "+s"(tile));
        const int sbase = tile * tile_s_bytes;
#pragma unroll
        for (int j = 0; j < SJ; ++j) {
            // thread u fetches words u (and u + T) of the tile's block of 16 x NG scales
            const int f = (int)threadIdx.x + j * T;
            scv[slot][j] = __builtin_amdgcn_raw_buffer_load_b32(sres, (f < 16 * NG ? f * 4 : kOutOfRange) + sbase, 0, 0);
        }
    };
    // One K step of a tile's weights: 16 bytes per lane.
    auto issue_weight_step = [&](int slot, int i, int tile) {
        asm volatile("" : "+s"(tile));
        const int step_base = i < ns ? tile * tile_w_bytes + i * (kStepK / 2) : kOutOfRange;  // wave-uniform
        wq[slot][i] = __builtin_amdgcn_raw_buffer_load_b128(wres, woff + step_base, 0, 0);
    };
    auto issue_chan_scale = [&](int slot, int tile) {
        asm volatile("" : "+s"(tile));
        // channel scale of this thread's output column (no channel scales at all: an empty descriptor, reads 0)
        if constexpr (INT_SCALE) cs[slot] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(cres, cs_off + tile * 64, 0, 0));
    };
    auto issue_weights = [&](int slot, int tile) {
#pragma unroll
        for (int i = 0; i < XS; ++i) issue_weight_step(slot, i, tile);
        issue_chan_scale(slot, tile);
    };
    // ---- role of this thread in the epilogue: outputs (m_out[o], tile*16 + n_out) of every tile
    int m_out[OPT];
    float sa_out[OPT];
    bool writer[OPT];
#pragma unroll
    for (int o = 0; o < OPT; ++o) {
        m_out[o] = (threadIdx.x + o * T) >> 4;  // 0 .. 16*MT-1 for the threads that take part
        writer[o] = threadIdx.x + o * T < 256 * MT && m_out[o] < a.M;
        if constexpr (FUSEQ) sa_out[o] = 0.0f;  // known once the token's absmax is
        else sa_out[o] = writer[o] ? a.a_scale[m_out[o]] : 0.0f;
    }

    // Loads come back in the order they were issued.  With several tiles in flight per wave, whatever is requested
    // after the stream's first requests arrives after all of them: the token scales above and, below, the
    // activations go out first where the window is deep (DT >= 2), so that the first tile is multiplied and written
    // while the others are still on their way.  (They are a few requests per lane; with one tile in flight, and the
    // long activation slices that go with it, the stream starts first instead.)
    constexpr bool kStageX = WAVES == 8 && MT == 4;
    constexpr bool kXFirst = DT >= 2 && !kStageX && !FUSEQ && !XLDS;
    // fused quantiser: lane l takes k = 2l, 2l+1 of every step of its wave's K slice (two fp16 values, one word)
    [[maybe_unused]] int xh[XS];
    if constexpr (FUSEQ) {
#pragma unroll
        for (int i = 0; i < XS; ++i)
            xh[i] = __builtin_amdgcn_raw_buffer_load_b32(xres, i < ns ? ((s0 + i) * kStepK + 2 * lane) * 2 : kOutOfRange, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    // operands from LDS, quantised token in: the same two values per lane and step, as codes (one 16-bit word)
    [[maybe_unused]] int xb[XLDS && !FUSEQ ? XS : 1];
    if constexpr (XLDS && !FUSEQ) {
#pragma unroll
        for (int i = 0; i < XS; ++i)
            xb[i] = __builtin_amdgcn_raw_buffer_load_b16(xres, i < ns ? (s0 + i) * kStepK + 2 * lane : kOutOfRange, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    [[maybe_unused]] v4i xr0[kXFirst ? XS : 1][kXFirst ? MT : 1], xr1[kXFirst ? XS : 1][kXFirst ? MT : 1];
    if constexpr (kXFirst) {
#pragma unroll
        for (int i = 0; i < XS; ++i)
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const int m = 16 * t + li;
                const int off = (i < ns && m < a.M) ? m * a.K + (s0 + i) * kStepK + kb * 32 : kOutOfRange;
                xr0[i][t] = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 0, 0);
                xr1[i][t] = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 16, 0);
            }
        __builtin_amdgcn_sched_barrier(0);
    }
    // First requests of the stream go out before anything else that waits on memory (but see above).
#pragma unroll
    for (int u = 0; u < SD; ++u) {
        if (u < my_tiles) issue_scales(u, tile0 + u * G);
        if (u < DT && u < my_tiles) issue_weights(u, tile0 + u * G);
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the compiler from hoisting the activation loads above the stream's

    // ---- activations of this wave's K range, MFMA-ready, loaded once
    v4i x_even[XLDS ? 1 : XS][MT], x_odd[XLDS ? 1 : XS][MT];
    // With 64 token rows a workgroup reads 64 x K bytes of activations, several times its share of the weights, and
    // the operand layout (a lane takes 2 x 16 bytes of one of 16 rows a whole row apart) is a poor way to fetch them:
    // there the wave fetches 16 rows at a time the coalesced way (consecutive lanes, consecutive 16 bytes of a row's
    // XS*128-byte slice) and turns them into the operand layout through a private piece of LDS.  No barrier: LDS
    // serves one wave's requests in order.  Chunk index XOR row keeps both sides off each other's banks.
    [[maybe_unused]] unsigned char* xstage = reinterpret_cast<unsigned char*>(lds_wide + 2 * W) + wave * (XS * 2048);
    // fused quantiser: one absmax word per wave, then per wave the codes of its slice, even k and odd k apart
    [[maybe_unused]] float* lds_amax = reinterpret_cast<float*>(lds_wide + 2 * W);
    [[maybe_unused]] signed char* qstage = reinterpret_cast<signed char*>(lds_amax + W) + wave * (XS * 128);
    [[maybe_unused]] float xf0[XS], xf1[XS];
    if constexpr (FUSEQ) {
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            const float2 f = __half22float2(*reinterpret_cast<const __half2*>(&xh[i]));
            xf0[i] = f.x;
            xf1[i] = f.y;
            amax = fmaxf(amax, fmaxf(fabsf(f.x), fabsf(f.y)));
        }
        amax = wave_max(amax);
        if (lane == 0) lds_amax[wave] = amax;
    }
    constexpr int kChunks = XS * 8;  // 16-byte chunks of a row's slice
    [[maybe_unused]] auto fetch_rows = [&](int t, v4i (&raw)[XS * 2]) {
#pragma unroll
        for (int q = 0; q < XS * 2; ++q) {
            const int e = q * kWave + lane, r = e / kChunks, c = e % kChunks;
            const int m = 16 * t + r;
            const int off = (m < a.M && c < ns * 8) ? m * a.K + s0 * kStepK + c * 16 : kOutOfRange;
            raw[q] = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 0, 0);
        }
    };
    [[maybe_unused]] auto turn_rows = [&](int t, const v4i (&raw)[XS * 2]) {
#pragma unroll
        for (int q = 0; q < XS * 2; ++q) {
            const int e = q * kWave + lane, r = e / kChunks, c = e % kChunks;
            *reinterpret_cast<v4i*>(xstage + r * (XS * 128) + ((c ^ r) << 4)) = raw[q];
        }
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            const v4i x0 = *reinterpret_cast<const v4i*>(xstage + li * (XS * 128) + (((i * 8 + kb * 2) ^ li) << 4));
            const v4i x1 = *reinterpret_cast<const v4i*>(xstage + li * (XS * 128) + (((i * 8 + kb * 2 + 1) ^ li) << 4));
            x_even[i][t][0] = pick_even(x0[0], x0[1]);
            x_even[i][t][1] = pick_even(x0[2], x0[3]);
            x_even[i][t][2] = pick_even(x1[0], x1[1]);
            x_even[i][t][3] = pick_even(x1[2], x1[3]);
            x_odd[i][t][0] = pick_odd(x0[0], x0[1]);
            x_odd[i][t][1] = pick_odd(x0[2], x0[3]);
            x_odd[i][t][2] = pick_odd(x1[0], x1[1]);
            x_odd[i][t][3] = pick_odd(x1[2], x1[3]);
        }
    };
    if constexpr (kStageX) {
        static_assert(!kStageX || kChunks == 32, "the staging swizzle assumes 32 chunks per row slice");
        v4i raw[2][XS * 2];
        fetch_rows(0, raw[0]);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (t + 1 < MT) fetch_rows(t + 1, raw[(t + 1) & 1]);  // the next 16 rows are on their way meanwhile
            turn_rows(t, raw[t & 1]);
        }
    }
#pragma unroll
    for (int i = 0; i < XS; ++i)
#pragma unroll
        for (int t = 0; t < (kStageX || FUSEQ || XLDS ? 0 : MT); ++t) {
            v4i x0, x1;
            if constexpr (kXFirst) {
                x0 = xr0[i][t];
                x1 = xr1[i][t];
            } else {
                const int m = 16 * t + li;
                const int off = (i < ns && m < a.M) ? m * a.K + (s0 + i) * kStepK + kb * 32 : kOutOfRange;
                x0 = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 0, 0);
                x1 = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 16, 0);
            }
            x_even[i][t][0] = pick_even(x0[0], x0[1]);
            x_even[i][t][1] = pick_even(x0[2], x0[3]);
            x_even[i][t][2] = pick_even(x1[0], x1[1]);
            x_even[i][t][3] = pick_even(x1[2], x1[3]);
            x_odd[i][t][0] = pick_odd(x0[0], x0[1]);
            x_odd[i][t][1] = pick_odd(x0[2], x0[3]);
            x_odd[i][t][2] = pick_odd(x1[0], x1[1]);
            x_odd[i][t][3] = pick_odd(x1[2], x1[3]);
        }

    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);  // 2^-alpha_log2, exact

    // ---- role of this thread in staging a tile's group scales: the tile's 16 x NG scales are one contiguous block
    // of the scale tensor; thread u copies word u (and u + T where NG can exceed T / 16) of it.  Word f
    // = (row r, group c) goes to LDS word r * (NG + 1) + c = f + r.
    const float inv_ng = 1.0f / (float)NG, half_inv_ng = 0.5f * inv_ng;

    // LDS word of the group scale of step i for this lane's weight row: scale_row + group_of[i], the latter the same
    // for the whole wave (scalar registers)
    const int scale_row = li * srow_ints + g0;
    int group_of[XS];
    {
        int g = 0, sub = 0;
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            group_of[i] = g;
            if (++sub == p.spg) {
                sub = 0;
                ++g;
            }
        }
    }

    auto stage_scales = [&](int slot, int buf) {
        int f = threadIdx.x;
        asm volatile("" : "+v"(f));  // worked out here every time rather than held in registers throughout
#pragma unroll
        for (int j = 0; j < SJ; ++j, f += T) {
            // r = f / NG for f < 4096, NG <= 224: (f + 0.5) / NG is at least 0.5 / NG away from an integer, far more
            // than the rounding error of the float arithmetic
            const int r = (int)fmaf((float)f, inv_ng, half_inv_ng);
            if (f < 16 * NG) lds_scale[buf * scale_ints + f + r] = scv[slot][j];
        }
        if constexpr (INT_SCALE && kTileFlag) {
            // v_mad_i32_i24 is exact while the scale fits 24 signed bits (|P| <= 2^17 always does); a tile with a
            // wider scale takes full 32-bit multiplies.  Words past the block were fetched as 0.
            bool wide = false;
#pragma unroll
            for (int j = 0; j < SJ; ++j) wide |= ((uint32_t)(scv[slot][j] + (1 << 23)) >> 24) != 0;
            const bool any_wide = __any(wide);
            if (lane == 0) lds_wide[buf * W + wave] = any_wide ? 1 : 0;
        }
    };

    // The pass over this workgroup's tiles.
    {
        stage_scales(0, 0);
        if (SD < my_tiles) issue_scales(0, tile0 + SD * G);
        lds_barrier();
        if constexpr (XLDS && !FUSEQ) {
            // the codes of this wave's K slice, even k and odd k apart, in its own piece of LDS
#pragma unroll
            for (int i = 0; i < XS; ++i) {
                qstage[i * 128 + lane] = (signed char)(xb[i] & 0xFF);
                qstage[i * 128 + 64 + lane] = (signed char)((xb[i] >> 8) & 0xFF);
            }
        }
        if constexpr (FUSEQ) {
            // Appendix A.1, n = 8: s_a = absmax / 127 and codes clamp(rne(x / s_a)), rounded as the true quotient
            // rounds, as in the stand-alone quantiser.  The codes of the wave's slice go through its own piece of LDS into the operand
            // layout.  (Behind the barrier that publishes the first tile's scales: a barrier of its own, earlier, was slower.)
            static_assert(!FUSEQ || (W <= 16 && (W & (W - 1)) == 0), "one absmax word per wave, read by lane & (W - 1)");
            const float amax = wave_max(lds_amax[lane & (W - 1)]);
            const float s_a = amax / 127.0f;
            float xv[2 * XS], qv[2 * XS];
#pragma unroll
            for (int i = 0; i < XS; ++i) {
                xv[2 * i] = xf0[i];
                xv[2 * i + 1] = xf1[i];
            }
            quant_codes<2 * XS>(xv, s_a, qv);
#pragma unroll
            for (int i = 0; i < XS; ++i) {
                qstage[i * 128 + lane] = (signed char)(int)qv[2 * i];
                qstage[i * 128 + 64 + lane] = (signed char)(int)qv[2 * i + 1];
            }
            if constexpr (!XLDS) {
#pragma unroll
                for (int i = 0; i < XS; ++i) {
                    // every lane of a K slice takes the token's codes: operand rows 1..15 then repeat row 0, and their
                    // results are never written (there is one token)
                    x_even[i][0] = *reinterpret_cast<const v4i*>(qstage + i * 128 + kb * 16);
                    x_odd[i][0] = *reinterpret_cast<const v4i*>(qstage + i * 128 + 64 + kb * 16);
                }
            }
#pragma unroll
            for (int o = 0; o < OPT; ++o) sa_out[o] = writer[o] ? s_a : 0.0f;
            if (a.a_scale_out && blockIdx.x == 0 && threadIdx.x == 0) *a.a_scale_out = s_a;
        }

        for (int k = 0; k < my_tiles; k += SD) {
#pragma unroll
            for (int u = 0; u < SD; ++u) {
                if (k + u < my_tiles) {
                    const int dt = u % DT;  // weight slot of this tile
                    const int cur = tile0 + (k + u) * G;
                    // group scales of the next tile go to the other scale buffer (the barrier below publishes them),
                    // and their register slot takes the request for the tile SD after that one
                    if (k + u + 1 < my_tiles) {
                        stage_scales((u + 1) % SD, (k + u + 1) & 1);
                        if (k + u + 1 + SD < my_tiles) issue_scales((u + 1) % SD, cur + (1 + SD) * G);
                    }

                    int my_row = ((k + u) & 1) * scale_ints + scale_row;
                    // opaque to the optimiser: it would otherwise keep the address of every (buffer, step) pair in a
                    // register of its own for the whole kernel, and spill
                    asm volatile("" : "+v"(my_row));
                    const int* my_scales = lds_scale + my_row;
                    const bool refill = k + u + DT < my_tiles;
                    acc_t acc[MT][4];
#pragma unroll
                    for (int t = 0; t < MT; ++t)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[t][j] = 0;

                    // Integer scale step: v_mad_i32_i24 is exact while the scale fits 24 signed bits (|P| <= 2^17
                    // always does); a tile (or step) with a wider scale takes 32-bit multiplies.  Both are exact
                    // modulo 2^32.
                    // operands from LDS: this lane's offset in a step's codes, opaque per tile so that the reads are
                    // not hoisted out of the tile loop and kept in registers for all steps, which is what does not fit
                    [[maybe_unused]] int qbase = kb * 16;
                    if constexpr (XLDS) asm volatile("" : "+v"(qbase));
                    bool wide_tile = false;
                    if constexpr (INT_SCALE && kTileFlag)
                        wide_tile = __any(lds_wide[((k + u) & 1) * W + (lane & (W - 1))] != 0);
#pragma unroll
                    for (int i = 0; i < XS; ++i) {
                        v4i w_even, w_odd;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t pk = (uint32_t)wq[dt][i][q];
                            w_even[q] = (int)((pk << 4) & 0xF0F0F0F0u);
                            w_odd[q] = (int)(pk & 0xF0F0F0F0u);
                        }
                        // With a single weight slot the registers of this step, now used up, take the same step of
                        // the next tile at once, so that the stream never pauses for a whole tile (where registers
                        // are scarce, 16 waves, the longer live ranges would spill: there the slot refills below).
                        if constexpr (kStepRefill) {
                            if (refill) issue_weight_step(dt, i, cur + DT * G);
                        }
                        const int s_i = i < ns ? my_scales[group_of[i]] : 0;
                        const float s_f = __int_as_float(s_i) * 0.0625f;  // 16*P * (s/16) = float(P) * s exactly
                        bool wide = wide_tile;
                        if constexpr (INT_SCALE && !kTileFlag) wide = __any(((uint32_t)(s_i + (1 << 23)) >> 24) != 0);
                        v4i part[MT];
#pragma unroll
                        for (int t = 0; t < MT; ++t) {
                            if constexpr (XLDS) {
                                const v4i xe = *reinterpret_cast<const v4i*>(qstage + qbase + i * 128);
                                const v4i xo = *reinterpret_cast<const v4i*>(qstage + qbase + i * 128 + 64);
                                part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xe, w_even, v4i{0, 0, 0, 0}, 0, 0, 0);
                                part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xo, w_odd, part[t], 0, 0, 0);
                            } else {
                                part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(x_even[i][t], w_even, v4i{0, 0, 0, 0}, 0, 0, 0);
                                part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(x_odd[i][t], w_odd, part[t], 0, 0, 0);
                            }
                        }
                        if constexpr (!INT_SCALE) {
#pragma unroll
                            for (int t = 0; t < MT; ++t)
#pragma unroll
                                for (int j = 0; j < 4; ++j) acc[t][j] = fmaf((float)part[t][j], s_f, acc[t][j]);  // C' += float(C_g) * s_g
                        } else if (__builtin_expect(wide, 0)) {
#pragma unroll
                            for (int t = 0; t < MT; ++t)
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    int prod = (part[t][j] >> 4) * s_i;
                                    asm volatile("" : "+v"(prod));  // else a 64-bit multiply-add with register pairs
                                    acc[t][j] += prod;
                                }
                        } else {
#pragma unroll
                            for (int t = 0; t < MT; ++t)
#pragma unroll
                                for (int j = 0; j < 4; ++j) acc[t][j] += __mul24(part[t][j] >> 4, s_i);          // C'' += C_g * s_g^INT
                        }
                        // The step's scale arithmetic is done here, not later: left alone, the compiler moves it below
                        // the following steps (keeping every step's partial products in registers) and, with many
                        // token tiles, unpacks several steps ahead; both spill.
#pragma unroll
                        for (int t = 0; t < MT; ++t)
#pragma unroll
                            for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(acc[t][j]));
                        if constexpr (MT * XS >= 8) __builtin_amdgcn_sched_barrier(0);
                    }
                    const float c_out = a.chan_scale ? cs[dt] : 1.0f;
                    if (refill) {
                        if constexpr (kStepRefill) issue_chan_scale(dt, cur + DT * G);
                        else issue_weights(dt, cur + DT * G);
                    }

                    // partials of this tile -> LDS buffer (k+dt)&1, slot [wave][t][lane][j]
                    int* buf = lds + ((k + u) & 1) * part_ints;
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        v4i v;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if constexpr (INT_SCALE) v[j] = acc[t][j];
                            else v[j] = __float_as_int(acc[t][j]);
                        }
                        *reinterpret_cast<v4i*>(buf + ((wave * MT + t) * kWave + lane) * 4) = v;
                    }
                    lds_barrier();

                    const int n = cur * 16 + n_out;
#pragma unroll
                    for (int o = 0; o < OPT; ++o) {
                        if (writer[o] && n < a.N) {
                            // where that output sits in a wave's partials: tile t, lane (4 rows per lane-group),
                            // register j (worked out here, per tile, to keep it out of the long-lived registers)
                            int mo = m_out[o];
                            asm volatile("" : "+v"(mo));
                            const int src_slot = ((mo >> 4) * kWave + ((mo & 15) >> 2) * 16 + n_out) * 4 + (mo & 3);
                            acc_t tot = 0;
                            for (int w = 0; w < W; ++w) {
                                const int v = buf[w * MT * kWave * 4 + src_slot];
                                if constexpr (INT_SCALE) tot += v;
                                else tot += __int_as_float(v);
                            }
                            float out_v;
                            if constexpr (INT_SCALE) {
                                out_v = (float)tot * sa_out[o] * (c_out * inv_alpha);
                                if (a.acc_out) a.acc_out[(size_t)m_out[o] * a.N + n] = tot;
                            } else {
                                out_v = tot * sa_out[o];
                            }
                            a.out[(size_t)m_out[o] * a.N + n] = __float2half_rn(out_v);
                        }
                    }
                }
            }
        }
    }

}

template <int MT, int XS, int DT, int WAVES, bool INT_SCALE, bool FUSEQ = false, bool XLDS = false>
hipError_t launch_decode(const GemmArgs& a, const DecodePlan& p, int grid, hipStream_t stream) {
    // partial accumulators, group scales, wide-scale words, activation staging (64 token rows)
    const size_t smem = 2 * (size_t)WAVES * MT * kWave * 16 + 2 * 16 * (size_t)(p.num_groups + 1) * 4 +
                        2 * (size_t)WAVES * 4 +
                        (WAVES == 8 && MT == 4 ? (size_t)WAVES * XS * 2048 : 0) +
                        (FUSEQ || XLDS ? (size_t)WAVES * (4 + XS * 128) : 0);
    auto kern = gemm_decode_kernel<MT, XS, DT, WAVES, INT_SCALE, FUSEQ, XLDS>;
    if (smem > 64 * 1024) {
        static LdsLimit limit;  // per instantiation
        const hipError_t e = limit.raise(reinterpret_cast<const void*>(kern));
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES * kWave), smem, stream, a, p);
    return hipGetLastError();
}

template <bool INT_SCALE>
hipError_t dispatch(const GemmArgs& a, const DecodePlan& p, int mt, int xs, int grid, hipStream_t stream) {
    if (mt == 1 && xs > 6) {  // one token, a long K slice per wave: operands from LDS (quantised or fp16 token)
        if (a.x_fp16) return launch_decode<1, 10, 1, 16, INT_SCALE, true, true>(a, p, grid, stream);
        return launch_decode<1, 10, 1, 16, INT_SCALE, false, true>(a, p, grid, stream);
    }
    if (a.x_fp16) {  // one fp16 token, quantised in the kernel
        if (xs <= 2) return launch_decode<1, 2, 4, 16, INT_SCALE, true>(a, p, grid, stream);
        if (xs <= 4) return launch_decode<1, 4, 2, 16, INT_SCALE, true>(a, p, grid, stream);
        return launch_decode<1, 6, 1, 16, INT_SCALE, true>(a, p, grid, stream);
    }
    if (mt == 1) {
        if (xs <= 2) return launch_decode<1, 2, 4, 16, INT_SCALE>(a, p, grid, stream);
        if (xs <= 4) return launch_decode<1, 4, 2, 16, INT_SCALE>(a, p, grid, stream);
        return launch_decode<1, 6, 1, 16, INT_SCALE>(a, p, grid, stream);
    }
    if (mt == 2) {
        if (p.waves == 16) return launch_decode<2, 2, 4, 16, INT_SCALE>(a, p, grid, stream);
        return launch_decode<2, 8, 1, 8, INT_SCALE>(a, p, grid, stream);
    }
    return launch_decode<4, 4, 1, 8, INT_SCALE>(a, p, grid, stream);
}

}  // namespace

// True (and the launch done) if the decode kernel covers this problem; false leaves it to the general kernel.
bool try_launch_gemm_decode(const GemmArgs& a, bool int_scale, hipStream_t stream, hipError_t* err) {
    if (a.row_offsets || a.M > 64 || a.M < 1) return false;
    if (a.x_fp16 && a.M != 1) return false;
    const int NG = a.K / a.group;
    const int spg = a.group / kStepK;
    const int mt = a.M <= 16 ? 1 : a.M <= 32 ? 2 : 4;
    // A wave's resident activations take 8 registers per token tile and step of its K slice: with 16 waves (128
    // registers each) up to 6 steps for one token tile and 2 for two, with 8 waves (256 registers) 8 steps for two
    // token tiles and 4 for four.
    const int xs16 = ((NG + 15) / 16) * spg;
    const int waves = (mt == 1 || (mt == 2 && xs16 <= 2)) ? 16 : 8;
    if (waves > NG) return false;
    const int xs = ((NG + waves - 1) / waves) * spg;
    // one token: up to 10 steps per wave with the operands in LDS (K up to 20480)
    if (xs > (mt == 1 ? (a.M == 1 ? 10 : 6) : mt == 2 ? (waves == 16 ? 2 : 8) : 4)) return false;
    // (a tile's 16 x NG group scales are staged by the workgroup's threads, ceil(16 XS WAVES / threads) words each:
    // NG <= XS * WAVES / spg by construction)
    DecodePlan p;
    p.tiles = (a.N + 15) / 16;
    p.waves = waves;
    p.num_groups = NG;
    p.gq = NG / waves;
    p.gr = NG % waves;
    p.spg = spg;
    const int grid = p.tiles < cu_count() ? p.tiles : cu_count();
    p.tiles_q = p.tiles / grid;
    p.tiles_r = p.tiles % grid;
    *err = int_scale ? dispatch<true>(a, p, mt, xs, grid, stream) : dispatch<false>(a, p, mt, xs, grid, stream);
    return true;
}

bool try_launch_linear_decode(const GemmArgs& a, bool int_scale, hipStream_t stream, hipError_t* err) {
    if (!a.x_fp16) return false;
    return try_launch_gemm_decode(a, int_scale, stream, err);
}

}  // namespace intscale
