// MFMA-bound regime (many token rows: prefill, and the per-expert slices of a mixture-of-experts layer) of the
// fine-grained W4A8 GEMM.  Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper; float-scale
// form: Eq. (1) / Table 2 "Atom".  The two differ only in the per-group scale step, which is where the paper's
// saving lives: one v_mad_i32_i24 per partial product against a convert plus a multiply-add.
//
// Tiling.  A workgroup of 8 waves (2 x 4) owns 128 token rows x 256 weight rows; a wave owns 64 x 64, as 4 x 4
// sub-tiles of v_mfma_i32_16x16x64_i8 (operand A = 16 token rows, operand B = 16 weight rows, so a lane's 4 results
// share one weight row and with it one group scale).  A wave stays below 256 registers, so two waves share a SIMD
// and one's scale step overlaps the other's matrix work; inside a wave the three stages of a K step (unpack
// sub-tile ns+2, multiply ns+1, scale ns) are software-pipelined for the same reason.  Workgroups are numbered so
// that the ones an XCD runs together form an 8 x 4 block of tiles and share their operand tiles through that XCD's L2.
//
// Operand pipeline.  K advances in steps of 128 through a ring of 4 LDS stages.  The tiles travel from global memory
// straight into LDS (buffer loads with the LDS bit: no staging registers, no vector instructions), three steps
// ahead of their use, so a miss in L2 is covered by two full steps of arithmetic.  Such a load writes lane i's
// 16 bytes at (base + 16 i); the XOR swizzles that keep the later operand reads free of bank conflicts are therefore
// applied to the *global* address each lane fetches.  The loads are issued from inline assembly so that the only
// waits on them are the counted ones written here (the compiler would wait for all of them before any LDS read).
//
// The group scales are transposed to [group][weight row] by a second preparation kernel (which also finds out whether
// every integer scale fits the 24-bit multiplier), so that the 256 scales of a step are one contiguous kilobyte.
//
// Activations are not read in their canonical layout: a preparation kernel writes a copy whose 16-byte chunks hold
// [even k of 0..7 | even k of 8..15 | odd k of 0..7 | odd k of 8..15], the order in which the unpacked weights come
// out (a dot product does not care about the order of its terms as long as both operands agree).
//
// int4 -> int8 with a zero point instead of a sign extension: a packed word is XORed with 0x88888888 (q -> q + 8),
// then a byte is unpacked with one AND (even k) or a shift and an AND (odd k), and the product sum comes out as
// P + 8 * sum_k x[m,k].  The correction -8 * sum_k x[m,k] per (token row, K step) is computed once by the
// preparation kernel and enters each MFMA chain as its initial accumulator, so the chain returns P exactly and the
// scale step costs one instruction per element.
#include "act_common.h"
#include "tile_common.h"

namespace intscale {
namespace {

constexpr int kStepK = 128;
constexpr int kBM = kTileRows;
constexpr int kBN = 256;
constexpr int kThreads = 512;
constexpr int kXcds = 8;    // workgroup i is dispatched to XCD i % 8
constexpr int kGroupM = 8;  // tile rows of the block of tiles an XCD works on at a time
constexpr int kStages = 4;  // LDS ring; tiles are requested kStages - 1 steps ahead
constexpr int kTileLoads = 4;  // buffer-to-LDS loads per wave and step: 2 activation, 2 weight (+1 on waves 0 and 1)
constexpr int kXBytes = kBM * 128, kWBytes = kBN * 64, kAuxBytes = 2048;  // aux: 256 scales, 128 corrections
constexpr int kStageBytes = kXBytes + kWBytes + kAuxBytes;
constexpr int kSwzA = 1;  // activation rows (128 B): 16-byte chunk index ^= (row >> kSwzA) & 7
constexpr int kSwzB = 1;  // weight rows (64 B): 16-byte chunk index ^= (row >> kSwzB) & 3

__device__ __forceinline__ int pick_even(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u); }
__device__ __forceinline__ int pick_odd(uint32_t lo, uint32_t hi) { return (int)__builtin_amdgcn_perm(hi, lo, 0x07050301u); }

// Preparation, one workgroup per token row: xp = the activations with every 16-byte chunk reordered to
// [even | even | odd | odd] (see the top of the file), and s8[step][m] = -8 * sum over the 128 k of the step of
// xq[m,k], the zero-point correction of the q + 8 weight bytes (8 lanes share a step).
__global__ __launch_bounds__(256) void prepare_activations_kernel(const int8_t* __restrict__ xq, int M, int K,
                                                                  int8_t* __restrict__ xp, int32_t* __restrict__ s8,
                                                                  int32_t* __restrict__ wide_flag,
                                                                  const int32_t* __restrict__ row_offsets,
                                                                  int num_experts, int2* __restrict__ tile_table) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *wide_flag = 0;  // prepare_scales_kernel, next in the stream, may set it
    // Grouped form: the list of (expert, row tile) pairs that exist, one per slot, the rest marked empty.  The sum
    // over experts of ceil(rows / 128) is at most ceil(M / 128) + num_experts, the number of slots the tile kernel is
    // launched with; without the list it would need ceil(M / 128) row tiles per expert, nearly all of them empty.
    if (row_offsets != nullptr && blockIdx.x == gridDim.x - 1 && threadIdx.x == 255) {
        const int slots = tile_slots(M, num_experts);
        int slot = 0;
        for (int e = 0; e < num_experts; ++e) {
            const int rows = row_offsets[e + 1] - row_offsets[e];
            for (int t = 0; t * kBM < rows && slot < slots; ++t) tile_table[slot++] = make_int2(e, t);
        }
        for (; slot < slots; ++slot) tile_table[slot] = make_int2(-1, 0);
    }
    const int m = blockIdx.x;
    const int lane = threadIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(xq + (size_t)m * K);
    uint4* prow = reinterpret_cast<uint4*>(xp + (size_t)m * K);
    const int nchunk = K >> 4;
    for (int c0 = 0; c0 < nchunk; c0 += 256) {
        const int c = c0 + lane;
        int sum = 0;
        if (c < nchunk) {
            const uint4 v = row[c];
            sum = __builtin_amdgcn_sdot4((int)v.x, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)v.y, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)v.z, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)v.w, 0x01010101, sum, false);
            uint4 p;
            p.x = (uint32_t)pick_even(v.x, v.y);
            p.y = (uint32_t)pick_even(v.z, v.w);
            p.z = (uint32_t)pick_odd(v.x, v.y);
            p.w = (uint32_t)pick_odd(v.z, v.w);
            prow[c] = p;
        }
        sum += __shfl_xor(sum, 1, kWave);
        sum += __shfl_xor(sum, 2, kWave);
        sum += __shfl_xor(sum, 4, kWave);
        if ((lane & 7) == 0 && c < nchunk) s8[(size_t)(c >> 3) * M + m] = -8 * sum;
    }
}

// The same preparation straight from fp16 activations (the linear call): the per-token quantiser of Appendix A.1 and
// the preparation in one pass, a workgroup per token row, the row held in registers (CH chunks of 16 values per lane)
// between the absmax and the rounding.  Saves writing the canonical codes and reading them back.  (A wave per row, as
// in the preparation above, keeps four times the registers per lane and was slower.)
template <int CH>
__global__ __launch_bounds__(256) void quantize_prepare_activations_kernel(const __half* __restrict__ x, int M, int K,
                                                                           int8_t* __restrict__ xp,
                                                                           int32_t* __restrict__ s8,
                                                                           float* __restrict__ a_scale,
                                                                           int32_t* __restrict__ wide_flag) {
    __shared__ float red[4];
    if (blockIdx.x == 0 && threadIdx.x == 0) *wide_flag = 0;
    constexpr int kLanes = 256;  // lanes per token row
    const int m = blockIdx.x;
    const int lane = threadIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(x + (size_t)m * K);  // 8 fp16 values each
    uint4* prow = reinterpret_cast<uint4*>(xp + (size_t)m * K);
    const int nchunk = K >> 4;
    uint4 v[CH][2];
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = lane + j * kLanes;
        v[j][0] = c < nchunk ? row[2 * c] : make_uint4(0u, 0u, 0u, 0u);
        v[j][1] = c < nchunk ? row[2 * c + 1] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int j = 0; j < CH; ++j) amax = fmaxf(amax, fmaxf(absmax8(v[j][0]), absmax8(v[j][1])));
    amax = block_max<4>(amax, red);
    const float s = amax / 127.0f;
    if (lane == 0) a_scale[m] = s;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = lane + j * kLanes;
        int sum = 0;
        if (c < nchunk) {
            const uint2 lo = quantize8(v[j][0], s), hi = quantize8(v[j][1], s);  // the canonical 16 codes, in k order
            sum = __builtin_amdgcn_sdot4((int)lo.x, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)lo.y, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)hi.x, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4((int)hi.y, 0x01010101, sum, false);
            uint4 p;
            p.x = (uint32_t)pick_even(lo.x, lo.y);
            p.y = (uint32_t)pick_even(hi.x, hi.y);
            p.z = (uint32_t)pick_odd(lo.x, lo.y);
            p.w = (uint32_t)pick_odd(hi.x, hi.y);
            prow[c] = p;
        }
        sum += __shfl_xor(sum, 1, kWave);
        sum += __shfl_xor(sum, 2, kWave);
        sum += __shfl_xor(sum, 4, kWave);
        if ((lane & 7) == 0 && c < nchunk) s8[(size_t)(c >> 3) * M + m] = -8 * sum;
    }
}

// One output tile.  WIDE selects the integer scale step: false = v_mad_i32_i24 (exact while every scale fits 24
// bits), true = full 32-bit multiplies (exact modulo 2^32 for any scale).  `scale_t` are the transposed scales.
// COARSE is the coarse-grained GEMM (one group spanning all of K; Table 2, first column): the partial products stay in
// the MFMA accumulators from the first K step to the last, nothing but unpacking is left for the vector ALU, and the
// one scale per weight row is applied in the epilogue.  Its zero-point correction is the sum over all K steps, which a
// third preparation kernel leaves in the slot of step 0; it enters as the initial value of the accumulators.
template <bool INT_SCALE, bool WIDE, bool COARSE = false>
__device__ __forceinline__ void gemm_prefill_tile(const GemmArgs& a, const int8_t* __restrict__ xp,
                                                  const int32_t* __restrict__ s8, const int32_t* __restrict__ scale_t,
                                                  const int2* __restrict__ tile_table, unsigned char* smem) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave >> 2, wn = wave & 3;

    // ---- which tile.  Linear tile numbers are dealt out so that XCD x (workgroups x, x+8, ...) gets one contiguous
    // range of them, and a range walks the output in blocks of kGroupM tile rows, column by column.
    const int tiles_n = (a.N + kBN - 1) / kBN;
    const int tiles_m = a.row_offsets ? tile_slots(a.M, a.num_experts) : (a.M + kBM - 1) / kBM;  // grouped: slots
    int tile_m, tile_n;
    if (a.row_offsets) {
        // Grouped form: the slots that exist come first and how many there are is known on the device only, so the
        // tiles are simply taken in order, slot by slot: workgroup i runs on XCD i % 8, every XCD gets every eighth
        // tile (equal shares of the real work, to within one tile), and the two row tiles of an expert with more than
        // 128 rows meet on the same XCD for the same tile column whenever the number of tile columns divides by 8.
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
        const int2 entry = tile_table[tile_m];  // which expert and which of its row tiles this slot stands for
        if (entry.x < 0) return;                // an empty slot (uniform over the workgroup, before any barrier)
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
    const int row_bytes = a.K >> 1;

    // ---- loader roles: per step a wave requests two 1 KB blocks of the activation tile (8 rows each) and two of the
    // weight tile (16 rows each).  Rows past the end of a tensor lie outside its descriptor and read as zero.  A
    // lane's LDS slot is fixed by the load; the swizzle picks the global chunk that belongs there.
    const v4i xdesc = make_desc(xp + (size_t)m0 * a.K, (size_t)m_rows * a.K);
    const v4i wdesc = make_desc(a.qweight + (expert * (size_t)a.N + n0) * row_bytes, (size_t)n_rows * row_bytes);
    // wave 0 also fetches the step's 256 scales (1 KB of the transposed copy), wave 1 its 128 corrections
    v4i adesc = make_desc(nullptr, 0);
    int aux_voff = lane * 16, aux_inc = 0, grp_inc = 0;  // advance of aux_soff per K step / per finished group
    if (wave == 0) {
        adesc = make_desc(scale_t + (expert * NG) * (size_t)a.N + n0, ((size_t)(NG - 1) * a.N + n_rows) * 4);
        grp_inc = a.N * 4;
    } else if (wave == 1) {
        adesc = make_desc(s8 + m0, ((size_t)(steps - 1) * a.M + m_rows) * 4);
        if (lane >= 32) aux_voff = (int)0x80000000u;  // 128 rows = 32 lanes; the rest reads nothing
        aux_inc = a.M * 4;
    }
    int x_voff[2], w_voff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int xr = 8 * (wave + 8 * i) + (lane >> 3);
        x_voff[i] = xr * a.K + (((lane & 7) ^ ((xr >> kSwzA) & 7)) << 4);
        const int wr = 16 * (wave + 8 * i) + (lane >> 2);
        w_voff[i] = wr * row_bytes + (((lane & 3) ^ ((wr >> kSwzB) & 3)) << 4);
    }
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;  // LDS byte offset
    // Request state, all scalar and advanced by additions: the stage's LDS base, the step's offsets into the two
    // tensors, the scale / correction offset.  Steps past the last one request nothing.
    const unsigned lds_x0 = wave * 1024, lds_x1 = lds_x0 + 8192, lds_w0 = kXBytes + lds_x0, lds_w1 = kXBytes + lds_x1;
    const unsigned lds_aux = kXBytes + kWBytes + wave * 1024;
    unsigned rq_base = lds0;
    int rq_x = 0, rq_w = 0, aux_soff = 0;
    int ld_sub = 0;  // K steps already requested of the current group (steps are requested in order)
    auto request_step = [&](int t) {
        if (t < steps) {
            load_to_lds_b128(xdesc, rq_base, lds_x0, x_voff[0], rq_x);
            load_to_lds_b128(xdesc, rq_base, lds_x1, x_voff[1], rq_x);
            load_to_lds_b128(wdesc, rq_base, lds_w0, w_voff[0], rq_w);
            load_to_lds_b128(wdesc, rq_base, lds_w1, w_voff[1], rq_w);
            if (wave < 2) load_to_lds_b128(adesc, rq_base, lds_aux, aux_voff, aux_soff);
        }
        rq_x += kStepK;
        rq_w += kStepK / 2;
        rq_base = rq_base + kStageBytes == lds0 + kStages * kStageBytes ? lds0 : rq_base + kStageBytes;
        const bool group_done = ++ld_sub == spg;
        ld_sub = group_done ? 0 : ld_sub;
        aux_soff += aux_inc + (group_done ? grp_inc : 0);
    };

    // ---- consumer roles.  MFMA 16x16x64: lane l feeds token row / weight row (l & 15) and 16 of the 64 k of each
    // half step, chosen by (l >> 4); its 4 results are weight row (l & 15), token rows 4*(l >> 4)..+3.  Lane group
    // lq takes the 32 k of its 16 packed weight bytes: activation chunks 2 lq (first half step) and 2 lq + 1.
    constexpr int MS = 4;  // 16-row token sub-tiles per wave
    constexpr int NS = 4;  // 16-row weight sub-tiles per wave
    const int l16 = lane & 15, lq = lane >> 4;
    int a_off[2];
    {
        const int ar = wm * 64 + l16;  // + 16 ms: the swizzle bits used are below 16 for kSwzA <= 1
        a_off[0] = ar * 128 + (((2 * lq) ^ ((ar >> kSwzA) & 7)) << 4);
        a_off[1] = ar * 128 + (((2 * lq + 1) ^ ((ar >> kSwzA) & 7)) << 4);
    }
    const int br = wn * 64 + l16;
    const int b_off = kXBytes + br * 64 + ((lq ^ ((br >> kSwzB) & 3)) << 4);
    const int sc_off = kXBytes + kWBytes + (wn * 64 + l16) * 4;
    const int ci_off = kXBytes + kWBytes + 1024 + (wm * 64 + 4 * lq) * 4;

    using acc4 = typename std::conditional<INT_SCALE, v4i, v4f>::type;
    acc4 acc[MS][NS];
    [[maybe_unused]] v4i chain[MS][NS];  // COARSE: the unscaled integer sums, carried from step to step by the MFMAs
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int ns = 0; ns < NS; ++ns)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                acc[ms][ns][r] = 0;
                if constexpr (COARSE) chain[ms][ns][r] = 0;
            }

    // Operand registers of one K step.  Two sets alternate: while step s is multiplied out of one, the other is
    // filled from the LDS stage of step s+1, so that no step starts by waiting for LDS.
    struct Operands {
        v4i af[MS][2];  // activation fragments
        v4i cinit[MS];  // initial accumulators: -8 * sum_k x[m,k] for this lane's 4 token rows
        v4i braw[NS];   // packed weight fragments
        int scl[NS];    // group scales
    };
    auto read_fragments = [&](Operands& o, const unsigned char* st) {
#pragma unroll
        for (int ns = 0; ns < 2; ++ns) o.braw[ns] = *reinterpret_cast<const v4i*>(st + b_off + ns * 1024);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) o.af[ms][kk] = *reinterpret_cast<const v4i*>(st + ms * 2048 + a_off[kk]);
#pragma unroll
        for (int ns = 2; ns < NS; ++ns) o.braw[ns] = *reinterpret_cast<const v4i*>(st + b_off + ns * 1024);
    };
    auto read_corrections = [&](Operands& o, const unsigned char* st) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) o.cinit[ms] = *reinterpret_cast<const v4i*>(st + ci_off + ms * 64);
#pragma unroll
        for (int ns = 0; ns < NS; ++ns) o.scl[ns] = *reinterpret_cast<const int*>(st + sc_off + ns * 64);
    };
    // The wait that makes step t's tile visible: this wave's requests up to step t have landed once only those of the
    // two steps after it are outstanding (waves 0 and 1 issue one more per step; near the end fewer steps are in
    // flight and the wait is for all of them), its own LDS reads are done, and past the barrier the same holds for
    // every wave.
    auto wait_tile_and_sync = [&](bool full_flight) {
        if (!full_flight) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");  // the last steps
        else if (wave < 2) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * (kTileLoads + 1)) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * kTileLoads) : "memory");
    };

    // One K step: cur holds step s, nxt receives step s+1.  The three phases of weight sub-tile ns -- unpack,
    // multiply, scale -- are issued as unpack(ns+2), multiply(ns+1), scale(ns), so that the matrix pipe and the
    // vector ALU work together.  Half way, the barrier that publishes step s+1 (everybody has then also finished
    // reading step s out of LDS, whose stage is handed to step s+4), then the reads for nxt as its registers or
    // their predecessors' fall free.
    auto compute_step = [&](Operands& cur, Operands& nxt, int s) {
        v4i bfu[2][2], part[2][MS];
        auto unpack = [&](int ns) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                // q -> q + 8 flips the top bit of a nibble; XOR and mask fuse into one three-input bit operation
                const uint32_t p0 = (uint32_t)cur.braw[ns][2 * kk], p1 = (uint32_t)cur.braw[ns][2 * kk + 1];
                bfu[ns & 1][kk][0] = (int)((p0 ^ 0x08080808u) & 0x0F0F0F0Fu);
                bfu[ns & 1][kk][1] = (int)((p1 ^ 0x08080808u) & 0x0F0F0F0Fu);
                bfu[ns & 1][kk][2] = (int)(((p0 >> 4) ^ 0x08080808u) & 0x0F0F0F0Fu);
                bfu[ns & 1][kk][3] = (int)(((p1 >> 4) ^ 0x08080808u) & 0x0F0F0F0Fu);
            }
        };
        auto multiply = [&](int ns) {
            if constexpr (COARSE) {
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    chain[ms][ns] =
                        __builtin_amdgcn_mfma_i32_16x16x64_i8(cur.af[ms][0], bfu[ns & 1][0], chain[ms][ns], 0, 0, 0);
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    chain[ms][ns] =
                        __builtin_amdgcn_mfma_i32_16x16x64_i8(cur.af[ms][1], bfu[ns & 1][1], chain[ms][ns], 0, 0, 0);
                return;
            }
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                part[ns & 1][ms] =
                    __builtin_amdgcn_mfma_i32_16x16x64_i8(cur.af[ms][0], bfu[ns & 1][0], cur.cinit[ms], 0, 0, 0);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                part[ns & 1][ms] =
                    __builtin_amdgcn_mfma_i32_16x16x64_i8(cur.af[ms][1], bfu[ns & 1][1], part[ns & 1][ms], 0, 0, 0);
        };
        auto scale = [&](int ns) {  // per-group scale step of Table 2
            if constexpr (COARSE) return;  // one group: its scale waits for the epilogue
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
        unpack(0);
        multiply(0);
        unpack(1);
#pragma unroll
        for (int ns = 0; ns < NS; ++ns) {
            if (ns == 2) {
                wait_tile_and_sync(s + kStages - 1 < steps);  // steps s+2 and s+3 were both requested
                request_step(s + kStages);
                read_fragments(nxt, next_stage);
            }
            if (ns == 3) read_corrections(nxt, next_stage);
            if (ns + 1 < NS) multiply(ns + 1);
            if (ns + 2 < NS) unpack(ns + 2);
            scale(ns);
        }
        // keep the accumulators whole between steps: regrouped sums over two steps (two multiplies and a 3-input add)
        // cost more instructions than two multiply-adds
        if constexpr (!COARSE)
            asm volatile(""
                         : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[0][2]), "+v"(acc[0][3]), "+v"(acc[1][0]),
                           "+v"(acc[1][1]), "+v"(acc[1][2]), "+v"(acc[1][3]), "+v"(acc[2][0]), "+v"(acc[2][1]),
                           "+v"(acc[2][2]), "+v"(acc[2][3]), "+v"(acc[3][0]), "+v"(acc[3][1]), "+v"(acc[3][2]),
                           "+v"(acc[3][3]));
    };

    Operands ops0, ops1;
#pragma unroll
    for (int t = 0; t < kStages; ++t) request_step(t);
    if (steps < kStages) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    else if (wave < 2) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(3 * (kTileLoads + 1)) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(3 * kTileLoads) : "memory");
    if (wm * 64 >= m_rows) {
        // None of this wave's 64 token rows exists (the tile at the ragged end of the rows, typically the second tile
        // of a mixture-of-experts expert): it keeps up its share of the requests and the barriers, and leaves the
        // SIMD's issue slots to the wave that has rows.
        for (int s = 0; s < steps; ++s) {
            wait_tile_and_sync(s + kStages - 1 < steps);
            request_step(s + kStages);
        }
    } else {
        read_fragments(ops0, smem);
        read_corrections(ops0, smem);
        if constexpr (COARSE) {  // the slot of step 0 holds the correction of the whole row
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int ns = 0; ns < NS; ++ns) chain[ms][ns] = ops0.cinit[ms];
        }
        for (int s = 0; s < steps; s += 2) {
            compute_step(ops0, ops1, s);
            if (s + 1 < steps) compute_step(ops1, ops0, s + 1);  // uniform over the workgroup (it holds a barrier)
        }
    }

    // ---- epilogue, once per output: FLOAT(acc) * s_a[m] * c[n] / alpha (Eq. (2)), or facc * s_a[m] (Eq. (1))
    // all requests have landed (the emptied tail ones still write zeros) and nobody reads operand tiles any more
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
    // Rows of 8-aligned length go through an fp16 copy of the tile in LDS and leave as 16-byte stores, 512
    // contiguous bytes per token row; otherwise (and for the diagnostic accumulator output) element by element.
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
        [[maybe_unused]] int row_scale = 0;  // COARSE: the one scale of weight row n
        if constexpr (COARSE) row_scale = scale_t[expert * (size_t)a.N + n];
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int ml = wm * 64 + ms * 16 + 4 * lq + r;
                __half h;
                [[maybe_unused]] int acc_i = 0;
                if constexpr (COARSE) {
                    if constexpr (INT_SCALE) {
                        acc_i = chain[ms][ns][r] * row_scale;  // wraps modulo 2^32 like the grouped sum
                        h = __float2half_rn((float)acc_i * sa[ms][r] * c);
                    } else {
                        h = __float2half_rn((float)chain[ms][ns][r] * __int_as_float(row_scale) * sa[ms][r]);
                    }
                } else if constexpr (INT_SCALE) {
                    acc_i = acc[ms][ns][r];
                    h = __float2half_rn((float)acc_i * sa[ms][r] * c);
                } else {
                    h = __float2half_rn(acc[ms][ns][r] * sa[ms][r]);
                }
                if (staged) {
                    otile[ml * kPitch + nl] = h;
                } else if (ml < m_rows) {
                    const size_t o = (size_t)(m0 + ml) * a.N + n;
                    if constexpr (INT_SCALE) {
                        if (a.acc_out) a.acc_out[o] = acc_i;
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

// Coarse-grained form only: the correction of a whole token row, the sum of its per-step corrections, replaces the
// one of step 0.
__global__ __launch_bounds__(256) void sum_row_corrections_kernel(int32_t* __restrict__ s8, int steps, int M) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= M) return;
    int total = 0;
    for (int t = 0; t < steps; ++t) total += s8[(size_t)t * M + m];
    s8[m] = total;
}

// INT_SCALE: Eq. (2) with the scale step chosen by the flag the scale preparation left; else Eq. (1).  COARSE: one
// group over all of K.
template <bool INT_SCALE, bool COARSE>
__global__ __launch_bounds__(kThreads) void gemm_prefill_kernel(GemmArgs a, const int8_t* __restrict__ xp,
                                                                const int32_t* __restrict__ s8,
                                                                const int32_t* __restrict__ scale_t,
                                                                const int32_t* __restrict__ wide_flag,
                                                                const int2* __restrict__ tile_table) {
    extern __shared__ __align__(16) unsigned char smem[];  // [kStages][activations 16 KB | weights 16 KB | aux 2 KB]
    if constexpr (COARSE) {
        gemm_prefill_tile<INT_SCALE, false, true>(a, xp, s8, scale_t, tile_table, smem);
    } else if constexpr (INT_SCALE) {
        if (*wide_flag != 0) gemm_prefill_tile<true, true>(a, xp, s8, scale_t, tile_table, smem);
        else gemm_prefill_tile<true, false>(a, xp, s8, scale_t, tile_table, smem);
    } else {
        gemm_prefill_tile<false, false>(a, xp, s8, scale_t, tile_table, smem);
    }
}

template <bool INT_SCALE, bool COARSE>
hipError_t launch_tile(const GemmArgs& a, const int8_t* xp, const int32_t* s8, const int32_t* scale_t,
                       const int32_t* flag, const int2* tile_table, hipStream_t stream) {
    const size_t smem = (size_t)kStages * kStageBytes;
    const int tiles_m = a.row_offsets ? tile_slots(a.M, a.num_experts) : (a.M + kBM - 1) / kBM;
    const int tiles = ((a.N + kBN - 1) / kBN) * tiles_m;
    static LdsLimit limit;  // per instantiation
    const hipError_t e = limit.raise(reinterpret_cast<const void*>(gemm_prefill_kernel<INT_SCALE, COARSE>));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_prefill_kernel<INT_SCALE, COARSE>), dim3(tiles), dim3(kThreads), smem, stream, a, xp, s8,
                       scale_t, flag, tile_table);
    return hipGetLastError();
}

// the workspace starts with the wide-scale flag (16 bytes), then the table of row-tile slots
size_t header_bytes(int experts, int M) { return pad256(16 + (size_t)tile_slots(M, experts) * sizeof(int2)); }
size_t corrections_bytes(int M, int K) { return pad256((size_t)(K / kStepK) * (size_t)M * 4); }
size_t scales_bytes(int experts, int N, int K, int group) { return pad256((size_t)experts * N * (K / group) * 4); }

}  // namespace

// workspace = [flag and row-tile slots, padded to 256 B | s8: K/128 x M words | transposed scales: experts x K/group x
//              N words | reordered activations: M x K bytes]
size_t gemm_prefill_workspace_bytes(int num_experts, int M, int N, int K, int group) {
    return header_bytes(num_experts, M) + corrections_bytes(M, K) + scales_bytes(num_experts, N, K, group) + (size_t)M * K;
}

// rows the fused quantiser + preparation holds in registers: 8 chunks of 16 values per lane, 256 lanes
bool gemm_prefill_takes_fp16(int K) { return (K & 15) == 0 && (K >> 4) <= 8 * 256; }

hipError_t launch_gemm_prefill(const GemmArgs& a, bool int_scale, void* workspace, hipStream_t stream) {
    const int experts = a.row_offsets ? a.num_experts : 1;
    const int NG = a.K / a.group;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const size_t header = header_bytes(experts, a.M);
    int32_t* flag = reinterpret_cast<int32_t*>(ws);
    int2* tile_table = reinterpret_cast<int2*>(ws + 16);
    int32_t* s8 = reinterpret_cast<int32_t*>(ws + header);
    int32_t* scale_t = reinterpret_cast<int32_t*>(ws + header + corrections_bytes(a.M, a.K));
    int8_t* xp = reinterpret_cast<int8_t*>(ws + header + corrections_bytes(a.M, a.K) +
                                           scales_bytes(experts, a.N, a.K, a.group));
    if (a.x_fp16) {  // fp16 activations (plain form only): quantised on the way, the token scales go to a.a_scale_out
        const int nchunk = a.K >> 4;
#define QP_LAUNCH(CH, GRID) \
    hipLaunchKernelGGL(quantize_prepare_activations_kernel<CH>, dim3(GRID), dim3(256), 0, stream, a.x_fp16, a.M, a.K, xp, \
                       s8, a.a_scale_out, flag)
        if (nchunk <= 256) QP_LAUNCH(1, a.M);
        else if (nchunk <= 2 * 256) QP_LAUNCH(2, a.M);
        else if (nchunk <= 4 * 256) QP_LAUNCH(4, a.M);
        else QP_LAUNCH(8, a.M);
#undef QP_LAUNCH
    } else {
        hipLaunchKernelGGL(prepare_activations_kernel, dim3(a.M), dim3(256), 0, stream, a.xq, a.M, a.K, xp, s8,
                           flag, a.row_offsets, experts, tile_table);
    }
    const dim3 sgrid((a.N + 63) / 64, (NG + 63) / 64, experts);
    const int32_t* scale = static_cast<const int32_t*>(a.scale);
    if (int_scale) hipLaunchKernelGGL(prepare_scales_kernel<true>, sgrid, dim3(256), 0, stream, scale, a.N, NG, scale_t, flag);
    else hipLaunchKernelGGL(prepare_scales_kernel<false>, sgrid, dim3(256), 0, stream, scale, a.N, NG, scale_t, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.group == a.K && a.K > kStepK) {  // coarse-grained: one group over several K steps
        hipLaunchKernelGGL(sum_row_corrections_kernel, dim3((a.M + 255) / 256), dim3(256), 0, stream, s8, a.K / kStepK, a.M);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        return int_scale ? launch_tile<true, true>(a, xp, s8, scale_t, flag, tile_table, stream)
                         : launch_tile<false, true>(a, xp, s8, scale_t, flag, tile_table, stream);
    }
    return int_scale ? launch_tile<true, false>(a, xp, s8, scale_t, flag, tile_table, stream)
                     : launch_tile<false, false>(a, xp, s8, scale_t, flag, tile_table, stream);
}

}  // namespace intscale
