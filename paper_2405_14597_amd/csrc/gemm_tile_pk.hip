// MFMA-bound regime (more than 64 token rows: prefill) of the fine-grained W4A8 GEMM on prepacked weights.
// Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale paper; float-scale form: Eq. (1) / Table 2 "Atom".
// The two differ only in the per-group scale step, where the paper's saving lives: one v_mad_i32_i24 per partial
// product against a convert plus a multiply-add.
//
// What bounds this regime on gfx950.  A v_mfma_i32_16x16x64_i8 keeps the matrix pipe busy for 16 cycles, and an
// ordinary vector instruction costs the SIMD's issue port about 4; Eq. (2)'s scale step alone is 2 of those per MFMA
// at group size 128 (Eq. (1)'s is 4), so every further vector instruction per MFMA comes straight off the matrix
// pipe's share.  The int4 -> int8 unpacking is the largest such cost, and it is paid per wave and K step for the
// wave's weight rows whatever the number of token rows it multiplies them with; so a wave here owns 128 token rows x
// 64 weight rows (8 x 4 MFMA sub-tiles): 0.75 unpack instructions per MFMA, half of what a 64 x 64 wave tile pays.
//
// Tiling.  A workgroup is 4 waves (1 x 4) on 128 token rows x 256 weight rows, one wave per SIMD, 256 registers per
// wave; two workgroups share a CU (their 67 KB of LDS each allow it), so every SIMD holds two waves of DIFFERENT
// workgroups: they meet no common barrier, drift apart by themselves, and one's unpacking and LDS waits fall under the
// other's MFMAs.  (A SIMD issues one instruction at a time over all its waves, so the second wave adds about a fifth,
// not a factor of two: a workgroup alone on a CU runs at 1.7 times the rate of one that shares it.)
//
// Rounds.  The chip works on 2 x CUs tiles at a time.  When the tiles left for the last round are fewer than half the
// CUs their K range is cut into parts, one workgroup each, and the last part of a tile to arrive adds the partial
// tiles up (TileSplit below).  The mixture-of-experts form runs the same tile code on row tiles listed per expert
// (TileGroups), in four instances for tiles of up to 16, 32, 64 and 128 token rows: a wave's instructions per K step
// are a fixed share plus a share per 16 token rows, and an expert's last tile is often a dozen rows.
//
// Operand pipeline.  K advances in steps of 128 (one MFMA pair) through two LDS stages.  Both operands come in
// layouts that are already the order the MFMA lanes want (weights: the prepacked 1 KB blocks of pk_common.h;
// activations: 2 KB blocks of 16 token rows x 128 k written by the preparation kernel below), so they travel from
// global memory straight into LDS (buffer loads with the LDS bit: no staging registers, no address arithmetic per
// lane beyond one offset) and every LDS read of a wave is one contiguous kilobyte: no bank conflicts, no swizzle.
// The group scales of the step's 256 weight rows and the zero-point corrections of its 128 token rows ride along.
//
// int4 -> int8 with a zero point: a packed word XOR 0x08.. AND 0x0F.. is q + 8 for the low nibbles (one three-input
// bit operation), the high nibbles take a shift more; the product sum comes out as P + 8 * sum_k x[m,k], and the
// correction -8 * sum_k x[m,k] per (token row, K step), computed once by the preparation kernel, enters each MFMA
// chain as its initial accumulator, so the chain returns P exactly and the scale step costs one instruction per element.
#include <stdio.h>

#include <algorithm>
#include <stdlib.h>

#include "act_common.h"
#include "pk_common.h"
#include "tile_common.h"

namespace intscale {
namespace {

constexpr int kTM = 128, kTN = 256;     // workgroup tile: token rows x weight rows
constexpr int kTThreads = 256;          // 4 waves, one per SIMD
constexpr int kMS = 8, kNS = 4;         // 16-row sub-tiles per wave: token rows, weight rows
// (the corrections take 512 bytes; their load writes a full kilobyte, the upper half zeros)
constexpr int kBBytes = kTN * 64, kScBytes = kTN * 4, kC0Bytes = 1024;
// One LDS stage of a tile of MS 16-row sub-tiles per wave (MS * 16 token rows): 34816 bytes at 128 rows, 26624 at 64
constexpr int stage_bytes(int MS) { return MS * 16 * 128 + kBBytes + kScBytes + kC0Bytes; }
constexpr int kXcdCount = 8;            // workgroup i is dispatched to XCD i % 8
constexpr int kGroupRows = 8;           // tile rows of the block of tiles an XCD works on at a time

// The last, partial round of tiles.  With two workgroups per compute unit the chip works on `slots` tiles at a time;
// when the tiles % slots left for the last round are fewer than half the compute units, most of the chip would idle
// for a whole tile time.  Their K range is then cut into `parts`, one workgroup each: it stores its accumulators (exact int32, or the float
// partial sums) as a partial tile in the workspace, and the last of a tile's parts to arrive adds them up in part
// order and runs the epilogue (same protocol as the K split of the decode kernel: device-scope stores, one counter
// per tile, which the last arriver sets back to zero).
struct TileSplit {
    int whole;           // tiles computed over all of K by one workgroup: workgroups [0, whole)
    int rem;             // tiles of the last round: workgroup whole + p works on part p / rem of tile whole + p % rem
    int parts;           // K parts per such tile (1: rem = 0)
    int32_t* counters;   // [rem], zero when the kernel starts
    int32_t* partials;   // [rem][parts][kPartWords]
};
// Mixture-of-experts form: token rows sorted by expert, expert e owning rows [row_offsets[e], row_offsets[e+1]) and the
// e-th of num_experts prepacked weight sets.  The preparation kernel pads every expert to whole 16-row tiles (so that no
// operand block mixes experts) and lists the 128-row tiles that exist in a table; a workgroup of the tiled kernel
// takes one table entry and one tile column.
struct TileGroups {
    const int32_t* row_offsets;  // device, [num_experts + 1]
    int num_experts;
    int slots;                   // table entries there is room for: ceil(M/128) + num_experts
    int padded16;                // 16-row tiles there is room for: ceil(M/16) + num_experts
    int32_t* table;              // [0] = entries in use, then 4 words per entry: expert, first 16-row tile, first row, rows
    size_t wstride, sstride;     // bytes from one expert's packed weights / scales to the next
};
constexpr int kPartWords = kTM * kTN;                      // one partial tile of 128 rows: 128 KB
constexpr size_t kCounterBytes = 2048;                     // up to 512 tiles in the last round
constexpr size_t kPartialCap = (size_t)64 << 20;           // at most this much workspace for partial tiles
constexpr int kMinPartSteps = 8;                           // K steps a part has at least

// ---- preparation of the activations: 2 KB blocks [16-row tile][K step] = [MFMA half h][k chunk kb][row r][16 codes],
// the 16 codes of (h, kb) being k = 128 s + 64 h + 16 kb .. + 15 of row 16 mt + r, and the zero-point corrections
// c0[tile][step][r] = -8 * sum over the step's 128 codes.  A wave works on whole blocks of one 16-row tile: lane
// (kb, r) fetches its 16 codes of row r and the wave writes each half block as one contiguous kilobyte; rows past M
// become zeros.
__device__ __forceinline__ int sum16(uint4 v) {
    int sum = __builtin_amdgcn_sdot4((int)v.x, 0x01010101, 0, false);
    sum = __builtin_amdgcn_sdot4((int)v.y, 0x01010101, sum, false);
    sum = __builtin_amdgcn_sdot4((int)v.z, 0x01010101, sum, false);
    return __builtin_amdgcn_sdot4((int)v.w, 0x01010101, sum, false);
}

// One block: the two half blocks of lane (kb, r), and the row's correction through the four kb lanes of the row.
__device__ __forceinline__ void store_block(size_t blk, int lane, uint4 lo, uint4 hi, int8_t* __restrict__ xp,
                                            int32_t* __restrict__ c0) {
    uint4* dst = reinterpret_cast<uint4*>(xp + blk * 2048);
    dst[lane] = lo;
    dst[64 + lane] = hi;
    int sum = sum16(lo) + sum16(hi);
    sum += __shfl_xor(sum, 16, kWave);
    sum += __shfl_xor(sum, 32, kWave);
    if (lane < 16) c0[blk * 16 + lane] = -8 * sum;
}

constexpr int kPrepSteps = 4;  // K steps per wave of the int8 preparation (8 loads of 16 bytes in flight per lane)

// Quantised activations in: grid (16-row tiles, K steps / (4 waves * kPrepSteps)).
__global__ __launch_bounds__(256) void prepare_activations_pk_kernel(const int8_t* __restrict__ xq, int M, int K,
                                                                     int8_t* __restrict__ xp, int32_t* __restrict__ c0,
                                                                     int32_t* __restrict__ counters, int ncounters) {
    if (blockIdx.x == 0 && blockIdx.y == 0)  // the tiled kernel's arrival counters start at zero
        for (int i = threadIdx.x; i < ncounters; i += 256) counters[i] = 0;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r = lane & 15, kb = lane >> 4;
    const int mt = blockIdx.x, m = 16 * mt + r;
    const int steps = K >> 7;
    const int s0 = (blockIdx.y * 4 + wave) * kPrepSteps;
    const int8_t* src = xq + (size_t)min(m, M - 1) * K + kb * 16;
    uint4 v[kPrepSteps][2];
#pragma unroll
    for (int j = 0; j < kPrepSteps; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int st = min(s0 + j, steps - 1);
            v[j][h] = *reinterpret_cast<const uint4*>(src + st * 128 + h * 64);
            if (m >= M) v[j][h] = make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
    for (int j = 0; j < kPrepSteps; ++j)
        if (s0 + j < steps) store_block((size_t)mt * steps + s0 + j, lane, v[j][0], v[j][1], xp, c0);
}

// Mixture-of-experts form of the kernel above: block x is a 16-row tile of the padded row space (the 16-row tiles of
// expert 0, then those of expert 1, ...); the first workgroup also lists the 128-row tiles.
__global__ __launch_bounds__(256) void prepare_activations_grouped_pk_kernel(const int8_t* __restrict__ xq, int K,
                                                                             TileGroups tg, int8_t* __restrict__ xp,
                                                                             int32_t* __restrict__ c0,
                                                                             int32_t* __restrict__ counters,
                                                                             int ncounters) {
    if (blockIdx.x == 0 && blockIdx.y == 0)  // the tiled kernel's arrival counters start at zero
        for (int i = threadIdx.x; i < ncounters; i += 256) counters[i] = 0;
    // (every workgroup fetches the row offsets into LDS in one round trip: the search for its expert below, and the
    // table, which one thread builds in four passes, would otherwise wait for global memory expert by expert)
    __shared__ int32_t offs[kPkMaxExperts + 1];
    for (int i = threadIdx.x; i <= tg.num_experts; i += 256) offs[i] = tg.row_offsets[i];
    __syncthreads();
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        // Entries with the most rows first (the tiled kernel's cost grows with an entry's rows and workgroups start in
        // grid order: the short ones then fill the gaps the long ones leave).  Only an expert's last entry can be
        // short: the first pass lists every entry of more than 64 rows, the others the last entries of 33..64,
        // 17..32 and 1..16 rows.
        constexpr int tr = kTM;
        int used = 0;
        for (int pass = 0; pass < 4; ++pass) {
            const int above = pass == 0 ? 64 : pass == 1 ? 32 : pass == 2 ? 16 : 0;
            const int upto = pass == 0 ? tr : pass == 1 ? 64 : pass == 2 ? 32 : 16;
            int base16 = 0;
            for (int e = 0; e < tg.num_experts; ++e) {
                const int lo = offs[e], rows = offs[e + 1] - lo;
                const int nt = (rows + tr - 1) / tr;
                for (int t = tr > upto ? max(nt - 1, 0) : 0; t < nt && used < tg.slots; ++t) {  // (full entries: tr rows)
                    const int have = min(tr, rows - t * tr);
                    if (have <= above || have > upto) continue;
                    int32_t* entry = tg.table + 4 + 4 * used++;
                    entry[0] = e;
                    entry[1] = base16 + t * (tr / 16);
                    entry[2] = lo + t * tr;
                    entry[3] = have;
                }
                base16 += (rows + 15) >> 4;
            }
        }
        tg.table[0] = used;
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r = lane & 15, kb = lane >> 4;
    // which expert's rows this 16-row tile holds (uniform over the workgroup)
    const int pt = blockIdx.x;
    int row0 = 0, rows = 0;
    for (int e = 0, base16 = 0; e < tg.num_experts; ++e) {
        const int lo = offs[e], me = offs[e + 1] - lo;
        const int n16 = (me + 15) >> 4;
        if (pt < base16 + n16) {
            row0 = lo + 16 * (pt - base16);
            rows = min(16, me - 16 * (pt - base16));
            break;
        }
        base16 += n16;
    }
    if (rows == 0) return;  // past the last expert's tiles
    const int steps = K >> 7;
    const int s0 = (blockIdx.y * 4 + wave) * kPrepSteps;
    const int8_t* src = xq + (size_t)(row0 + min(r, rows - 1)) * K + kb * 16;
    uint4 v[kPrepSteps][2];
#pragma unroll
    for (int j = 0; j < kPrepSteps; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int st = min(s0 + j, steps - 1);
            v[j][h] = *reinterpret_cast<const uint4*>(src + st * 128 + h * 64);
            if (r >= rows) v[j][h] = make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
    for (int j = 0; j < kPrepSteps; ++j)
        if (s0 + j < steps) store_block((size_t)pt * steps + s0 + j, lane, v[j][0], v[j][1], xp, c0);
}

// The same straight from fp16 activations (the linear call): the per-token quantiser of Appendix A.1 and the
// preparation in one kernel.  A workgroup of 16 waves takes 8 token rows (half of a 16-row
// tile), reads them once, keeps the first kResidentSteps K steps of every wave in registers between the row maximum and
// the rounding (longer rows are read a second time, from cache), and writes its half of every 2 KB block as 128-byte
// pieces.  256 workgroups for 2048 rows: the chip is full, and the activations cross the memory interface once.
// Lane (h, kb, r): row r of the eight, the 16 codes k = 64 h + 16 kb .. + 15 of a K step; wave w takes the K steps
// w, w + 16, ...
constexpr int kRowsPerWg = 8, kRowWaves = 16, kResidentSteps = 8;

__global__ __launch_bounds__(kRowWaves* kWave) void quantize_prepare_rows_pk_kernel(const __half* __restrict__ x, int M, int K,
                                                                                   float* __restrict__ a_scale,
                                                                                   int8_t* __restrict__ xp,
                                                                                   int32_t* __restrict__ c0,
                                                                                   int32_t* __restrict__ counters,
                                                                                   int ncounters) {
    __shared__ float red[kRowWaves][kRowsPerWg];
    if (blockIdx.x == 0)  // the tiled kernel's arrival counters start at zero
        for (int i = threadIdx.x; i < ncounters; i += kRowWaves * kWave) counters[i] = 0;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r = lane & 7, kb = (lane >> 3) & 3, h = lane >> 5;
    const int mt = blockIdx.x >> 1, half = blockIdx.x & 1;
    const int m = 16 * mt + 8 * half + r;
    const int steps = K >> 7;
    const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)min(m, M - 1) * K + h * 64 + kb * 16);  // + 16 uint4 per step
    uint4 v[kResidentSteps][2];
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < kResidentSteps; ++j) {
        const int st = wave + j * kRowWaves;
        v[j][0] = v[j][1] = make_uint4(0u, 0u, 0u, 0u);
        if (st < steps) {  // (uniform over the wave)
            v[j][0] = src[st * 16];
            v[j][1] = src[st * 16 + 1];
        }
    }
#pragma unroll
    for (int j = 0; j < kResidentSteps; ++j) amax = fmaxf(amax, fmaxf(absmax8(v[j][0]), absmax8(v[j][1])));
    for (int st = wave + kResidentSteps * kRowWaves; st < steps; st += kRowWaves)
        amax = fmaxf(amax, fmaxf(absmax8(src[st * 16]), absmax8(src[st * 16 + 1])));
    // the row's maximum: over the lanes (h, kb) of the row, then over the waves
    amax = fmaxf(amax, __shfl_xor(amax, 8, kWave));
    amax = fmaxf(amax, __shfl_xor(amax, 16, kWave));
    amax = fmaxf(amax, __shfl_xor(amax, 32, kWave));
    if (lane < kRowsPerWg) red[wave][lane] = amax;
    __syncthreads();
    amax = red[0][r];
#pragma unroll
    for (int w = 1; w < kRowWaves; ++w) amax = fmaxf(amax, red[w][r]);
    const float s = amax / 127.0f;  // Appendix A.1, n = 8
    if (threadIdx.x < kRowsPerWg && m < M) a_scale[m] = s;
    auto emit = [&](int st, uint4 lo8, uint4 hi8) {
        const uint2 lo = quantize8(lo8, s), hi = quantize8(hi8, s);  // the canonical 16 codes
        const uint4 codes = m < M ? make_uint4(lo.x, lo.y, hi.x, hi.y) : make_uint4(0u, 0u, 0u, 0u);
        const size_t blk = (size_t)mt * steps + st;
        reinterpret_cast<uint4*>(xp + blk * 2048)[h * 64 + kb * 16 + 8 * half + r] = codes;
        int sum = sum16(codes);
        sum += __shfl_xor(sum, 8, kWave);
        sum += __shfl_xor(sum, 16, kWave);
        sum += __shfl_xor(sum, 32, kWave);
        if (lane < kRowsPerWg) c0[blk * 16 + 8 * half + lane] = -8 * sum;
    };
#pragma unroll
    for (int j = 0; j < kResidentSteps; ++j) {
        const int st = wave + j * kRowWaves;
        if (st < steps) emit(st, v[j][0], v[j][1]);  // (uniform over the wave)
    }
    for (int st = wave + kResidentSteps * kRowWaves; st < steps; st += kRowWaves) emit(st, src[st * 16], src[st * 16 + 1]);
}

typedef float v4f_t __attribute__((ext_vector_type(4)));

// One output tile.  WIDE: 32-bit multiplies in the integer scale step (some scale does not fit 24 signed bits).
// GROUPED: the mixture-of-experts form; `entry` is the workgroup's line of the tile table and `tile_n_g` its tile column.
// MS: 16-row token sub-tiles per wave (the tile has MS * 16 token rows).
// SILU: the weight rows alternate gate / up by 16-row tile and the epilogue writes fp16(SiLU(gate) * up), half as wide.
template <bool INT_SCALE, bool WIDE, bool GROUPED, int MS, bool SILU = false>
__device__ __forceinline__ void tile_pk(const PkArgs& a, const int8_t* __restrict__ xp, const int32_t* __restrict__ c0,
                                        const TileSplit& sp, const TileGroups& tg, const int32_t* entry, int tile_n_g,
                                        unsigned char* smem) {
    constexpr int TM = MS * 16, ABytes = TM * 128, Stage = stage_bytes(MS);
    constexpr int RB = MS < 4 ? MS : 4;       // sub-tiles of a partial tile read at a time when parts are added up
    constexpr int XL = MS >= 2 ? MS / 2 : 1;  // kilobyte loads of activations per wave and step
    static_assert(MS == 1 || MS == 2 || MS == 4 || MS == 8, "the tile has 16, 32, 64 or 128 token rows");
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wn = __builtin_amdgcn_readfirstlane(tid / kWave);  // the wave's 64 weight rows of the tile's 256
    const int li = lane & 15, kb = lane >> 4;

    // ---- which tile: XCD x (workgroups x, x + 8, ...) gets one contiguous range of linear tile numbers, and a range
    // walks the output in blocks of kGroupRows tile rows, column by column (shared operand tiles meet in that XCD's L2)
    const int tiles_n = (a.N + kTN - 1) / kTN;
    const int tiles_m = (a.M + TM - 1) / TM;
    int tile_m = 0, tile_n;
    int part = 0, tail_tile = -1;  // a tile of the last round: which K part, which of the round's tiles
    if constexpr (GROUPED) {
        tile_n = tile_n_g;
        if (sp.parts > 1) {  // every tile's K range is cut (few tiles for the chip): workgroup = (tile, part)
            part = blockIdx.x % sp.parts;
            tail_tile = blockIdx.x / sp.parts;
        }
    } else {
        int lid;
        if ((int)blockIdx.x < sp.whole) {
            const int q = sp.whole / kXcdCount, rem = sp.whole - q * kXcdCount;
            const int xcd = blockIdx.x % kXcdCount, idx = blockIdx.x / kXcdCount;
            lid = xcd * q + min(xcd, rem) + idx;
        } else {
            const int pidx = blockIdx.x - sp.whole;
            part = pidx / sp.rem;
            tail_tile = pidx - part * sp.rem;
            lid = sp.whole + tail_tile;
        }
        const int gsz = kGroupRows * tiles_n;
        const int g = lid / gsz, r = lid - g * gsz;
        const int gm = min(kGroupRows, tiles_m - g * kGroupRows);
        tile_n = r / gm;
        tile_m = g * kGroupRows + (r - tile_n * gm);
    }
    const int n0 = tile_n * kTN;
    // the tile's token rows: first 16-row tile of the prepared activations, first row of the tensors, how many
    const int expert = GROUPED ? entry[0] : 0;
    const int mt0 = GROUPED ? entry[1] : tile_m * MS;
    const int m0 = GROUPED ? entry[2] : tile_m * TM;
    const int m_rows = GROUPED ? entry[3] : min(TM, a.M - m0);
    const int mt_end = mt0 + ((m_rows + 15) >> 4);  // 16-row tiles from here on are not this tile's (they read as zero)
    const uint8_t* wpack = a.wpack + (GROUPED ? (size_t)expert * tg.wstride : 0);
    const uint8_t* spack = a.spack + (GROUPED ? (size_t)expert * tg.sstride : 0);
    const float* chan_scale = a.chan_scale ? a.chan_scale + (GROUPED ? (size_t)expert * a.N : 0) : nullptr;
    const int steps = a.K >> 7;
    const int NG = a.K / a.group;
    const int spg = a.group >> 7;
    // this workgroup's K steps
    const int s_begin = tail_tile < 0 ? 0 : (part * steps) / sp.parts;
    const int s_end = tail_tile < 0 ? steps : ((part + 1) * steps) / sp.parts;
    const int m16 = GROUPED ? tg.padded16 : (a.M + 15) >> 4, n16 = (a.N + 15) >> 4;

    // ---- loader roles.  Per step and wave: a quarter of the tile's 2 KB blocks of 16 token rows (XL loads of 1 KB),
    // the 1 KB blocks of four 16-row weight tiles; wave 0 also the step's 256 scales, wave 1 the corrections of its
    // token rows.  Tiles past the end of a tensor lie outside its descriptor and read as zero.
    const v4i xdesc = make_desc(xp, (size_t)m16 * steps * 2048);
    const v4i wdesc = make_desc(wpack, (size_t)n16 * steps * kPkBlockBytes);
    v4i adesc = make_desc(nullptr, 0);
    int aux_voff = (int)0x80000000u, aux_step = 0, aux_group = 0;
    if (wn == 0) {
        adesc = make_desc(spack + kPkHeaderBytes, (size_t)n16 * NG * 64);
        const int nt = (n0 >> 4) + (lane >> 2);
        aux_voff = nt < n16 ? nt * NG * 64 + (lane & 3) * 16 : (int)0x80000000u;
        aux_group = 64;
    } else if (wn == 1) {
        adesc = make_desc(c0, (size_t)m16 * steps * 64);
        const int mt = mt0 + (lane >> 2);
        aux_voff = (lane < 4 * MS && mt < mt_end) ? mt * steps * 64 + (lane & 3) * 16 : (int)0x80000000u;
        aux_step = 64;
    }
    // (the offsets of the 8 tile loads are a scalar each plus the lane's 16 bytes: kept in scalar registers and added
    // at the request; the whole offset has to travel in the vector offset, which is what the range check sees)
    int x_soff[XL], w_soff[4];
#pragma unroll
    for (int i = 0; i < XL; ++i) {  // the wave's half blocks wn * XL + i of the tile's 2 * MS
        const int mt = mt0 + ((wn * XL + i) >> 1);
        x_soff[i] = mt < mt_end ? mt * steps * 2048 + ((wn * XL + i) & 1) * 1024 : (int)0x80000000u;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int nt = (n0 >> 4) + 4 * wn + i;
        w_soff[i] = nt < n16 ? nt * steps * kPkBlockBytes : (int)0x80000000u;
    }
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const unsigned lds_x = wn * XL * 1024, lds_w = ABytes + wn * 4096;
    const unsigned lds_aux = ABytes + kBBytes + (wn == 1 ? kScBytes : 0);
    const int g_begin = s_begin / spg;
    int rq_x = s_begin * 2048, rq_w = s_begin * kPkBlockBytes, rq_sub = s_begin - g_begin * spg;
    int rq_aux = s_begin * aux_step + g_begin * aux_group;
    auto request_step = [&](int t) {
        const unsigned base = lds0 + (t & 1) * Stage;
        if (t < s_end) {
#pragma unroll
            for (int i = 0; i < XL; ++i)
                if (MS >= 2 || wn < 2)  // (a 16-row tile has two half blocks: waves 0 and 1)
                    load_to_lds_b128(xdesc, base, lds_x + i * 1024, x_soff[i] + rq_x + lane * 16, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) load_to_lds_b128(wdesc, base, lds_w + i * 1024, w_soff[i] + rq_w + lane * 16, 0);
            if (wn < 2) load_to_lds_b128(adesc, base, lds_aux, aux_voff, rq_aux);
        }
        rq_x += 2048;
        rq_w += kPkBlockBytes;
        const bool group_done = ++rq_sub == spg;
        rq_sub = group_done ? 0 : rq_sub;
        rq_aux += aux_step + (group_done ? aux_group : 0);
    };

    // ---- consumer roles: lane (li, kb) of MFMA 16x16x64 feeds row / column li and k chunk kb; its 4 results are
    // weight row li, token rows 4 kb .. + 3 of the sub-tile
    const int lane16 = lane * 16;
    const int b_off = ABytes + wn * 4096 + lane16;
    const int sc_off = ABytes + kBBytes + (wn * 64 + li) * 4;
    const int ci_off = ABytes + kBBytes + kScBytes + kb * 16;

    using acc4 = typename std::conditional<INT_SCALE, v4i, v4f_t>::type;
    acc4 acc[MS][kNS];
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int j = 0; j < kNS; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0;

    auto scale_into = [&](acc4& dst, const v4i& part, int sc_i) {
        const float s_f = __int_as_float(sc_i);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if constexpr (!INT_SCALE) dst[r] = fmaf((float)part[r], s_f, dst[r]);  // C' += float(C_g) * s_g
            else if constexpr (WIDE) {
                int prod = part[r] * sc_i;
                asm volatile("" : "+v"(prod));  // else a 64-bit multiply-add with register pairs
                dst[r] += prod;
            } else dst[r] += __mul24(part[r], sc_i);  // C'' += C_g * s_g^INT
        }
    };

    request_step(s_begin);
    for (int s = s_begin; s < s_end; ++s) {
        // this wave's requests for step s have landed; past the barrier so have everybody's, and everybody has
        // finished reading the other stage, which the requests for step s + 1 now overwrite
        asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        request_step(s + 1);
        const unsigned char* st = smem + (s & 1) * Stage;

        // the wave's four weight sub-tiles of this step: unpack once, use for all eight token sub-tiles
        v4i bu[kNS][2];
        int scl[kNS];
#pragma unroll
        for (int j = 0; j < kNS; ++j) {
            const v4i raw = *reinterpret_cast<const v4i*>(st + b_off + j * 1024);
            scl[j] = *reinterpret_cast<const int*>(st + sc_off + j * 64);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t pw = (uint32_t)raw[q];
                bu[j][0][q] = (int)((pw ^ 0x08080808u) & 0x0F0F0F0Fu);         // k 0..63 of the step: low nibbles
                bu[j][1][q] = (int)(((pw >> 4) ^ 0x08080808u) & 0x0F0F0F0Fu);  // k 64..127: high nibbles
            }
        }
        v4i part[2][kNS];
        v4i af[2][2], ci[2];
        af[0][0] = *reinterpret_cast<const v4i*>(st + lane16);
        af[0][1] = *reinterpret_cast<const v4i*>(st + 1024 + lane16);
        ci[0] = *reinterpret_cast<const v4i*>(st + ci_off);
#pragma unroll
        for (int i = 0; i < MS; ++i) {
            const int cur = i & 1, nxt = cur ^ 1;
            if (i + 1 < MS) {  // operands of the next token sub-tile, read while this one is multiplied
                af[nxt][0] = *reinterpret_cast<const v4i*>(st + (i + 1) * 2048 + lane16);
                af[nxt][1] = *reinterpret_cast<const v4i*>(st + (i + 1) * 2048 + 1024 + lane16);
                ci[nxt] = *reinterpret_cast<const v4i*>(st + ci_off + (i + 1) * 64);
            }
#pragma unroll
            for (int j = 0; j < kNS; ++j)
                part[cur][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[cur][0], bu[j][0], ci[cur], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < kNS; ++j)
                part[cur][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[cur][1], bu[j][1], part[cur][j], 0, 0, 0);
            // the scale step of the sub-tile before, under this one's MFMAs
            if (i > 0) {
#pragma unroll
                for (int j = 0; j < kNS; ++j) scale_into(acc[i - 1][j], part[nxt][j], scl[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < kNS; ++j) scale_into(acc[MS - 1][j], part[(MS - 1) & 1][j], scl[j]);
    }

    // ---- epilogue, once per output: FLOAT(acc) * s_a[m] * c[n] / alpha (Eq. (2)), or facc * s_a[m] (Eq. (1))
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");  // nobody reads operand tiles any more
    if (tail_tile >= 0) {
        // a K part of a tile of the last round: through the workspace; partial tile = [sub-tile i][j][thread][4],
        // written and read 16 bytes per lane with device-scope accesses (they go past the L2 of the writer's or
        // reader's own XCD, so that no cache has to be written back or invalidated as a whole)
        v4i* mine = reinterpret_cast<v4i*>(sp.partials + ((size_t)tail_tile * sp.parts + part) * kPartWords) + tid;
#pragma unroll
        for (int i = 0; i < MS; ++i)
#pragma unroll
            for (int j = 0; j < kNS; ++j) {
                v4i bits4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if constexpr (INT_SCALE) bits4[r] = acc[i][j][r];
                    else bits4[r] = __float_as_int(acc[i][j][r]);
                }
                // (a store of more than 8 bytes reads its data registers up to two cycles after it issues, and the
                // compiler, which inserts the wait for its own stores, does not see one inside an asm statement:
                // without the two idle cycles the next address computation may land in the first data registers)
                asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(mine + (i * kNS + j) * kTThreads), "v"(bits4)
                             : "memory");
            }
        // every wave's partial sums have been written through before the tile's counter is raised
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        int* flag = reinterpret_cast<int*>(smem);
        if (tid == 0)
            *flag = __hip_atomic_fetch_add(sp.counters + tail_tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int arrived = *flag;
        __syncthreads();  // (the flag's place is the output tile's below)
        if (arrived != sp.parts - 1) return;
        // the last part to arrive: all parts are in the workspace; add them in part order, whoever came last
#pragma unroll
        for (int i = 0; i < MS; ++i)
#pragma unroll
            for (int j = 0; j < kNS; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = 0;
        for (int q = 0; q < sp.parts; ++q) {
            const v4i* src = reinterpret_cast<const v4i*>(sp.partials + ((size_t)tail_tile * sp.parts + q) * kPartWords) + tid;
#pragma unroll
            for (int i = 0; i < MS; i += RB) {  // up to 16 loads of 16 bytes in flight per lane (the operand registers are free now)
                v4i got[RB][kNS];
#pragma unroll
                for (int ii = 0; ii < RB; ++ii)
#pragma unroll
                    for (int j = 0; j < kNS; ++j)
                        asm volatile("global_load_dwordx4 %0, %1, off sc1"
                                     : "=v"(got[ii][j])
                                     : "v"(src + ((i + ii) * kNS + j) * kTThreads)
                                     : "memory");
                // (the results pass through the wait, so that nothing is scheduled to use them before it)
#pragma unroll
                for (int ii = 0; ii < RB; ++ii)  // (the first of these waits, the others only tie their registers)
                    asm volatile("s_waitcnt vmcnt(0)"
                                 : "+v"(got[ii][0]), "+v"(got[ii][1]), "+v"(got[ii][2]), "+v"(got[ii][3])
                                 :
                                 : "memory");
#pragma unroll
                for (int ii = 0; ii < RB; ++ii)
#pragma unroll
                    for (int j = 0; j < kNS; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if constexpr (INT_SCALE) acc[i + ii][j][r] += got[ii][j][r];
                            else acc[i + ii][j][r] += __int_as_float(got[ii][j][r]);
                        }
            }
        }
        if (tid == 0) __hip_atomic_store(sp.counters + tail_tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);
    const int n_rows = min(kTN, a.N - n0);
    // Rows of 8-aligned length go through an fp16 copy of the tile in LDS and leave as 16-byte stores; otherwise (and
    // for the diagnostic accumulator output) element by element.
    const bool staged = (a.N & (SILU ? 15 : 7)) == 0 && a.acc_out == nullptr;
    constexpr int kPitch = 264;  // halves per LDS row: 256 + 8, so that rows keep 16-byte alignment
    __half* otile = reinterpret_cast<__half*>(smem);
    float sa[MS][4];
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ml = i * 16 + 4 * kb + r;
            sa[i][r] = ml < m_rows ? a.a_scale[m0 + ml] : 0.0f;
        }
    auto channel = [&](int j) {  // what an accumulator of weight sub-tile j is multiplied by besides the token scale
        const int nl = wn * 64 + j * 16 + li;
        float c = 1.0f;
        if constexpr (INT_SCALE) {
            if (chan_scale && nl < n_rows) c = chan_scale[n0 + nl];
            c *= inv_alpha;
        }
        return c;
    };
    auto result = [&](const acc4& v, int r, float s, float c) {
        if constexpr (INT_SCALE) return (float)v[r] * s * c;
        else return v[r] * s;
    };
    if constexpr (SILU) {
        // Sub-tiles 2q and 2q + 1 of a wave are the gate and up rows of the same 16 outputs: the lane holds both.  The
        // result is DEFINED as the unfused pipeline (GEMM output rounded to fp16, then SiLU * up on those values), so
        // that fusing changes no bit; it saves the [M, N] tensor's trip through memory.
        const int out_n = a.N >> 1, out_n0 = n0 >> 1, out_rows = n_rows >> 1;
#pragma unroll
        for (int q = 0; q < kNS / 2; ++q) {
            const float cg = channel(2 * q), cu = channel(2 * q + 1);
            const int ol = wn * 32 + q * 16 + li;  // output column inside the tile's 128
#pragma unroll
            for (int i = 0; i < MS; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int ml = i * 16 + 4 * kb + r;
                    const float g = __half2float(__float2half_rn(result(acc[i][2 * q], r, sa[i][r], cg)));
                    const float u = __half2float(__float2half_rn(result(acc[i][2 * q + 1], r, sa[i][r], cu)));
                    const __half h = __float2half_rn(silu_mul(g, u));  // (the product arrives rounded to fp32)
                    if (staged) {
                        otile[ml * kPitch + ol] = h;
                    } else if (ml < m_rows && ol < out_rows) {
                        a.out[(size_t)(m0 + ml) * out_n + out_n0 + ol] = h;
                        if constexpr (INT_SCALE) {
                            if (a.acc_out) {
                                const size_t o = (size_t)(m0 + ml) * a.N + n0 + wn * 64 + 2 * q * 16 + li;
                                a.acc_out[o] = acc[i][2 * q][r];
                                a.acc_out[o + 16] = acc[i][2 * q + 1][r];
                            }
                        }
                    }
                }
        }
        if (staged) {
            __syncthreads();
            const int chunk = tid & 15;  // 8 outputs
            if (chunk * 8 < out_rows) {
#pragma unroll
                for (int pass = 0; pass < TM / 16; ++pass) {
                    const int ml = pass * 16 + (tid >> 4);
                    if (ml < m_rows)
                        *reinterpret_cast<uint4*>(a.out + (size_t)(m0 + ml) * out_n + out_n0 + chunk * 8) =
                            *reinterpret_cast<const uint4*>(otile + ml * kPitch + chunk * 8);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < kNS; ++j) {
        const int nl = wn * 64 + j * 16 + li;
        const int n = n0 + nl;
        const float c = channel(j);
#pragma unroll
        for (int i = 0; i < MS; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int ml = i * 16 + 4 * kb + r;
                const __half h = __float2half_rn(result(acc[i][j], r, sa[i][r], c));
                if (staged) {
                    otile[ml * kPitch + nl] = h;
                } else if (ml < m_rows && nl < n_rows) {
                    const size_t o = (size_t)(m0 + ml) * a.N + n;
                    if constexpr (INT_SCALE) {
                        if (a.acc_out) a.acc_out[o] = acc[i][j][r];
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
            for (int pass = 0; pass < TM / 8; ++pass) {
                const int ml = pass * 8 + (tid >> 5);
                if (ml < m_rows)
                    *reinterpret_cast<uint4*>(a.out + (size_t)(m0 + ml) * a.N + n0 + chunk * 8) =
                        *reinterpret_cast<const uint4*>(otile + ml * kPitch + chunk * 8);
            }
        }
    }
}

// The dense form's tile code: 128 token rows per tile, or, for calls of at most 64 rows (33..64 rows on large weight
// matrices take this kernel, see pk_takes_tile), the 64-row instance, which runs half the MFMAs and scale steps.
template <bool INT_SCALE, bool SILU, int MS>
__device__ __forceinline__ void dense_tile_rows(const PkArgs& a, const int8_t* __restrict__ xp, const int32_t* __restrict__ c0,
                                                const TileSplit& sp, const TileGroups& none, unsigned char* smem) {
    if constexpr (INT_SCALE) {
        const int flags = *reinterpret_cast<const int32_t*>(a.spack);
        if (flags & kPkFlagWide) tile_pk<true, true, false, MS, SILU>(a, xp, c0, sp, none, nullptr, 0, smem);
        else tile_pk<true, false, false, MS, SILU>(a, xp, c0, sp, none, nullptr, 0, smem);
    } else {
        tile_pk<false, false, false, MS, SILU>(a, xp, c0, sp, none, nullptr, 0, smem);
    }
}
template <bool INT_SCALE, bool SILU>
__device__ __forceinline__ void dense_tile(const PkArgs& a, const int8_t* __restrict__ xp, const int32_t* __restrict__ c0,
                                           const TileSplit& sp, const TileGroups& none, unsigned char* smem) {
    if (a.M <= 64) dense_tile_rows<INT_SCALE, SILU, 4>(a, xp, c0, sp, none, smem);
    else dense_tile_rows<INT_SCALE, SILU, kMS>(a, xp, c0, sp, none, smem);
}

// (two waves per SIMD, from two workgroups: this also keeps the MFMA results in ordinary vector registers, where the
// scale step reads them; with a whole SIMD to itself the compiler would put them into accumulation registers and copy)
template <bool INT_SCALE>
__global__ __launch_bounds__(kTThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_tile_pk_kernel(PkArgs a, const int8_t* __restrict__ xp,
                                                                 const int32_t* __restrict__ c0, TileSplit sp) {
    extern __shared__ __align__(16) unsigned char smem_tpk[];
    const TileGroups none{};
    dense_tile<INT_SCALE, false>(a, xp, c0, sp, none, smem_tpk);
}

// The same on gate / up rows that alternate by 16-row tile, with SiLU(gate) * up as the epilogue (Sec. 4.2 names kernel
// fusion around the GEMM; the LLaMA feed-forward block applies this to the fused gate_up projection).
template <bool INT_SCALE>
__global__ __launch_bounds__(kTThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_tile_silu_pk_kernel(
    PkArgs a, const int8_t* __restrict__ xp, const int32_t* __restrict__ c0, TileSplit sp) {
    extern __shared__ __align__(16) unsigned char smem_tpk[];
    const TileGroups none{};
    dense_tile<INT_SCALE, true>(a, xp, c0, sp, none, smem_tpk);
}

// Mixture-of-experts form: workgroup b takes table entry b / (tile columns) and tile column b % (tile columns); the
// entries in use come first, so the workgroups without one sit at the end of the grid and leave at once.  An entry is
// up to 128 token rows of one expert; a wave's instructions per K step are a fixed share (its weights' unpacking, the
// requests, the bookkeeping) plus a share per 16 token rows, so the entry's rows pick the instance: 16, 32, 64 or 128.
template <bool INT_SCALE, int MS>
__device__ __forceinline__ void grouped_tile(const PkArgs& a, const int8_t* __restrict__ xp, const int32_t* __restrict__ c0,
                                             const TileSplit& sp, const TileGroups& tg, const int32_t* entry, int tile_n,
                                             unsigned char* smem) {
    if constexpr (INT_SCALE) {
        const int flags = *reinterpret_cast<const int32_t*>(a.spack + (size_t)entry[0] * tg.sstride);  // this expert's
        if (flags & kPkFlagWide) tile_pk<true, true, true, MS>(a, xp, c0, sp, tg, entry, tile_n, smem);
        else tile_pk<true, false, true, MS>(a, xp, c0, sp, tg, entry, tile_n, smem);
    } else {
        tile_pk<false, false, true, MS>(a, xp, c0, sp, tg, entry, tile_n, smem);
    }
}

template <bool INT_SCALE>
__global__ __launch_bounds__(kTThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_tile_grouped_pk_kernel(
    PkArgs a, const int8_t* __restrict__ xp, const int32_t* __restrict__ c0, TileGroups tg, TileSplit sp) {
    extern __shared__ __align__(16) unsigned char smem_tpk[];
    const int tiles_n = (a.N + kTN - 1) / kTN;
    const int tile = blockIdx.x / sp.parts;  // (slot, tile column); sp.parts workgroups share it
    const int slot = tile / tiles_n;
    if (slot >= tg.table[0]) return;  // uniform over the workgroup, before any barrier
    const int32_t* entry = tg.table + 4 + 4 * slot;
    const int tile_n = tile - slot * tiles_n;
    const int rows = entry[3];
    if (rows > 64) grouped_tile<INT_SCALE, 8>(a, xp, c0, sp, tg, entry, tile_n, smem_tpk);
    else if (rows > 32) grouped_tile<INT_SCALE, 4>(a, xp, c0, sp, tg, entry, tile_n, smem_tpk);
    else if (rows > 16) grouped_tile<INT_SCALE, 2>(a, xp, c0, sp, tg, entry, tile_n, smem_tpk);
    else grouped_tile<INT_SCALE, 1>(a, xp, c0, sp, tg, entry, tile_n, smem_tpk);
}

size_t xp_bytes(int M, int K) { return pad256((size_t)((M + 15) / 16) * 16 * K); }
size_t c0_bytes(int M, int K) { return pad256((size_t)((M + 15) / 16) * (K / 128) * 64); }

// The split of the last round, given `avail` bytes for partial tiles (0: no split).
void plan_tail(int M, int N, int K, size_t avail, int* whole, int* rem, int* parts) {
    const int tiles = ((N + kTN - 1) / kTN) * ((M + kTM - 1) / kTM);
    const int steps = K >> 7;
    const int slots = min(2 * cu_count(), (int)(kCounterBytes / 4));
    const int left = tiles % slots;
    int p = 1;
    if (left > 0) {
        // up to one workgroup per compute unit: a workgroup that has its compute unit to itself runs at about 1.7 times
        // the rate of one that shares it, so filling both places of a unit with half-length parts gains nothing
        p = min(min((slots / 2) / left, 8), steps / kMinPartSteps);
        static const int env_parts = env_int("INTSCALE_TILE_PARTS", 0);  // experiments (read once): at most this many
        if (env_parts) p = min(p, max(1, env_parts));
        p = (int)min((size_t)p, min(avail, kPartialCap) / ((size_t)left * kPartWords * 4));
    }
    if (p < 2) {
        *whole = tiles;
        *rem = 0;
        *parts = 1;
    } else {
        *whole = tiles - left;
        *rem = left;
        *parts = p;
    }
}

}  // namespace

// workspace = [prepared activations: ceil(M/16) x K/128 blocks of 2 KB | corrections: ceil(M/16) x K/128 x 16 words |
//              arrival counters of the last round's tiles | their partial tiles]; the launch splits the last round as
//              far as the bytes it is given allow, and not at all below gemm_tile_pk_min_workspace_bytes + one round
size_t gemm_tile_pk_min_workspace_bytes(int M, int K) { return xp_bytes(M, K) + c0_bytes(M, K) + kCounterBytes; }
size_t gemm_tile_pk_workspace_bytes(int M, int N, int K) {
    int whole, rem, parts;
    plan_tail(M, N, K, kPartialCap, &whole, &rem, &parts);
    return gemm_tile_pk_min_workspace_bytes(M, K) + (size_t)rem * parts * kPartWords * 4;
}

bool gemm_tile_pk_takes_fp16(int K) { return (K & 127) == 0; }

void gemm_tile_pk_kernel_names(int K, bool int_scale, bool fp16_in, char* buf, size_t len, bool silu) {
    char prep[96];
    if (fp16_in) snprintf(prep, sizeof prep, "quantize_prepare_rows_pk_kernel");
    else snprintf(prep, sizeof prep, "prepare_activations_pk_kernel");
    snprintf(buf, len, "%s\ngemm_tile%s_pk_kernel<%s>", prep, silu ? "_silu" : "", int_scale ? "true" : "false");
}

// The preparation of quantised activations on its own (for activations that several GEMMs share): fills the fixed part
// of the workspace and sets every arrival counter of the last-round split to zero, whatever N the GEMMs will have.
hipError_t launch_prepare_activations_pk(const int8_t* xq, int M, int K, void* workspace, hipStream_t stream) {
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int8_t* xp = reinterpret_cast<int8_t*>(ws);
    int32_t* c0 = reinterpret_cast<int32_t*>(ws + xp_bytes(M, K));
    int32_t* counters = reinterpret_cast<int32_t*>(ws + gemm_tile_pk_min_workspace_bytes(M, K) - kCounterBytes);
    const int per_wg = 4 * kPrepSteps;
    const dim3 blocks((M + 15) / 16, ((K >> 7) + per_wg - 1) / per_wg);
    hipLaunchKernelGGL(prepare_activations_pk_kernel, blocks, dim3(256), 0, stream, xq, M, K, xp, c0, counters,
                       (int)(kCounterBytes / 4));
    return hipGetLastError();
}

// prepared: the workspace already holds the activations' blocks, corrections and zeroed counters (the call above, or an
// earlier launch on the same activations: every launch leaves the counters zero); only the tiled kernel is launched.
hipError_t launch_gemm_tile_pk(const PkArgs& a, bool int_scale, void* workspace, size_t workspace_bytes,
                               hipStream_t stream, bool prepared) {
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int8_t* xp = reinterpret_cast<int8_t*>(ws);
    int32_t* c0 = reinterpret_cast<int32_t*>(ws + xp_bytes(a.M, a.K));
    const size_t fixed = gemm_tile_pk_min_workspace_bytes(a.M, a.K);
    if (workspace_bytes < fixed) return hipErrorInvalidValue;
    TileSplit sp;
    plan_tail(a.M, a.N, a.K, workspace_bytes - fixed, &sp.whole, &sp.rem, &sp.parts);
    sp.counters = reinterpret_cast<int32_t*>(ws + fixed - kCounterBytes);
    sp.partials = reinterpret_cast<int32_t*>(ws + fixed);
    const int mtiles = (a.M + 15) / 16;
    const int per_wg = 4 * kPrepSteps;
    const dim3 blocks(mtiles, ((a.K >> 7) + per_wg - 1) / per_wg);
    if (prepared) {
        // nothing to prepare
    } else if (a.x_fp16) {  // fp16 activations: quantised on the way, the token scales go to a.a_scale_out (= a.a_scale)
        hipLaunchKernelGGL(quantize_prepare_rows_pk_kernel, dim3(2 * mtiles), dim3(kRowWaves * kWave), 0, stream, a.x_fp16,
                           a.M, a.K, a.a_scale_out, xp, c0, sp.counters, sp.rem);
    } else {
        hipLaunchKernelGGL(prepare_activations_pk_kernel, blocks, dim3(256), 0, stream, a.xq, a.M, a.K, xp, c0,
                           sp.counters, sp.rem);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t smem = 2 * (size_t)stage_bytes(kMS);
    const int tiles = sp.whole + sp.rem * sp.parts;  // workgroups
    static LdsLimit limits[4];
    auto launch = [&](auto kernel, int which) -> hipError_t {
        const hipError_t r = limits[which].raise(reinterpret_cast<const void*>(kernel), (int)smem);
        if (r != hipSuccess) return r;
        hipLaunchKernelGGL(kernel, dim3(tiles), dim3(kTThreads), smem, stream, a, xp, c0, sp);
        return hipGetLastError();
    };
    if (a.pair) return int_scale ? launch(gemm_tile_silu_pk_kernel<true>, 2) : launch(gemm_tile_silu_pk_kernel<false>, 3);
    return int_scale ? launch(gemm_tile_pk_kernel<true>, 0) : launch(gemm_tile_pk_kernel<false>, 1);
}

// ---- mixture-of-experts form
// workspace = [prepared activations, every expert padded to whole 16-row tiles | corrections | table of row tiles |
//              arrival counters and partial tiles when the K range is cut]
// K parts per tile of the grouped form: when all the tiles there can be fit the chip at once several times over
static int grouped_parts(int E, int M, int N, int K) {
    const long long tiles = ((long long)(M + kTM - 1) / kTM + E) * ((N + kTN - 1) / kTN);
    const long long p = (2LL * cu_count()) / tiles;
    int parts = (int)std::min<long long>(std::min<long long>(p, 8), (K >> 7) / kMinPartSteps);
    if (parts < 2 || tiles * parts * (long long)kPartWords * 4 > (long long)kPartialCap) parts = 1;
    return parts;
}

size_t gemm_tile_grouped_pk_workspace_bytes(int E, int M, int N, int K) {
    const size_t padded16 = (size_t)(M + 15) / 16 + E;
    const size_t slots = (size_t)(M + kTM - 1) / kTM + E;
    const size_t tiles = slots * ((N + kTN - 1) / kTN);
    const int parts = grouped_parts(E, M, N, K);
    return pad256(padded16 * 16 * K) + pad256(padded16 * (K / 128) * 64) + pad256((4 + 4 * slots) * 4) +
           (parts > 1 ? pad256(tiles * 4) + tiles * parts * (size_t)kPartWords * 4 : 0);
}

void gemm_tile_grouped_pk_kernel_names(int E, int M, bool int_scale, char* buf, size_t len) {
    snprintf(buf, len, "prepare_activations_grouped_pk_kernel\ngemm_tile_grouped_pk_kernel<%s>", int_scale ? "true" : "false");
}

template <typename Kernel>
static hipError_t launch_grouped_instance(Kernel kernel, int which, size_t smem, const PkArgs& a, const int8_t* xp,
                                          const int32_t* c0, const TileGroups& tg, const TileSplit& sp, int grid,
                                          hipStream_t stream) {
    static LdsLimit limits[2];  // (this template has one instantiation per kernel type: `which` tells its two users apart)
    const hipError_t r = limits[which].raise(reinterpret_cast<const void*>(kernel), (int)smem);
    if (r != hipSuccess) return r;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kTThreads), smem, stream, a, xp, c0, tg, sp);
    return hipGetLastError();
}

hipError_t launch_gemm_tile_grouped_pk(const PkArgs& a, const int32_t* row_offsets, int E, size_t wstride,
                                       size_t sstride, bool int_scale, void* workspace, hipStream_t stream) {
    TileGroups tg;
    tg.row_offsets = row_offsets;
    tg.num_experts = E;
    tg.padded16 = (a.M + 15) / 16 + E;
    tg.slots = (a.M + kTM - 1) / kTM + E;
    tg.wstride = wstride;
    tg.sstride = sstride;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int8_t* xp = reinterpret_cast<int8_t*>(ws);
    const size_t xbytes = pad256((size_t)tg.padded16 * 16 * a.K);
    int32_t* c0 = reinterpret_cast<int32_t*>(ws + xbytes);
    unsigned char* at = ws + xbytes + pad256((size_t)tg.padded16 * (a.K / 128) * 64);
    tg.table = reinterpret_cast<int32_t*>(at);
    at += pad256((4 + 4 * (size_t)tg.slots) * 4);
    const int tiles = tg.slots * ((a.N + kTN - 1) / kTN);
    TileSplit sp{};
    sp.parts = grouped_parts(E, a.M, a.N, a.K);
    sp.rem = sp.parts > 1 ? tiles : 0;
    sp.counters = reinterpret_cast<int32_t*>(at);
    sp.partials = reinterpret_cast<int32_t*>(at + pad256((size_t)tiles * 4));
    const int per_wg = 4 * kPrepSteps;
    hipLaunchKernelGGL(prepare_activations_grouped_pk_kernel, dim3(tg.padded16, ((a.K >> 7) + per_wg - 1) / per_wg),
                       dim3(256), 0, stream, a.xq, a.K, tg, xp, c0, sp.counters, sp.rem);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int grid = tiles * sp.parts;
    const size_t smem = 2 * (size_t)stage_bytes(kMS);
    return int_scale ? launch_grouped_instance(gemm_tile_grouped_pk_kernel<true>, 0, smem, a, xp, c0, tg, sp, grid, stream)
                     : launch_grouped_instance(gemm_tile_grouped_pk_kernel<false>, 1, smem, a, xp, c0, tg, sp, grid, stream);
}

}  // namespace intscale
