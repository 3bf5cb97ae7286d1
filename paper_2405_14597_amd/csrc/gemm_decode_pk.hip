// Decode regime (at most 64 token rows) of the fine-grained W4A8 GEMM on prepacked weights: a weight-streaming kernel
// with no synchronisation inside its main loop.  Integer-scale form: Eq. (2) / Table 2 "Ours" of the Integer Scale
// paper; float-scale form: Eq. (1) / Table 2 "Atom".
//
// Work split.  The weight matrix is a grid of 1 KB blocks (16 weight rows x 128 k, see pk_common.h).  K is cut into
// `slabs` ranges of K steps, each slab owned by its own set of workgroups (one per CU in total); inside a slab a
// workgroup owns a range of whole row tiles, and its blocks, taken tile after tile and along K inside a tile, are dealt
// out evenly over its waves as contiguous ranges.  So every wave streams one contiguous piece of the packed weights,
// all waves of the chip carry the same number of blocks to within one, and nobody waits for anybody until the end.
// The quantised activations of the slab sit in LDS in MFMA operand order (written once per workgroup); a wave keeps
// its int32 accumulators in registers while it walks along K and meets the other waves only when a row tile is
// finished: pieces of a tile that several waves hold are added in LDS behind the single barrier at the end of the
// kernel (int32 adds are order-free; the float-scale partials are added in wave order), and with more than one slab
// the slabs' partial tiles meet in a workspace: each workgroup stores its partial, raises the tile's arrival counter,
// and the one that arrives last adds the partials in slab order and runs the epilogue.  Nobody ever waits for another
// workgroup.
//
// Per block: one 16-byte load per lane (issued DT blocks ahead), two bit operations per register for the two B
// operands (16 * q as signed bytes: the nibble in the high half of a byte), two v_mfma_i32_16x16x64_i8 per token tile
// whose A operands come from LDS, one shift and one v_mad_i32_i24 per partial product (Eq. (2): C'' += C_g * s_g^INT),
// against a convert and a multiply-add for the float-scale form (Eq. (1)).  The epilogue is the one conversion of
// Eq. (2): float(acc) * s_a[m] * c[n] / alpha.
#include <stdio.h>
#include <stdlib.h>

#include "act_common.h"
#include "pk_common.h"

namespace intscale {
namespace {

constexpr int kOutOfRange = (int)0x80000000u;  // a buffer offset past every descriptor here: the load returns 0
constexpr int kFill = 8;                       // activation chunks a thread has in flight while it fills LDS
constexpr int kFuseChunks = 4;                 // fused quantiser: 16-byte chunks of the fp16 token per thread

using rsrc_t = __amdgpu_buffer_rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
    const unsigned n = bytes > 0x7FFFFFFFull ? 0x7FFFFFFFu : (unsigned)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}

// Workgroup barrier that only waits for this wave's LDS traffic (not for the weight loads in flight).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct PkKernelPlan {
    int n16;          // row tiles
    int steps;        // K / 128
    int num_groups;   // K / group
    int spg;          // K steps per group
    int slabs;        // K split across workgroups
    int steps_q, steps_r;  // K steps per slab: steps_q, one more for the first steps_r slabs
    int tiles_q, tiles_r;  // row tiles per workgroup of a slab: tiles_q, one more for the first tiles_r workgroups
    int rows;         // token rows kept per tile in LDS (power of two)
    int slot_offset;  // LDS byte offset of the pieces of shared tiles (0: they reuse the activations' space)
    int cs_offset;    // LDS byte offset of the workgroup's channel scales
    size_t wbytes, sbytes;
};

// Optional timeline of a launch (built with -DPK_TRACE only; used to find where a short kernel's time goes).
#ifdef PK_TRACE
__device__ unsigned long long g_pk_trace[256 * 2 * 8];
#define PK_MARK(i)                                                                                          \
    do {                                                                                                    \
        if ((wave == 0 || wave == W - 1) && lane == 0 && blockIdx.y == 0 && blockIdx.x < 256)               \
            g_pk_trace[(blockIdx.x * 2 + (wave ? 1 : 0)) * 8 + (i)] = __builtin_amdgcn_s_memrealtime();    \
    } while (0)
#else
#define PK_MARK(i)
#endif

__device__ __forceinline__ int mad_i24(int a, int b, int c) {
    int r;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// NR: result registers per lane and token tile that carry token rows of the call (lane (li, kb) holds token rows
// 16 t + 4 kb + r): 4 in general, 1 for a single token row, whose scale step then costs a quarter of the instructions.
template <int MT, int DT, int WAVES, int NR, bool INT_SCALE, bool FUSEQ>
__device__ __forceinline__ void decode_pk_body(const PkArgs& a, const PkKernelPlan& p, unsigned char* smem) {
    using acc_t = typename std::conditional<INT_SCALE, int, float>::type;
    static_assert(DT >= 2 && DT <= 8, "ring of 2 to 8 blocks");
    constexpr int W = WAVES;
    static_assert((W & (W - 1)) == 0, "waves per workgroup: a power of two");
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int li = lane & 15, kb = lane >> 4;
    PK_MARK(0);
    // "some integer scale needs more than 24 signed bits" (left in the header by the prepacking): asked for here,
    // needed only in the first scale step, so that the request is not waited for ahead of the weight stream
    const int pk_flags = *reinterpret_cast<const int32_t*>(a.spack);
    // All kernel arguments travel in one round trip: without this the ones first used behind a branch are asked for
    // there, and waited for a second time.
    asm volatile("" ::"s"(a.xq), "s"(a.x_fp16), "s"(a.a_scale), "s"(a.a_scale_out), "s"(a.chan_scale), "s"(a.out),
                 "s"(a.acc_out), "s"(a.counters), "s"(a.partials), "s"(a.M), "s"(a.N), "s"(a.alpha_log2), "s"(p.rows),
                 "s"(p.slot_offset), "s"(p.cs_offset), "s"(p.n16), "s"(p.slabs));

    // ---- this workgroup's slab and row tiles, this wave's blocks.  (Grid: x = workgroup inside its slab, y = slab.
    // Even shares without a division: the first `..._r` owners take one more than `..._q`.)  Everything up to the
    // first requests of the weight stream is kept short: all waves of a SIMD run it at the same time, and the HBM
    // latency only starts to count down behind it.
    const int slab = blockIdx.y;
    const int jw = blockIdx.x;
    const int s_lo = slab * p.steps_q + min(slab, p.steps_r);
    const int ksl = p.steps_q + (slab < p.steps_r ? 1 : 0);
    const int t0 = jw * p.tiles_q + min(jw, p.tiles_r);
    const int t1 = t0 + p.tiles_q + (jw < p.tiles_r ? 1 : 0);
    const int B = (t1 - t0) * ksl;  // (a workgroup without blocks leaves behind its first, empty, requests: an early
                                    // exit here would split the kernel-argument loads into two round trips)
    const int b0 = (wave * B) / W, b1 = ((wave + 1) * B) / W;
    const rsrc_t wres = make_rsrc(a.wpack, p.wbytes);
    const rsrc_t sres = make_rsrc(a.spack + kPkHeaderBytes, p.sbytes);

    // ---- the weight stream.  A wave's blocks are cut into segments (its run of K steps inside one row tile), a
    // segment into turns of DT blocks; the last turn of a segment is filled up with empty blocks (requests that lie
    // outside the buffer and return zeros), so that the ring of DT register slots always starts a segment at slot 0
    // and slot u of a turn is requested while slot u of the turn before is used, in straight-line code.
    v4i wq[DT];
    int scl[DT];
    const int w_lane = lane * 16, s_lane = li * 4;
    // issue cursor (one turn ahead of the consume cursor)
    int rem_i = b1 - b0;
    // the tile of the wave's first block: floor(floor(wave * tiles * ksl / W) / ksl) = floor(wave * tiles / W)
    const int q0 = (wave * (t1 - t0)) / W;
    int tile_i = t0 + q0, step_i = b0 - q0 * ksl;
    int left_i = min(ksl - step_i, rem_i);
    int woff_i = 0, soff_i = 0, sub_i = 0;
    auto issue_state = [&]() {
        const int s_abs = s_lo + step_i;
        int g = s_abs;  // s_abs / spg
        if (p.spg != 1) {
            g = __builtin_amdgcn_readfirstlane((int)(((float)s_abs + 0.5f) * __builtin_amdgcn_rcpf((float)p.spg)));
            if (g * p.spg > s_abs) --g;
            else if ((g + 1) * p.spg <= s_abs) ++g;
        }
        woff_i = (tile_i * p.steps + s_abs) * kPkBlockBytes;
        soff_i = (tile_i * p.num_groups + g) * 64;
        sub_i = s_abs - g * p.spg;
    };
    auto issue_advance = [&]() {
        const int adv = min(DT, left_i);
        rem_i -= adv;
        step_i += adv;
        left_i -= adv;
        if (left_i == 0) {
            ++tile_i;
            step_i = 0;
            left_i = min(ksl, rem_i);
        }
        issue_state();
    };
    int sub_run = 0, goff_run = 0;  // inside a turn: K step in its group, byte offset of its group from the turn's first
    auto issue = [&](int u) {
        // the whole offset travels in the vector offset: that is what the descriptor's range check sees
        const bool ok = u < left_i;
        wq[u] = __builtin_amdgcn_raw_buffer_load_b128(wres, w_lane + (ok ? woff_i + u * kPkBlockBytes : kOutOfRange), 0, 0);
        scl[u] = __builtin_amdgcn_raw_buffer_load_b32(sres, s_lane + (ok ? soff_i + goff_run : kOutOfRange), 0, 0);
        if (++sub_run == p.spg) {
            sub_run = 0;
            goff_run += 64;
        }
    };
    // ---- the activations of the slab: requested in FRONT of the weight stream and written to LDS below.  A wave's
    // loads return in order, and these come from L2: asked for first, they are in LDS while the first weights are
    // still on their way from HBM; asked for behind the ring's first blocks they arrive behind them, and the fill
    // and its barrier then stand between the weights' arrival and their use (about 1 us per call).
    // A fill unit is 8 token rows x one K step (8 x 128 bytes); unit u = step * (row blocks) + row block.
    const int rs = p.rows;
    const int unit_b = 64 * rs;  // bytes of one (step, token tile, MFMA half) unit: 4 k-chunks x rs rows x 16 bytes
    const int step_stride = MT * 2 * unit_b;
    [[maybe_unused]] uint4 xh[FUSEQ ? kFuseChunks : 1];
    [[maybe_unused]] v4i xraw[FUSEQ ? 1 : kFill];
    // row blocks of 8 token rows, rounded up to a power of two (rows past M are masked): unit -> (step, row block) by shifts
    const int rb_log = a.M <= 8 ? 0 : a.M <= 16 ? 1 : a.M <= 32 ? 2 : 3;
    const int units = ksl << rb_log;
    // A wave's units of one batch are W apart: the same row block, K steps (W >> rb_log) apart.  What depends on the
    // lane is worked out once; a request or an LDS write then costs one addition (all waves of the unit run this
    // prologue at the same time, and its instructions queue in front of the weight stream's first use).
    const int fill_dstep = W >> rb_log;
    const int fill_step0 = wave >> rb_log;
    const int fill_row = ((wave & ((1 << rb_log) - 1)) << 3) + (lane >> 3);
    const int fill_c8 = lane & 7;
    const int fill_goff =
        fill_row < a.M ? fill_row * a.K + (s_lo + fill_step0) * 128 + fill_c8 * 16 : kOutOfRange;  // stays out of range
    const int fill_loff = ((fill_step0 * MT + (fill_row >> 4)) * 2 + (fill_c8 >> 2)) * unit_b + (fill_c8 & 3) * 16 * rs +
                          (fill_row & 15) * 16;
    // (a batch made of whole rounds over the waves, the usual case, runs without a test per unit)
    const bool fill_has_place = fill_row < (MT == 1 ? rs : 16 * MT);  // rows past M arrive as zeros; rows without a place in LDS are not written
    // One token row: its codes are contiguous and the operand order is the natural order of k, so the fill is a plain
    // copy, 16 bytes per lane, and only the first waves take part (8 KB are 8 wave loads; dealt by the unit scheme
    // above, every wave would fetch four pieces of 128 bytes, and the barrier behind the fill would wait for the
    // last wave's share, which is requested a microsecond and more after the first wave's).
    const int row_chunks = ksl * 8;
    const bool one_row = MT == 1 && rs == 1 && row_chunks <= kFill * W * kWave;
    [[maybe_unused]] auto fill_load = [&](int base) {
        const rsrc_t xres = make_rsrc(a.xq, (size_t)a.M * a.K);
        if (one_row) {
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                if ((i * W + wave) * kWave >= row_chunks) break;  // uniform over the wave
                const int c = (int)threadIdx.x + i * W * kWave;
                xraw[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, c < row_chunks ? s_lo * 128 + c * 16 : kOutOfRange, 0, 0);
            }
            return;
        }
        const int st0 = base >> rb_log;
        const int rounds = min(kFill, (units - base) / W);  // rounds in which every wave has a unit
        if (rounds == kFill || rounds * W == units - base) {  // and no wave has one beyond them
            const int goff = fill_goff + st0 * 128;
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                if (i >= rounds) break;
                xraw[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, goff + i * fill_dstep * 128, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                if (i > 0 && base + i * W >= units) break;  // uniform: nothing left for any wave
                const int st = st0 + i * fill_dstep;
                xraw[i] = __builtin_amdgcn_raw_buffer_load_b128(
                    xres, st + fill_step0 < ksl ? fill_goff + st * 128 : kOutOfRange, 0, 0);
            }
        }
    };
    [[maybe_unused]] auto fill_store = [&](int base) {
        if (one_row) {
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                if ((i * W + wave) * kWave >= row_chunks) break;
                const int c = (int)threadIdx.x + i * W * kWave;
                if (c < row_chunks) *reinterpret_cast<v4i*>(smem + c * 16) = xraw[i];
            }
            return;
        }
        const int st0 = base >> rb_log;
        if (!fill_has_place) return;
        const int rounds = min(kFill, (units - base) / W);
        if (rounds == kFill || rounds * W == units - base) {
            unsigned char* dst = smem + fill_loff + st0 * step_stride;
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                if (i >= rounds) break;
                *reinterpret_cast<v4i*>(dst + i * fill_dstep * step_stride) = xraw[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                if (i > 0 && base + i * W >= units) break;
                const int st = st0 + i * fill_dstep;
                if (st + fill_step0 < ksl) *reinterpret_cast<v4i*>(smem + fill_loff + st * step_stride) = xraw[i];
            }
        }
    };
    if constexpr (FUSEQ) {
        const uint4* xrow = reinterpret_cast<const uint4*>(a.x_fp16);
        const int chunks = a.K >> 3;
#pragma unroll
        for (int i = 0; i < kFuseChunks; ++i) {
            const int c = (int)threadIdx.x + i * W * kWave;
            xh[i] = c < chunks ? xrow[c] : make_uint4(0u, 0u, 0u, 0u);
        }
    } else {
        fill_load(0);
    }
    __builtin_amdgcn_sched_barrier(0);

    // The channel scales of this workgroup's row tiles pass through LDS in front of the main loop (so that an epilogue in
    // mid-stream never waits on the vector memory counter, behind which the whole weight stream queues).  Up to 32 token
    // rows they are asked for here, in front of the weight stream, so that the LDS writes below wait for them and not
    // for the whole first ring; with four token tiles (8 waves, twice the loads per lane) that costs more than it saves.
    float* lds_cs = reinterpret_cast<float*>(smem + p.cs_offset);
    constexpr int kCsPerThread = 1024 / (W * kWave) * 4;  // 256 row tiles x 16 rows per workgroup at most
    constexpr bool kCsFirst = MT < 4;
    const int cs_words = (t1 - t0) * 16;
    float cs_reg[kCsPerThread];
    auto load_cs = [&]() {
        const rsrc_t cres = make_rsrc(a.chan_scale, a.chan_scale ? (size_t)a.N * 4 : 0);
#pragma unroll
        for (int i = 0; i < kCsPerThread; ++i) {
            if (i > 0 && i * W * kWave >= cs_words) break;  // uniform: a workgroup seldom has more than a few tiles
            const int w = (int)threadIdx.x + i * W * kWave;
            cs_reg[i] = __int_as_float(
                __builtin_amdgcn_raw_buffer_load_b32(cres, w < cs_words ? (t0 * 16 + w) * 4 : kOutOfRange, 0, 0));
        }
    };
    if constexpr (kCsFirst) load_cs();
    issue_state();
    sub_run = sub_i;
#pragma unroll
    for (int u = 0; u < DT; ++u) issue(u);
    issue_advance();
    __builtin_amdgcn_sched_barrier(0);
    PK_MARK(1);
    if (B <= 0) return;  // uniform over the workgroup, before any barrier; its requests lay outside the buffers

    // ---- token scales of this lane's output rows
    float sa[MT][4];
    if constexpr (!FUSEQ) {
        const rsrc_t ares = make_rsrc(a.a_scale, (size_t)a.M * 4);  // rows past M read as zero
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                sa[t][r] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(ares, (16 * t + 4 * kb + r) * 4, 0, 0));
    }
    if constexpr (!kCsFirst) load_cs();
    __builtin_amdgcn_sched_barrier(0);
    PK_MARK(2);

    // ---- activations into LDS
    if constexpr (FUSEQ) {
        // Appendix A.1, n = 8, for the one token: s_a = absmax / 127, codes clamp(rne(x / s_a)) rounded as the true
        // quotient rounds (as the stand-alone quantiser).  With one row the operand order is the natural order of k.
        float* red = reinterpret_cast<float*>(smem + p.cs_offset - 64);
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < kFuseChunks; ++i) amax = fmaxf(amax, absmax8(xh[i]));
        amax = wave_max(amax);
        if (lane == 0) red[wave] = amax;
        lds_barrier();
        float v = red[0];
#pragma unroll
        for (int i = 1; i < W; ++i) v = fmaxf(v, red[i]);
        const float s_a = v / 127.0f;
        const int chunks = a.K >> 3;
#pragma unroll
        for (int i = 0; i < kFuseChunks; ++i) {
            const int c = (int)threadIdx.x + i * W * kWave;
            if (c < chunks) *reinterpret_cast<uint2*>(smem + 8 * c) = quantize8(xh[i], s_a);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) sa[0][r] = s_a;
        if (a.a_scale_out && slab == 0 && t0 == 0 && threadIdx.x == 0) *a.a_scale_out = s_a;  // the owner of tile 0
    } else {
        fill_store(0);
        for (int base = kFill * W; base < units && !one_row; base += kFill * W) {
            fill_load(base);
            fill_store(base);
        }
    }
#pragma unroll
    for (int i = 0; i < kCsPerThread; ++i) {
        if (i > 0 && i * W * kWave >= cs_words) break;
        const int w = (int)threadIdx.x + i * W * kWave;
        if (w < cs_words) lds_cs[w] = a.chan_scale ? cs_reg[i] : 1.0f;
    }
    lds_barrier();
    PK_MARK(3);

    // ---- main loop
    const float inv_alpha = __int_as_float((127 - a.alpha_log2) << 23);  // 2^-alpha_log2, exact
    // (the fused quantiser leaves the whole token in LDS, not just this slab's K steps)
    const int a_lane = kb * 16 * rs + (li & (rs - 1)) * 16 + (FUSEQ ? s_lo * step_stride : 0);
    acc_t acc[MT][4], headp[MT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            acc[t][r] = 0;
            headp[t][r] = 0;
        }
    int head_tile = -1, tail_tile = -1;
    int done_lo = 0, done_hi = 0;  // K split: tiles [done_lo, done_hi) whose slab partial this wave stored whole

    // Epilogue of one row tile from accumulators in MFMA result layout: lane (li, kb) holds weight row 16 tile + li,
    // token rows 16 t + 4 kb .. + 3.
    auto epilogue = [&](int tile, const acc_t (&v)[MT][4]) {
        const int n = tile * 16 + li;
        if (n >= a.N) return;
        const float cc = lds_cs[(tile - t0) * 16 + li] * inv_alpha;
        // Element index of this lane's first output (M <= 64 rows: 32 bits are enough).  Opaque to the compiler, or it
        // keeps one 64-bit address per row and output tensor in registers across the whole K loop.
        int first = 4 * kb * a.N + n;
        asm volatile("" : "+v"(first));
        if constexpr (INT_SCALE) {
            if (a.acc_out) {  // (the diagnostic export of the accumulators: one test per tile, not per output)
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (16 * t + 4 * kb + r < a.M) a.acc_out[first + (16 * t + r) * a.N] = v[t][r];
            }
        }
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = 16 * t + 4 * kb + r;
                if (m < a.M) {
                    float o;
                    if constexpr (INT_SCALE) o = (float)v[t][r] * sa[t][r] * cc;
                    else o = v[t][r] * sa[t][r];
                    a.out[first + (16 * t + r) * a.N] = __float2half_rn(o);
                }
            }
    };
    // K split: a partial tile travels through the workspace as MT x 4 rows of 64 words (one per lane), written and read
    // with device-scope accesses (they go past the L2 of the writer's or reader's own XCD), so that no cache has to be
    // written back or invalidated as a whole.
    auto store_partial = [&](int tile, const acc_t (&v)[MT][4]) {
        int32_t* dst = a.partials + ((size_t)(tile * p.slabs + slab) * MT) * 256 + lane;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int o;
                if constexpr (INT_SCALE) o = v[t][r];
                else o = __float_as_int(v[t][r]);
                __hip_atomic_store(dst + (t * 4 + r) * kWave, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
    };

    // consume cursor
    int rem_c = b1 - b0;
    int tile_c = t0 + q0, step_c = b0 - q0 * ksl;
    int left_c = min(ksl - step_c, rem_c);
    bool seg_whole = step_c == 0 && left_c == ksl;
    bool seg_first = true;
    int a_addr = a_lane + step_c * step_stride;  // LDS address of this lane's first A operand of the next block
    // A operands of one block, from LDS
    auto read_operands = [&](v4i (&xa)[MT][2]) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if constexpr (MT > 1) xa[t][h] = *reinterpret_cast<const v4i*>(smem + a_addr + (t * 2 + h) * 1024);
                else xa[t][h] = *reinterpret_cast<const v4i*>(smem + a_addr + h * unit_b);
            }
        a_addr += step_stride;
    };
    // One block: unpack, multiply, scale step
    auto slot = [&](auto wide_c, int u, const v4i (&xa)[MT][2]) {
        constexpr bool WIDE = decltype(wide_c)::value;
        v4i w_lo, w_hi;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t pk = (uint32_t)wq[u][q];
            w_lo[q] = (int)((pk << 4) & 0xF0F0F0F0u);
            w_hi[q] = (int)(pk & 0xF0F0F0F0u);
        }
        const int s_i = scl[u];
        const float s_f = __int_as_float(s_i) * 0.0625f;  // 16 P * (s / 16) = float(P) * s exactly
        v4i part[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa[t][0], w_lo, v4i{0, 0, 0, 0}, 0, 0, 0);
            part[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa[t][1], w_hi, part[t], 0, 0, 0);
        }
        if constexpr (!INT_SCALE) {
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int r = 0; r < NR; ++r) acc[t][r] = fmaf((float)part[t][r], s_f, acc[t][r]);  // C' += float(C_g) * s_g
        } else if constexpr (WIDE) {
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    int prod = (part[t][r] >> 4) * s_i;
                    asm volatile("" : "+v"(prod));  // else a 64-bit multiply-add with register pairs
                    acc[t][r] += prod;
                }
        } else {
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int r = 0; r < NR; ++r) acc[t][r] = mad_i24(part[t][r] >> 4, s_i, acc[t][r]);  // C'' += C_g * s_g^INT
        }
    };
    // One turn of the ring.  REFILL: every slot, once used, takes the same slot of the next turn (the wave's last turn
    // requests nothing).  FULL: all DT blocks of the turn exist: no block is tested, and the operands of the next block
    // are read from LDS while the current one is multiplied.
    auto turn = [&](auto wide_c, auto refill_c, auto full_c) {
        constexpr bool REFILL = decltype(refill_c)::value;
        constexpr bool FULL = decltype(full_c)::value;
        sub_run = sub_i;
        goff_run = 0;
        v4i xa[2][MT][2];
        if constexpr (FULL) read_operands(xa[0]);
#pragma unroll
        for (int u = 0; u < DT; ++u) {
            if constexpr (FULL) {
                if (u + 1 < DT) read_operands(xa[(u + 1) & 1]);
                slot(wide_c, u, xa[u & 1]);
            } else {
                if (u < left_c) {  // an empty block at the end of a segment is skipped
                    read_operands(xa[0]);
                    slot(wide_c, u, xa[0]);
                }
            }
            if constexpr (REFILL) {
                // The slot's registers are free now.  (Not earlier: a request issued while the old weights or the old
                // scale are still needed gets registers of its own, and the compiler then copies them over behind a
                // wait for the whole ring.)
                __builtin_amdgcn_sched_barrier(0);
                issue(u);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // (the loop exists twice: with the 24-bit multiply of the scale step, and with full 32-bit multiplies)
    auto run_loop = [&](auto wide_c) {
        while (rem_c > 0) {
            if (rem_i > 0) {
                if (left_c >= DT) turn(wide_c, std::true_type{}, std::true_type{});
                else turn(wide_c, std::true_type{}, std::false_type{});
                issue_advance();
            } else {  // nothing is left to request: these blocks are the wave's last
                if (left_c >= DT) turn(wide_c, std::false_type{}, std::true_type{});
                else turn(wide_c, std::false_type{}, std::false_type{});
            }
            const int adv = min(DT, left_c);
            rem_c -= adv;
            step_c += adv;
            left_c -= adv;
            if (left_c == 0) {
                // ---- the segment is complete: its row tile is finished (epilogue, or this slab's partial), or it is one
                // of the two pieces a wave can share with its neighbours (its first and its last segment)
                if (seg_whole) {
                    if (p.slabs == 1) {
                        epilogue(tile_c, acc);
                    } else {
                        store_partial(tile_c, acc);
                        if (done_hi == done_lo) done_lo = tile_c;
                        done_hi = tile_c + 1;
                    }
                } else if (seg_first) {
    #pragma unroll
                    for (int t = 0; t < MT; ++t)
    #pragma unroll
                        for (int r = 0; r < 4; ++r) headp[t][r] = acc[t][r];
                    head_tile = tile_c;
                } else {
                    tail_tile = tile_c;  // a later unfinished segment can only be the wave's last one: it stays in acc
                }
                if (rem_c > 0) {
    #pragma unroll
                    for (int t = 0; t < MT; ++t)
    #pragma unroll
                        for (int r = 0; r < 4; ++r) acc[t][r] = 0;
                    seg_first = false;
                    ++tile_c;
                    step_c = 0;
                    a_addr = a_lane;
                    left_c = min(ksl, rem_c);
                    seg_whole = left_c == ksl;
                }
            }
        }
    };
    if (INT_SCALE && (pk_flags & kPkFlagWide) != 0) run_loop(std::true_type{});
    else run_loop(std::false_type{});
    PK_MARK(4);

    // ---- pieces of row tiles shared by several waves meet in LDS (in the activations' space once nobody reads them
    // any more, or behind them where there is room)
    if (p.slot_offset == 0) lds_barrier();
    // [wave][2][MT][64 lanes][4] words, then one tag per piece: the row tile it belongs to, or -1
    int* slots = reinterpret_cast<int*>(smem + p.slot_offset);
    int* tags = slots + W * 2 * MT * kWave * 4;
    auto slot_ptr = [&](int w, int which, int t) { return slots + (((w * 2 + which) * MT + t) * kWave + lane) * 4; };
    if (head_tile >= 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            v4i o;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (INT_SCALE) o[r] = headp[t][r];
                else o[r] = __float_as_int(headp[t][r]);
            }
            *reinterpret_cast<v4i*>(slot_ptr(wave, 0, t)) = o;
        }
    }
    if (tail_tile >= 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            v4i o;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (INT_SCALE) o[r] = acc[t][r];
                else o[r] = __float_as_int(acc[t][r]);
            }
            *reinterpret_cast<v4i*>(slot_ptr(wave, 1, t)) = o;
        }
    }
    if (lane < 2) tags[wave * 2 + lane] = lane == 0 ? head_tile : tail_tile;
    lds_barrier();
    PK_MARK(5);

    // Wave (tt - t0) mod W adds the pieces of row tile tt, in wave order; a tile without pieces was finished by a
    // single wave in the main loop.  Pieces are found by their tags: lane i < 2 W looks at piece i.
    static_assert(2 * W <= kWave, "one lane per piece tag");
    const int my_tag = lane < 2 * W ? tags[lane] : -1;
    auto shared_tile_sum = [&](int tt, acc_t (&v)[MT][4]) -> bool {
        unsigned long long pieces = __ballot(my_tag == tt);
        if (pieces == 0) return false;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[t][r] = 0;
        while (pieces != 0) {
            // up to four pieces at a time, their reads in flight together
            v4i o[4][MT];
            bool use[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                use[i] = pieces != 0;
                const int idx = use[i] ? __builtin_ctzll(pieces) : 0;
                if (use[i]) pieces &= pieces - 1;
#pragma unroll
                for (int t = 0; t < MT; ++t) o[i][t] = *reinterpret_cast<const v4i*>(slot_ptr(idx >> 1, idx & 1, t));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if constexpr (INT_SCALE) v[t][r] += use[i] ? o[i][t][r] : 0;
                        else v[t][r] += use[i] ? __int_as_float(o[i][t][r]) : 0.0f;
                    }
        }
        return true;
    };

    if (p.slabs == 1) {
        for (int tt = t0 + wave; tt < t1; tt += W) {
            acc_t v[MT][4];
            if (!shared_tile_sum(tt, v)) continue;
            epilogue(tt, v);
        }
        PK_MARK(6);
        return;
    }

    // ---- K split across workgroups: store this workgroup's partial tiles, then raise each tile's arrival counter;
    // whoever arrives last adds the slabs' partials in slab order and runs the epilogue.
    for (int tt = t0 + wave; tt < t1; tt += W) {
        acc_t v[MT][4];
        if (shared_tile_sum(tt, v)) store_partial(tt, v);
    }
    // the partials above (and the ones stored from the main loop) have been written through before a counter is raised
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    auto arrive = [&](int tt) {
        int old = 0;
        if (lane == 0) old = __hip_atomic_fetch_add(a.counters + tt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        old = __builtin_amdgcn_readfirstlane(old);
        if (old != p.slabs - 1) return;
        // the last to arrive: every slab's partial is in the workspace; add them in slab order
        acc_t v[MT][4];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[t][r] = 0;
        // (kSlabsAtOnce slabs' partials are in flight together: a round trip to memory per slab was most of what the
        // last arriver spends; they are added in slab order all the same)
        constexpr int kSlabsAtOnce = MT == 4 ? 2 : 4;
        for (int s0 = 0; s0 < p.slabs; s0 += kSlabsAtOnce) {
            int o[kSlabsAtOnce][MT][4];
#pragma unroll
            for (int u = 0; u < kSlabsAtOnce; ++u) {
                if (u > 0 && s0 + u >= p.slabs) break;  // uniform
                int32_t* src = a.partials + ((size_t)(tt * p.slabs + s0 + u) * MT) * 256 + lane;
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[u][t][r] = __hip_atomic_load(src + (t * 4 + r) * kWave, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int u = 0; u < kSlabsAtOnce; ++u) {
                if (u > 0 && s0 + u >= p.slabs) break;
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if constexpr (INT_SCALE) v[t][r] += o[u][t][r];
                        else v[t][r] += __int_as_float(o[u][t][r]);
                    }
            }
        }
        epilogue(tt, v);
        if (lane == 0) __hip_atomic_store(a.counters + tt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // zero for the next call
    };
    for (int tt = done_lo; tt < done_hi; ++tt) arrive(tt);
    for (int tt = t0 + wave; tt < t1; tt += W)
        if (__ballot(my_tag == tt) != 0) arrive(tt);
    PK_MARK(6);
}

template <int MT, int DT, int WAVES, int NR, bool INT_SCALE, bool FUSEQ>
__global__ __launch_bounds__(WAVES * kWave) void gemm_decode_pk_kernel(PkArgs a, PkKernelPlan p) {
    extern __shared__ __align__(16) unsigned char smem_pk[];
    decode_pk_body<MT, DT, WAVES, NR, INT_SCALE, FUSEQ>(a, p, smem_pk);
}

template <int MT, int DT, int WAVES, int NR, bool INT_SCALE, bool FUSEQ>
hipError_t launch_pk(const PkArgs& a, const PkKernelPlan& kp, const PkPlan& plan, hipStream_t stream) {
    auto kern = gemm_decode_pk_kernel<MT, DT, WAVES, NR, INT_SCALE, FUSEQ>;
    if (plan.lds_bytes > 64 * 1024) {
        static LdsLimit limit;  // per instantiation
        const hipError_t e = limit.raise(reinterpret_cast<const void*>(kern));
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(plan.wg_per_slab, plan.slabs), dim3(WAVES * kWave), plan.lds_bytes, stream, a, kp);
    return hipGetLastError();
}

// Blocks in flight per wave: four token tiles leave registers for six, fewer leave the latency to cover with four.
#ifndef INTSCALE_PK_RING  // (a build-time switch for experiments)
#define INTSCALE_PK_RING 4
#endif
constexpr int ring_depth(int mt) { return mt == 4 ? 6 : INTSCALE_PK_RING; }
// Waves per workgroup the instantiations exist for (dispatch_waves and pk_decode_kernel_name both round with this).
constexpr int waves_instance(int mt, int waves) { return waves <= 4 ? 4 : (waves <= 8 || mt == 4) ? 8 : 16; }

template <bool INT_SCALE, bool FUSEQ, int MT, int NR>
hipError_t dispatch_waves(const PkArgs& a, const PkKernelPlan& kp, const PkPlan& plan, hipStream_t stream) {
    constexpr int DT = ring_depth(MT);
    constexpr bool FQ = MT == 1 && FUSEQ;
    switch (waves_instance(MT, plan.waves)) {
        case 4: return launch_pk<MT, DT, 4, NR, INT_SCALE, FQ>(a, kp, plan, stream);
        case 8: return launch_pk<MT, DT, 8, NR, INT_SCALE, FQ>(a, kp, plan, stream);
        default:
            if constexpr (MT != 4) return launch_pk<MT, DT, 16, NR, INT_SCALE, FQ>(a, kp, plan, stream);
            return hipErrorInvalidValue;
    }
}

template <bool INT_SCALE>
hipError_t dispatch_pk(const PkArgs& a, const PkKernelPlan& kp, const PkPlan& plan, hipStream_t stream) {
    if (a.x_fp16) return dispatch_waves<INT_SCALE, true, 1, 1>(a, kp, plan, stream);
    if (a.M == 1) return dispatch_waves<INT_SCALE, false, 1, 1>(a, kp, plan, stream);
    if (plan.mt == 1) return dispatch_waves<INT_SCALE, false, 1, 4>(a, kp, plan, stream);
    if (plan.mt == 2) return dispatch_waves<INT_SCALE, false, 2, 4>(a, kp, plan, stream);
    return dispatch_waves<INT_SCALE, false, 4, 4>(a, kp, plan, stream);
}

constexpr size_t kActBudget = 128 * 1024;  // LDS bytes for the slab's activations (the fused quantiser's scratch follows)

}  // namespace

// The split of a problem over the chip; false if this kernel does not cover it.
bool pk_decode_plan(int M, int N, int K, int group, bool fp16_in, PkPlan* plan) {
    if (M < 1 || M > 64 || K % 128 != 0 || group % 128 != 0 || K % group != 0) return false;
    if (fp16_in && (M != 1 || (K >> 3) > kFuseChunks * 1024)) return false;
    if (pk_weight_bytes(N, K) >= (1ull << 31)) return false;
    PkPlan pl;
    pl.mt = M <= 16 ? 1 : M <= 32 ? 2 : 4;
    int rows = 16;
    if (pl.mt == 1) {
        rows = 1;
        while (rows < M) rows *= 2;
    }
    pl.rows = rows;
    const int steps = K / 128;
    const int n16 = (N + 15) / 16;
    const int cus = cu_count();
    const size_t per_step = (size_t)rows * pl.mt * 128;
    const int max_steps = (int)(kActBudget / per_step);  // >= 16
    const int s_min = (steps + max_steps - 1) / max_steps;
    // More slabs than the activations need can even out the shares (tiles per workgroup x steps per slab is what a
    // workgroup carries) at the price of more partial tiles: take the best of a few candidates.
    int best = s_min;
    static const int forced = env_int("INTSCALE_PK_SLABS", 0);  // =n (experiments; read once): n slabs, if the activations allow
    double best_cost = 0.0;
    for (int s = s_min; s <= s_min + 4 && s <= steps && s <= cus; ++s) {
        const int wgs = cus / s;
        // In units of one block's time (a CU takes about 23 per microsecond): the blocks a workgroup carries; for a K
        // split about 2 microseconds of store, counter and reload at the end, and its partial tiles, mt KB each, written
        // once and read once; the slab of the activations every workgroup pulls from L2 before its first block (about
        // 2 microseconds for 128 KB).
        const int slab_steps = (steps + s - 1) / s;
        const int wg_tiles = (n16 + wgs - 1) / wgs;
        const double load = (double)wg_tiles * (double)slab_steps;
        const double fill = 46.0 * (double)(per_step * slab_steps) / (double)kActBudget;
        const double cost = load + (s > 1 ? 46.0 + 2.0 * pl.mt * wg_tiles : 0.0) + fill;
        if (s == s_min || cost < best_cost) {
            best = s;
            best_cost = cost;
        }
    }
    if (forced >= s_min && forced <= steps && forced <= cus) best = forced;
    pl.slabs = best;
    pl.wg_per_slab = cus / best;
    if (pl.wg_per_slab < 1) return false;
    if (best > 1 && n16 > kPkMaxTiles) return false;
    pl.max_steps = (steps + best - 1) / best;
    const int tiles_max = (n16 + pl.wg_per_slab - 1) / pl.wg_per_slab;
    if (tiles_max > 256) return false;  // a workgroup stages at most 4096 channel scales
    // Waves per workgroup: enough for every wave to have a full turn of the ring (fewer, fatter waves start sooner and
    // leave fewer pieces to add up), 16 at most; four token tiles need more than 128 registers per lane: 8 at most.
    const int dt = ring_depth(pl.mt);
    const long long blocks = (long long)tiles_max * pl.max_steps;
    int waves = pl.mt == 4 ? 8 : 4;
    while (waves < (pl.mt == 4 ? 8 : 16) && (long long)waves * 2 * dt <= blocks) waves *= 2;
    if (fp16_in)
        while ((K >> 3) > kFuseChunks * waves * kWave) waves *= 2;  // the token's chunks over the threads
    static const int env_waves = env_int("INTSCALE_PK_WAVES", 0);  // experiments; read once
    if (env_waves) {
        const int w = env_waves;
        if ((w == 4 || w == 8 || (w == 16 && pl.mt != 4)) && (!fp16_in || (K >> 3) <= kFuseChunks * w * kWave)) waves = w;
    }
    pl.waves = waves;
    // LDS: [activations of the slab | pieces of shared tiles (behind the activations if there is room, else in their
    // place) | 64 bytes: the waves' absmax | channel scales]
    // (the fused quantiser keeps the whole token in LDS, whatever the slab)
    const size_t act = fp16_in ? (size_t)K : per_step * pl.max_steps;
    const size_t slots = (size_t)pl.waves * 2 * pl.mt * 1024 + 256;  // pieces, then their tags
    const size_t tail = 64 + (size_t)tiles_max * 64;
    if (act + slots + tail <= 160 * 1024) {
        pl.slot_offset = (int)act;
        pl.cs_offset = (int)(act + slots) + 64;
    } else {
        pl.slot_offset = 0;
        pl.cs_offset = (int)(act > slots ? act : slots) + 64;
    }
    pl.lds_bytes = (size_t)pl.cs_offset + (size_t)tiles_max * 64;
    *plan = pl;
    return true;
}

// The instantiation launch_gemm_decode_pk picks for this plan, as a kernel trace names it.
void pk_decode_kernel_name(const PkPlan& plan, bool int_scale, bool fp16_in, char* buf, size_t len) {
    const int mt = fp16_in ? 1 : plan.mt;
    const int nr = fp16_in || (plan.mt == 1 && plan.rows == 1) ? 1 : 4;  // one token row (plan.rows = 1 only then)
    snprintf(buf, len, "gemm_decode_pk_kernel<%d, %d, %d, %d, %s, %s>", mt, ring_depth(mt), waves_instance(mt, plan.waves), nr,
             int_scale ? "true" : "false", fp16_in ? "true" : "false");
}

size_t pk_decode_workspace_bytes(int M, int N, int K, int group) {
    PkPlan pl;
    if (!pk_decode_plan(M, N, K, group, false, &pl) || pl.slabs == 1) return 0;
    return kPkCounterBytes + (size_t)((N + 15) / 16) * pl.slabs * pl.mt * 1024;
}

hipError_t launch_gemm_decode_pk(const PkArgs& a, bool int_scale, hipStream_t stream) {
    PkPlan plan;
    if (!pk_decode_plan(a.M, a.N, a.K, a.group, a.x_fp16 != nullptr, &plan)) return hipErrorInvalidValue;
    PkKernelPlan kp;
    kp.n16 = (a.N + 15) / 16;
    kp.steps = a.K / 128;
    kp.num_groups = a.K / a.group;
    kp.spg = a.group / 128;
    kp.slabs = plan.slabs;
    kp.steps_q = kp.steps / plan.slabs;
    kp.steps_r = kp.steps % plan.slabs;
    kp.tiles_q = kp.n16 / plan.wg_per_slab;
    kp.tiles_r = kp.n16 % plan.wg_per_slab;
    kp.rows = plan.rows;
    kp.cs_offset = plan.cs_offset;
    kp.slot_offset = plan.slot_offset;
    kp.wbytes = pk_weight_bytes(a.N, a.K);
    kp.sbytes = pk_scale_bytes(a.N, a.K, a.group) - kPkHeaderBytes;
    return int_scale ? dispatch_pk<true>(a, kp, plan, stream) : dispatch_pk<false>(a, kp, plan, stream);
}

}  // namespace intscale
