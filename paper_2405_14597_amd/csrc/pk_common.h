// The kernel layout of a quantised weight matrix ("prepacked"; written once, offline, by is_prepack_w4) and what the
// kernels that consume it share.  The paper converts the amplified scales to INT32 offline and names an "efficient
// weight processing" step without describing it (Sec. 4.2); this is that step for gfx950.
//
// Weights.  The matrix is cut into blocks of 16 weight rows x 128 k (one MFMA operand pair of a K step), 1 KB each,
// stored [row tile t][K step s].  Inside a block, 16-byte chunk (kb, r) at byte kb * 256 + r * 16 belongs to MFMA
// lane kb * 16 + r: weight row 16 t + r, and in byte j of the chunk
//     bits 0-3 = q[n, 128 s + 16 kb + j]          (first  v_mfma_i32_16x16x64_i8 of the step: k 0..63)
//     bits 4-7 = q[n, 128 s + 64 + 16 kb + j]     (second one: k 64..127)
// as two's-complement nibbles.  So a wave fetches a block with one 16-byte load per lane, fully coalesced, and two
// bit operations per register turn it into the two B operands; the matching A operands are 16 consecutive codes of a
// token row.  Rows past N are zero.
//
// Scales.  [row tile t][group g][16 rows] 32-bit words (integer or float), after a 256-byte header:
//     word 0 = flags (bit 0: some integer scale does not fit 24 signed bits; bit 1: float scales), 1 = N, 2 = K, 3 = group.
// The 16 scales a wave needs with a block are 64 contiguous bytes, and consecutive groups of a tile follow each other.
#pragma once
#include "is_common.h"

namespace intscale {

constexpr int kPkHeaderBytes = 256;
constexpr int kPkFlagWide = 1, kPkFlagFloat = 2, kPkFlagPaired = 4;  // (paired: gate / up rows alternate by 16-row tile)
constexpr int kPkBlockBytes = 1024;
constexpr int kPkMaxExperts = 1024;  // weight sets of the grouped form at most

inline size_t pk_weight_bytes(int N, int K) { return (size_t)((N + 15) / 16) * (size_t)(K / 128) * kPkBlockBytes; }
inline size_t pk_scale_bytes(int N, int K, int group) {
    return kPkHeaderBytes + (size_t)((N + 15) / 16) * (size_t)(K / group) * 64;
}

// Cross-workgroup K split of the decode kernel: the first kPkCounterBytes of its workspace are one arrival counter per
// row tile (zero between calls), the partial accumulators follow.
constexpr size_t kPkCounterBytes = 64 * 1024;
constexpr int kPkMaxTiles = (int)(kPkCounterBytes / 4);

struct PkPlan {
    int waves;        // waves per workgroup
    int mt;           // 16-row token tiles (1, 2, 4)
    int rows;         // token rows kept per tile in LDS (power of two <= 16)
    int slabs;        // K split across workgroups (1 = none)
    int wg_per_slab;  // workgroups per slab
    int max_steps;    // K steps of the longest slab
    int slot_offset;  // LDS byte offset of the pieces of shared tiles (0: in the activations' place)
    int cs_offset;    // LDS byte offset of the workgroup's channel scales
    size_t lds_bytes;
};

// Arguments of the kernels that read the prepacked layout.
struct PkArgs {
    const int8_t* xq;        // [M,K] or nullptr when x_fp16 is given
    const __half* x_fp16;    // [M,K] (one token, quantised in the kernel) or nullptr
    const float* a_scale;    // [M]
    float* a_scale_out;      // x_fp16: receives the token scale (may be nullptr)
    const uint8_t* wpack;    // weights, kernel layout
    const uint8_t* spack;    // scales, kernel layout (header included)
    const float* chan_scale; // [N] or nullptr
    __half* out;             // [M,N]
    int32_t* acc_out;        // [M,N] or nullptr
    int32_t* counters;       // K split: arrival counters per row tile
    int32_t* partials;       // K split: [tile][slab][mt][64 lanes][4]
    int M, N, K, group;
    int alpha_log2;
    // 1: the weight rows alternate gate / up by 16-row tile (is_prepack_w4_gate_up) and the output is
    // fp16(SiLU(gate) * up), [M, N/2]; acc_out stays [M, N] in the packed row order.  Tiled kernel only.
    int pair = 0;
};

bool pk_decode_plan(int M, int N, int K, int group, bool fp16_in, PkPlan* plan);
size_t pk_decode_workspace_bytes(int M, int N, int K, int group);
hipError_t launch_prepack_w4(const uint8_t* qweight, const void* scale, bool float_scales, int N, int K, int group,
                             uint8_t* wpack, uint8_t* spack, hipStream_t stream, int pair_inter = 0,
                             const float* chan_scale = nullptr, float* chan_scale_packed = nullptr);
// out[m, n] = fp16(SiLU(gu[m, 32 p + r]) * gu[m, 32 p + 16 + r]) for n = 16 p + r: the fp16 output of a GEMM on paired rows
// (the route for up to 64 token rows, whose kernel has no fused epilogue)
hipError_t launch_silu_mul_paired(const __half* gu, int M, int N, __half* out, hipStream_t stream);
hipError_t launch_gemm_decode_pk(const PkArgs& a, bool int_scale, hipStream_t stream);
void pk_decode_kernel_name(const PkPlan& plan, bool int_scale, bool fp16_in, char* buf, size_t len);
// MFMA-bound tiled kernel on the prepacked layout (more than 64 token rows); x_fp16 set: a.a_scale_out (= a.a_scale)
// receives the token scales.
size_t gemm_tile_pk_workspace_bytes(int M, int N, int K);   // what the launch makes full use of
size_t gemm_tile_pk_min_workspace_bytes(int M, int K);      // what it needs at least (then without the K split of the last round)
bool gemm_tile_pk_takes_fp16(int K);
hipError_t launch_gemm_tile_pk(const PkArgs& a, bool int_scale, void* workspace, size_t workspace_bytes,
                               hipStream_t stream, bool prepared = false);
// Its preparation of quantised activations alone (then launch_gemm_tile_pk with prepared = true, any number of times).
hipError_t launch_prepare_activations_pk(const int8_t* xq, int M, int K, void* workspace, hipStream_t stream);
// Mixture-of-experts form of the tiled kernel: a.xq / a.a_scale / a.out hold all experts' rows sorted by expert,
// row_offsets (device, [E+1]) their ranges; a.wpack / a.spack point at E prepacked weight sets wstride / sstride bytes
// apart, a.chan_scale at [E][N] (or nullptr).  a.M is the total number of rows.
size_t gemm_tile_grouped_pk_workspace_bytes(int E, int M, int N, int K);
hipError_t launch_gemm_tile_grouped_pk(const PkArgs& a, const int32_t* row_offsets, int E, size_t wstride,
                                       size_t sstride, bool int_scale, void* workspace, hipStream_t stream);
// The kernels launch_gemm_tile_pk runs, in order, as a kernel trace names them, separated by '\n'.
void gemm_tile_pk_kernel_names(int K, bool int_scale, bool fp16_in, char* buf, size_t len, bool silu = false);
void gemm_tile_grouped_pk_kernel_names(int E, int M, bool int_scale, char* buf, size_t len);

}  // namespace intscale
