// Shared declarations of the gfx950 implementation (host side of the C ABI and the kernels behind it).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <atomic>

#include "intscale.h"

namespace intscale {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// An environment switch for experiments, as an integer (`unset` when absent).  Callers keep the value in a
// function-local static, so the environment is read once per process and not on every launch.
inline int env_int(const char* name, int unset) {
    const char* v = getenv(name);
    return v ? atoi(v) : unset;
}

// A kernel that uses more than 64 KB of dynamic LDS needs its limit raised, once per kernel and device.  One object per
// kernel (a function-local static of the launcher's instantiation); bit d of `done` = raised on device d.  Safe from
// several host threads: the attribute call is idempotent and the mask is only ever or-ed into.
struct LdsLimit {
    std::atomic<unsigned long long> done{0};
    hipError_t raise(const void* kernel, int bytes = 160 * 1024) {
        int device = -1;
        if (hipGetDevice(&device) != hipSuccess) device = -1;
        const bool tracked = device >= 0 && device < 64;
        if (tracked && ((done.load(std::memory_order_acquire) >> device) & 1ull)) return hipSuccess;
        const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess && tracked) done.fetch_or(1ull << device, std::memory_order_release);
        return e;
    }
};

// Everything a GEMM launch needs. Plain data so that it can be passed by value to a kernel.
struct GemmArgs {
    const int8_t* xq;           // [M,K]
    const float* a_scale;       // [M]
    const uint8_t* qweight;     // [E,N,K/2] int4 pairs, or [E,N,K] int8 codes when w_bits = 8
    const void* scale;          // int32 or float [E,N,NG]
    const float* chan_scale;    // [E,N] or nullptr
    const int32_t* row_offsets; // [E+1] or nullptr (plain GEMM)
    __half* out;                // [M,N]
    int32_t* acc_out;           // [M,N] or nullptr
    int M, N, K, group;
    int alpha_log2;
    int num_experts;
    int w_bits;                 // 4 (W4A8) or 8 (fine-grained W8A8)
    // Linear layer on fp16 activations: the activation quantiser runs inside the GEMM's kernels and xq above is unused.
    // Decode kernel (M = 1 only): a_scale is unused too, a_scale_out (may be nullptr) receives the token's scale.
    // Tiled kernel (plain form, gemm_prefill_takes_fp16(K)): the token scales are written to a_scale_out, and a_scale
    // must be the same pointer.
    const __half* x_fp16 = nullptr;
    float* a_scale_out = nullptr;
};

// Work split of the decode kernel (filled by its launcher).
struct DecodePlan {
    int tiles;       // 16-row weight tiles
    int waves;       // waves per workgroup = K split
    int num_groups;  // K / group
    int gq, gr;      // groups per wave: gq, and one more for the first gr waves
    int spg;         // 128-wide steps per group
    int tiles_q, tiles_r;  // tiles per workgroup: tiles_q, and one more for the first tiles_r workgroups
};

// Launchers (defined next to their kernels). Each returns a hipError_t from the launch.
hipError_t launch_quantize_act(const __half* x, int M, int K, int8_t* xq, float* a_scale, hipStream_t stream);
hipError_t launch_rmsnorm_quantize_act(const __half* x, const __half* gamma, float eps, int M, int K, int8_t* xq,
                                       float* a_scale, hipStream_t stream);
hipError_t launch_silu_mul_quantize_act(const __half* gate_up, int M, int inter, int8_t* xq, float* a_scale,
                                        hipStream_t stream);
hipError_t launch_quantize_weights(const __half* w, int N, int K, int group, int alpha_log2, int scale_mode,
                                   uint8_t* qweight, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                   int* alpha_log2_dev, hipStream_t stream, int bits = 4);  // bits: 4 or 8 (one byte per code)
hipError_t launch_gemm_skinny(const GemmArgs& a, bool int_scale, hipStream_t stream);
// Groups of 32 and 64 (gemm_small_group.hip): one kernel for every M, plain and grouped form.
bool gemm_small_group_covers(int group);
hipError_t launch_gemm_small_group(const GemmArgs& a, bool int_scale, hipStream_t stream);
bool try_launch_gemm_decode(const GemmArgs& a, bool int_scale, hipStream_t stream, hipError_t* err);
// The same with the activation quantiser inside the kernel (a.x_fp16 set, a.M == 1).
bool try_launch_linear_decode(const GemmArgs& a, bool int_scale, hipStream_t stream, hipError_t* err);
// MFMA-bound tiled kernel; `workspace` holds gemm_prefill_workspace_bytes(...) bytes (num_experts = 1 and M = all
// token rows for the plain form).
size_t gemm_prefill_workspace_bytes(int num_experts, int M, int N, int K, int group);
bool gemm_prefill_takes_fp16(int K);
hipError_t launch_gemm_prefill(const GemmArgs& a, bool int_scale, void* workspace, hipStream_t stream);

// Fine-grained W8A8 (gemm_tile_w8.hip): `a.qweight` holds int8 codes [N,K]; one tiled kernel for every M.
size_t gemm_w8_workspace_bytes(int num_experts, int M, int N, int K, int group);
hipError_t launch_gemm_w8(const GemmArgs& a, bool int_scale, void* workspace, hipStream_t stream);
int cu_count();

// Overflow handling (overflow.hip): the layer's worst-case |accumulator| into *bound_dev, and the float scales
// float(IS) * c * 2^-alpha_log2 of the overflow-safe form (`rows` = N, or E * N for stacked weight sets).
hipError_t launch_overflow_bound(const int32_t* scale_i32, int N, int NG, int group, unsigned long long* bound_dev,
                                 hipStream_t stream);
hipError_t launch_derive_safe_scales(const int32_t* scale_i32, const float* chan_scale, size_t rows, int NG,
                                     int alpha_log2, float* out, hipStream_t stream);  // compute units of the current device

// Measurement aids: a streaming read of `bytes` bytes, and a loop of independent int8 MFMAs (*ops = operations done).
hipError_t launch_probe_stream_read(const void* src, size_t bytes, int* sink, hipStream_t stream);
hipError_t launch_probe_mfma_i8(int iters, int* sink, double* ops, hipStream_t stream, bool random_operands = false);

}  // namespace intscale
