// C ABI of the library: argument validation (before any HIP call) and dispatch to the gfx950 kernels.
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "is_common.h"
#include "pk_common.h"

using namespace intscale;

// Workspace of the prepacked integer-scale GEMM for callers that cannot allocate.  Every GPU the library runs on holds
// one copy (at its own address) until the process ends; in host code the array's name is only a handle for
// hipGetSymbolAddress (static_scratch below), the kernels get the resolved address.
static __device__ __align__(256) unsigned char scratch[IS_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local char g_hip_error[256] = "";

int hip_status(hipError_t e) {
    if (e == hipSuccess) return IS_OK;
    strncpy(g_hip_error, hipGetErrorString(e), sizeof(g_hip_error) - 1);
    g_hip_error[sizeof(g_hip_error) - 1] = '\0';
    return IS_ERR_HIP;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool ok_ptr(const void* p) { return p != nullptr && aligned16(p); }
inline bool ok_opt(const void* p) { return p == nullptr || aligned16(p); }

// Shape rules shared by all GEMM entry points. Returns IS_OK, IS_ERR_INVALID_ARG or IS_ERR_UNSUPPORTED.
int check_gemm_shape(int M, int N, int K, int group) {
    if (M < 0 || N <= 0 || K <= 0 || group <= 0) return IS_ERR_INVALID_ARG;
    if (K % group != 0 || (K & 1) || (group & 1)) return IS_ERR_INVALID_ARG;
    // the kernels consume K in steps of 128; groups of 32 and 64 have a covering kernel of their own
    if (group % 128 != 0 && !gemm_small_group_covers(group)) return IS_ERR_UNSUPPORTED;
    if (M > (1 << 20)) return IS_ERR_UNSUPPORTED;  // launch-grid limit of the row-chunk dimension
    // the kernels address each tensor (one expert's weights and scales) with 32-bit byte offsets below 2 GB
    if ((long long)N * (K / 2) >= (1LL << 31) || (long long)N * (K / group) * 4 >= (1LL << 31) || K > (1 << 20))
        return IS_ERR_UNSUPPORTED;
    return IS_OK;
}

// Regime selection by the number of token rows.  More than 64 rows (per expert on average, for the grouped form)
// go to the MFMA-bound tiled kernel, which needs workspace for its zero-point corrections.
// Routing override (tests and experiments): 0 automatic, 1 everything the general kernel covers goes to it, 2 the
// W8A8 GEMMs go to the tiled kernel whatever M is, 3 the prepacked calls of 33..64 rows go to the tiled kernel.  Starts from INTSCALE_FORCE_KERNEL=general|tiled, read once;
// is_set_kernel_route changes it afterwards.  Nothing on the launch path reads the environment.
std::atomic<int> g_route{-1};
int kernel_route() {
    int r = g_route.load(std::memory_order_relaxed);
    if (r < 0) {
        const char* force = getenv("INTSCALE_FORCE_KERNEL");
        r = force == nullptr ? 0 : strcmp(force, "general") == 0 ? 1 : strcmp(force, "tiled") == 0 ? 2 : 0;
        int unset = -1;
        if (!g_route.compare_exchange_strong(unset, r)) r = unset;  // (a setter came first)
    }
    return r;
}
bool general_forced() { return kernel_route() == 1; }
bool general_forced_off() { return kernel_route() == 2; }

// Which of the two kernels on the prepacked layout a call takes.  More than 64 token rows: the tiled one.  33..64 rows:
// the weight-streaming kernel cannot keep a long K slab of 64 rows in LDS, so it splits K many times and moves partial
// tiles and activation slabs of about the weights' own size; from 2^27 weights on (measured: LLaMA-2-70B gate 50 -> 47 us,
// down 62 -> 53 us at 64 rows; every smaller shape of the LLaMA-2-7B / LLaMA-3-8B / LLaMA-2-70B layers is slower there)
// the tiled kernel's 64-row instance is ahead.  Same bits either way; route 3 sends every such call there (tests).
bool pk_takes_tile(int M, int N, int K) {
    return M > 64 || (M > 32 && (kernel_route() == 3 || (long long)N * K >= (1LL << 27)));
}

bool wants_prefill(int M, int num_experts, int group) {
    return !general_forced() && !gemm_small_group_covers(group) && M > 64 * num_experts;
}

hipError_t launch_gemm(const GemmArgs& a, bool int_scale, void* workspace, hipStream_t stream) {
    if (gemm_small_group_covers(a.group)) return launch_gemm_small_group(a, int_scale, stream);
    if (wants_prefill(a.M, a.num_experts, a.group)) return launch_gemm_prefill(a, int_scale, workspace, stream);
    hipError_t err = hipSuccess;
    if (!general_forced() && try_launch_gemm_decode(a, int_scale, stream, &err)) return err;
    return launch_gemm_skinny(a, int_scale, stream);
}

__global__ void zero_words_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// This device's copy of `scratch`, resolved once per device with that device current.
int static_scratch(void** ptr_out) {
    constexpr int kMaxDevices = 64;
    static void* resolved[kMaxDevices] = {};
    static std::mutex lock;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return hip_status(e);
    if (device < 0 || device >= kMaxDevices) return IS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(lock);
    if (resolved[device] == nullptr) {  // once per device, with that device current
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_status(e);
        if (p == nullptr) return IS_ERR_HIP;
        resolved[device] = p;
    }
    *ptr_out = resolved[device];
    return IS_OK;
}

}  // namespace

extern "C" {

int is_set_kernel_route(int route) {
    if (route < 0 || route > 3) return IS_ERR_INVALID_ARG;
    const int before = kernel_route();
    g_route.store(route, std::memory_order_relaxed);
    return before;
}

const char* is_status_string(int status) {
    switch (status) {
        case IS_OK: return "IS_OK";
        case IS_ERR_INVALID_ARG: return "IS_ERR_INVALID_ARG";
        case IS_ERR_UNSUPPORTED: return "IS_ERR_UNSUPPORTED";
        case IS_ERR_WORKSPACE: return "IS_ERR_WORKSPACE";
        case IS_ERR_HIP: return "IS_ERR_HIP";
        default: return "IS_ERR_UNKNOWN";
    }
}

const char* is_last_hip_error(void) { return g_hip_error; }

#ifndef INTSCALE_SOURCE_HASH
#define INTSCALE_SOURCE_HASH "0000000000000000"
#endif
const char* is_source_hash(void) {
    static const char tagged[] = "intscale-source-hash:" INTSCALE_SOURCE_HASH;
    return tagged + sizeof("intscale-source-hash:") - 1;
}

int is_probe_stream_read(const void* src, size_t bytes, int* sink, void* stream) {
    if (!ok_ptr(src) || sink == nullptr || (reinterpret_cast<uintptr_t>(sink) & 3u) || bytes == 0 || (bytes & 15))
        return IS_ERR_INVALID_ARG;
    return hip_status(launch_probe_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
}

int is_probe_mfma_i8(int iters, int* sink, double* ops_out, void* stream) {
    if (iters <= 0 || sink == nullptr || (reinterpret_cast<uintptr_t>(sink) & 3u)) return IS_ERR_INVALID_ARG;
    return hip_status(launch_probe_mfma_i8(iters, sink, ops_out, static_cast<hipStream_t>(stream)));
}

int is_probe_mfma_i8_random(int iters, int* sink, double* ops_out, void* stream) {
    if (iters <= 0 || sink == nullptr || (reinterpret_cast<uintptr_t>(sink) & 3u)) return IS_ERR_INVALID_ARG;
    return hip_status(launch_probe_mfma_i8(iters, sink, ops_out, static_cast<hipStream_t>(stream), true));
}

static int quantize_weights_common(const void* w_fp16, int N, int K, int group, int alpha_log2, int scale_mode,
                                   void* qweight, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                   int* alpha_log2_dev, void* stream, int bits) {
    if (!ok_ptr(w_fp16) || !ok_ptr(qweight) || !ok_ptr(scale_f32) || !ok_ptr(scale_i32) || !ok_ptr(chan_scale))
        return IS_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || group <= 0 || K % group != 0 || (K & 1) || (group & 1)) return IS_ERR_INVALID_ARG;
    if (alpha_log2 < IS_ALPHA_HEURISTIC || alpha_log2 > IS_ALPHA_LOG2_MAX) return IS_ERR_INVALID_ARG;
    if (scale_mode != IS_SCALE_RAW && scale_mode != IS_SCALE_NORM) return IS_ERR_INVALID_ARG;
    if (alpha_log2 == IS_ALPHA_HEURISTIC && alpha_log2_dev == nullptr) return IS_ERR_INVALID_ARG;
    if (alpha_log2_dev && (reinterpret_cast<uintptr_t>(alpha_log2_dev) & 3u)) return IS_ERR_INVALID_ARG;
    return hip_status(launch_quantize_weights(static_cast<const __half*>(w_fp16), N, K, group, alpha_log2, scale_mode,
                                              static_cast<uint8_t*>(qweight), scale_f32, scale_i32, chan_scale,
                                              alpha_log2_dev, static_cast<hipStream_t>(stream), bits));
}

int is_quantize_weights_int4_group(const void* w_fp16, int N, int K, int group, int alpha_log2, int scale_mode,
                                   void* qweight, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                   int* alpha_log2_dev, void* stream) {
    return quantize_weights_common(w_fp16, N, K, group, alpha_log2, scale_mode, qweight, scale_f32, scale_i32,
                                   chan_scale, alpha_log2_dev, stream, 4);
}

int is_quantize_weights_int8_group(const void* w_fp16, int N, int K, int group, int alpha_log2, int scale_mode,
                                   int8_t* qweight8, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                   int* alpha_log2_dev, void* stream) {
    return quantize_weights_common(w_fp16, N, K, group, alpha_log2, scale_mode, qweight8, scale_f32, scale_i32,
                                   chan_scale, alpha_log2_dev, stream, 8);
}

int is_quantize_act_int8_token(const void* x_fp16, int M, int K, int8_t* xq, float* a_scale, void* stream) {
    if (M < 0 || K <= 0 || (K & 7)) return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (!ok_ptr(x_fp16) || !ok_ptr(xq) || a_scale == nullptr || (reinterpret_cast<uintptr_t>(a_scale) & 3u))
        return IS_ERR_INVALID_ARG;
    return hip_status(launch_quantize_act(static_cast<const __half*>(x_fp16), M, K, xq, a_scale,
                                          static_cast<hipStream_t>(stream)));
}

int is_rmsnorm_quantize_act_int8_token(const void* x_fp16, const void* gamma_fp16, float eps, int M, int K,
                                       int8_t* xq, float* a_scale, void* stream) {
    if (M < 0 || K <= 0 || (K & 7) || !(eps > 0.0f) || !(eps < INFINITY)) return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (!ok_ptr(x_fp16) || !ok_ptr(gamma_fp16) || !ok_ptr(xq) || a_scale == nullptr ||
        (reinterpret_cast<uintptr_t>(a_scale) & 3u))
        return IS_ERR_INVALID_ARG;
    return hip_status(launch_rmsnorm_quantize_act(static_cast<const __half*>(x_fp16),
                                                  static_cast<const __half*>(gamma_fp16), eps, M, K, xq, a_scale,
                                                  static_cast<hipStream_t>(stream)));
}

int is_silu_mul_quantize_act_int8_token(const void* gate_up_fp16, int M, int inter, int8_t* xq, float* a_scale,
                                        void* stream) {
    if (M < 0 || inter <= 0 || (inter & 7) || inter > (1 << 29)) return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (!ok_ptr(gate_up_fp16) || !ok_ptr(xq) || a_scale == nullptr || (reinterpret_cast<uintptr_t>(a_scale) & 3u))
        return IS_ERR_INVALID_ARG;
    return hip_status(launch_silu_mul_quantize_act(static_cast<const __half*>(gate_up_fp16), M, inter, xq, a_scale,
                                                   static_cast<hipStream_t>(stream)));
}

size_t is_gemm_workspace_bytes(int M, int N, int K, int group) {
    if (check_gemm_shape(M, N, K, group) != IS_OK) return 0;
    // decode-sized problems reduce in LDS and need nothing; the tiled kernel keeps its zero-point corrections, a
    // transposed copy of the scales and a reordered copy of the activations
    return wants_prefill(M, 1, group) ? gemm_prefill_workspace_bytes(1, M, N, K, group) : 0;
}

size_t is_gemm_grouped_workspace_bytes(int num_experts, int M_total, int N, int K, int group) {
    if (num_experts <= 0 || check_gemm_shape(M_total, N, K, group) != IS_OK) return 0;
    return wants_prefill(M_total, num_experts, group) ? gemm_prefill_workspace_bytes(num_experts, M_total, N, K, group) : 0;
}

static int gemm_common(const int8_t* xq, const float* a_scale, const void* qweight, const void* scale,
                       const float* chan_scale, const int32_t* row_offsets, int num_experts, int M, int N, int K,
                       int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                       size_t workspace_bytes, void* stream, bool int_scale, bool grouped) {
    const int shape = check_gemm_shape(M, N, K, group);
    if (shape != IS_OK) return shape;
    if (int_scale && (alpha_log2 < 0 || alpha_log2 > 30)) return IS_ERR_INVALID_ARG;
    if (grouped && (num_experts <= 0 || num_experts > 65535)) return IS_ERR_INVALID_ARG;
    if (!ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    const size_t need = grouped ? is_gemm_grouped_workspace_bytes(num_experts, M, N, K, group)
                                : is_gemm_workspace_bytes(M, N, K, group);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return IS_ERR_WORKSPACE;
    if (!ok_ptr(qweight) || !ok_ptr(scale) || !ok_opt(chan_scale)) return IS_ERR_INVALID_ARG;
    if (grouped && (row_offsets == nullptr || (reinterpret_cast<uintptr_t>(row_offsets) & 3u)))
        return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (!ok_ptr(xq) || a_scale == nullptr || (reinterpret_cast<uintptr_t>(a_scale) & 3u) || !ok_ptr(out_fp16) ||
        !ok_opt(acc_out))
        return IS_ERR_INVALID_ARG;

    GemmArgs a;
    a.xq = xq;
    a.a_scale = a_scale;
    a.qweight = static_cast<const uint8_t*>(qweight);
    a.scale = scale;
    a.chan_scale = chan_scale;
    a.row_offsets = grouped ? row_offsets : nullptr;
    a.out = static_cast<__half*>(out_fp16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.K = K;
    a.group = group;
    a.alpha_log2 = int_scale ? alpha_log2 : 0;
    a.num_experts = grouped ? num_experts : 1;
    a.w_bits = 4;
    return hip_status(launch_gemm(a, int_scale, workspace, static_cast<hipStream_t>(stream)));
}

int is_gemm_w4a8_intscale(const int8_t* xq, const float* a_scale, const void* qweight, const int32_t* scale_i32,
                          const float* chan_scale, int M, int N, int K, int group, int alpha_log2, void* out_fp16,
                          int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_common(xq, a_scale, qweight, scale_i32, chan_scale, nullptr, 1, M, N, K, group, alpha_log2, out_fp16,
                       acc_out, workspace, workspace_bytes, stream, true, false);
}

int is_gemm_w4a8_floatscale(const int8_t* xq, const float* a_scale, const void* qweight, const float* scale_f32,
                            int M, int N, int K, int group, void* out_fp16, void* workspace, size_t workspace_bytes,
                            void* stream) {
    return gemm_common(xq, a_scale, qweight, scale_f32, nullptr, nullptr, 1, M, N, K, group, 0, out_fp16, nullptr,
                       workspace, workspace_bytes, stream, false, false);
}

int is_gemm_w4a8_intscale_grouped(const int8_t* xq, const float* a_scale, const void* qweight,
                                  const int32_t* scale_i32, const float* chan_scale, const int32_t* row_offsets,
                                  int num_experts, int M_total, int N, int K, int group, int alpha_log2,
                                  void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    return gemm_common(xq, a_scale, qweight, scale_i32, chan_scale, row_offsets, num_experts, M_total, N, K, group,
                       alpha_log2, out_fp16, acc_out, workspace, workspace_bytes, stream, true, true);
}

int is_gemm_w4a8_floatscale_grouped(const int8_t* xq, const float* a_scale, const void* qweight,
                                    const float* scale_f32, const int32_t* row_offsets, int num_experts, int M_total,
                                    int N, int K, int group, void* out_fp16, void* workspace, size_t workspace_bytes,
                                    void* stream) {
    return gemm_common(xq, a_scale, qweight, scale_f32, nullptr, row_offsets, num_experts, M_total, N, K, group, 0,
                       out_fp16, nullptr, workspace, workspace_bytes, stream, false, true);
}

// ---- linear layer on fp16 activations: quantiser + GEMM behind one call
static size_t pad_256(size_t n) { return (n + 255) & ~(size_t)255; }

size_t is_linear_workspace_bytes(int M, int N, int K, int group) {
    if (check_gemm_shape(M, N, K, group) != IS_OK || (K & 7)) return 0;
    // quantised activations and token scales for the two-kernel route, then the GEMM's own workspace
    return pad_256((size_t)M * K) + pad_256((size_t)M * 4) + is_gemm_workspace_bytes(M, N, K, group);
}

static int linear_common(const void* x_fp16, const void* qweight, const void* scale, const float* chan_scale, int M,
                         int N, int K, int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                         size_t workspace_bytes, void* stream, bool int_scale) {
    const int shape = check_gemm_shape(M, N, K, group);
    if (shape != IS_OK) return shape;
    if (K & 7) return IS_ERR_INVALID_ARG;
    if (int_scale && (alpha_log2 < 0 || alpha_log2 > 30)) return IS_ERR_INVALID_ARG;
    const size_t need = is_linear_workspace_bytes(M, N, K, group);  // 0 only for M = 0
    if (!ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return IS_ERR_WORKSPACE;
    if (!ok_ptr(qweight) || !ok_ptr(scale) || !ok_opt(chan_scale)) return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (!ok_ptr(x_fp16) || !ok_ptr(out_fp16) || !ok_opt(acc_out)) return IS_ERR_INVALID_ARG;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int8_t* xq = reinterpret_cast<int8_t*>(ws);
    float* sa = reinterpret_cast<float*>(ws + pad_256((size_t)M * K));
    unsigned char* rest = ws + pad_256((size_t)M * K) + pad_256((size_t)M * 4);
    if (M == 1 && !general_forced() && !gemm_small_group_covers(group)) {
        // one token: the decode kernel quantises it itself (every workgroup its own copy, the waves their K slices)
        GemmArgs a;
        a.xq = nullptr;
        a.a_scale = nullptr;
        a.qweight = static_cast<const uint8_t*>(qweight);
        a.scale = scale;
        a.chan_scale = chan_scale;
        a.row_offsets = nullptr;
        a.out = static_cast<__half*>(out_fp16);
        a.acc_out = acc_out;
        a.M = M;
        a.N = N;
        a.K = K;
        a.group = group;
        a.alpha_log2 = int_scale ? alpha_log2 : 0;
        a.num_experts = 1;
        a.w_bits = 4;
        a.x_fp16 = static_cast<const __half*>(x_fp16);
        a.a_scale_out = sa;
        hipError_t err = hipSuccess;
        if (try_launch_linear_decode(a, int_scale, static_cast<hipStream_t>(stream), &err)) return hip_status(err);
    }
    if (wants_prefill(M, 1, group) && gemm_prefill_takes_fp16(K)) {
        // many tokens: the tiled kernel's activation preparation quantises on the way (no canonical codes written)
        GemmArgs a;
        a.xq = nullptr;
        a.a_scale = sa;
        a.qweight = static_cast<const uint8_t*>(qweight);
        a.scale = scale;
        a.chan_scale = chan_scale;
        a.row_offsets = nullptr;
        a.out = static_cast<__half*>(out_fp16);
        a.acc_out = acc_out;
        a.M = M;
        a.N = N;
        a.K = K;
        a.group = group;
        a.alpha_log2 = int_scale ? alpha_log2 : 0;
        a.num_experts = 1;
        a.w_bits = 4;
        a.x_fp16 = static_cast<const __half*>(x_fp16);
        a.a_scale_out = sa;
        return hip_status(launch_gemm_prefill(a, int_scale, rest, static_cast<hipStream_t>(stream)));
    }
    const int st = hip_status(launch_quantize_act(static_cast<const __half*>(x_fp16), M, K, xq, sa,
                                                  static_cast<hipStream_t>(stream)));
    if (st != IS_OK) return st;
    return gemm_common(xq, sa, qweight, scale, chan_scale, nullptr, 1, M, N, K, group, alpha_log2, out_fp16, acc_out,
                       rest, workspace_bytes - (size_t)(rest - ws), stream, int_scale, false);
}

int is_linear_w4a8_intscale(const void* x_fp16, const void* qweight, const int32_t* scale_i32, const float* chan_scale,
                            int M, int N, int K, int group, int alpha_log2, void* out_fp16, int32_t* acc_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return linear_common(x_fp16, qweight, scale_i32, chan_scale, M, N, K, group, alpha_log2, out_fp16, acc_out,
                         workspace, workspace_bytes, stream, true);
}

int is_linear_w4a8_floatscale(const void* x_fp16, const void* qweight, const float* scale_f32, int M, int N, int K,
                              int group, void* out_fp16, void* workspace, size_t workspace_bytes, void* stream) {
    return linear_common(x_fp16, qweight, scale_f32, nullptr, M, N, K, group, 0, out_fp16, nullptr, workspace,
                         workspace_bytes, stream, false);
}

// ---- kernel layout of the weights ("prepacked"): offline conversion, and the GEMMs that consume it
static int check_pk_shape(int N, int K, int group) {
    if (N <= 0 || K <= 0 || group <= 0 || K % group != 0) return IS_ERR_INVALID_ARG;
    if (K % 128 != 0 || group % 128 != 0) return IS_ERR_UNSUPPORTED;  // blocks of 128 k; a block has one group scale
    if (K > (1 << 20) || pk_weight_bytes(N, K) >= (1ull << 31) || pk_scale_bytes(N, K, group) >= (1ull << 31))
        return IS_ERR_UNSUPPORTED;
    return IS_OK;
}

size_t is_prepack_w4_weight_bytes(int N, int K) {
    return check_pk_shape(N, K, 128) == IS_OK ? pk_weight_bytes(N, K) : 0;
}

size_t is_prepack_w4_scale_bytes(int N, int K, int group) {
    return check_pk_shape(N, K, group) == IS_OK ? pk_scale_bytes(N, K, group) : 0;
}

int is_prepack_w4(const void* qweight, const int32_t* scale_i32, const float* scale_f32, int N, int K, int group,
                  void* qweight_packed, void* scales_packed, void* stream) {
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    if ((scale_i32 == nullptr) == (scale_f32 == nullptr)) return IS_ERR_INVALID_ARG;  // exactly one kind of scales
    const void* scale = scale_i32 ? static_cast<const void*>(scale_i32) : static_cast<const void*>(scale_f32);
    if (!ok_ptr(qweight) || !ok_ptr(scale) || !ok_ptr(qweight_packed) || !ok_ptr(scales_packed)) return IS_ERR_INVALID_ARG;
    return hip_status(launch_prepack_w4(static_cast<const uint8_t*>(qweight), scale, scale_f32 != nullptr, N, K, group,
                                        static_cast<uint8_t*>(qweight_packed), static_cast<uint8_t*>(scales_packed),
                                        static_cast<hipStream_t>(stream)));
}

size_t is_gemm_prepacked_workspace_bytes(int M, int N, int K, int group) {
    if (M < 0 || check_pk_shape(N, K, group) != IS_OK) return 0;
    if (M == 0) return 0;
    if (!pk_takes_tile(M, N, K)) return pk_decode_workspace_bytes(M, N, K, group);
    return gemm_tile_pk_workspace_bytes(M, N, K);  // prepared activations, corrections, partial tiles of the last round
}

static int gemm_pk_common(const int8_t* xq, const void* x_fp16, const float* a_scale, float* a_scale_out,
                          const void* wpack, const void* spack, const float* chan_scale, int M, int N, int K, int group,
                          int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                          void* stream, bool int_scale, bool fixed_scratch = false, bool pair = false,
                          bool prepared = false) {
    if (M < 0) return IS_ERR_INVALID_ARG;
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    if (int_scale && (alpha_log2 < 0 || alpha_log2 > 30)) return IS_ERR_INVALID_ARG;
    if (M > (1 << 20)) return IS_ERR_UNSUPPORTED;
    if (!ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    PkPlan plan;
    const bool tiled = pk_takes_tile(M, N, K);
    if (M > 0 && !tiled && !pk_decode_plan(M, N, K, group, x_fp16 != nullptr, &plan)) return IS_ERR_UNSUPPORTED;
    if (tiled && (long long)((M + 15) / 16) * 16 * K >= (1LL << 31)) return IS_ERR_UNSUPPORTED;  // 32-bit offsets
    // (on the fixed scratch the tiled route takes what it needs at least: the K split of its last round uses what is left)
    if (prepared && M > 0 && !tiled) return IS_ERR_UNSUPPORTED;  // (the weight-streaming kernel reads the codes themselves)
    const size_t need = ((fixed_scratch || prepared) && tiled) ? gemm_tile_pk_min_workspace_bytes(M, K)
                                                  : is_gemm_prepacked_workspace_bytes(M, N, K, group);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return IS_ERR_WORKSPACE;
    if (!ok_ptr(wpack) || !ok_ptr(spack) || !ok_opt(chan_scale)) return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (x_fp16 ? !ok_ptr(x_fp16)
               : ((!prepared && !ok_ptr(xq)) || a_scale == nullptr || (reinterpret_cast<uintptr_t>(a_scale) & 3u)))
        return IS_ERR_INVALID_ARG;
    if (!ok_ptr(out_fp16) || !ok_opt(acc_out)) return IS_ERR_INVALID_ARG;
    PkArgs a;
    a.xq = xq;
    a.x_fp16 = static_cast<const __half*>(x_fp16);
    a.a_scale = a_scale;
    a.a_scale_out = a_scale_out;
    a.wpack = static_cast<const uint8_t*>(wpack);
    a.spack = static_cast<const uint8_t*>(spack);
    a.chan_scale = chan_scale;
    a.out = static_cast<__half*>(out_fp16);
    a.acc_out = acc_out;
    a.counters = static_cast<int32_t*>(workspace);
    a.partials = (need > 0 && !tiled) ? reinterpret_cast<int32_t*>(static_cast<unsigned char*>(workspace) + kPkCounterBytes) : nullptr;
    a.M = M;
    a.N = N;
    a.K = K;
    a.group = group;
    a.alpha_log2 = int_scale ? alpha_log2 : 0;
    a.pair = (pair && tiled) ? 1 : 0;  // (the fused epilogue is the tiled kernel's)
    if (tiled)
        return hip_status(launch_gemm_tile_pk(a, int_scale, workspace, workspace_bytes, static_cast<hipStream_t>(stream),
                                              prepared));
    if (fixed_scratch && a.partials != nullptr) {  // a workspace whose last user may not have left the counters zero
        const int n16 = (N + 15) / 16;
        hipLaunchKernelGGL(zero_words_kernel, dim3((n16 + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                           a.counters, n16);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_status(e);
    }
    return hip_status(launch_gemm_decode_pk(a, int_scale, static_cast<hipStream_t>(stream)));
}

int is_gemm_w4a8_intscale_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                    const void* scales_packed, const float* chan_scale, int M, int N, int K, int group,
                                    int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    return gemm_pk_common(xq, nullptr, a_scale, nullptr, qweight_packed, scales_packed, chan_scale, M, N, K, group,
                          alpha_log2, out_fp16, acc_out, workspace, workspace_bytes, stream, true);
}

int is_gemm_w4a8_floatscale_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                      const void* scales_packed, int M, int N, int K, int group, void* out_fp16,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_pk_common(xq, nullptr, a_scale, nullptr, qweight_packed, scales_packed, nullptr, M, N, K, group, 0,
                          out_fp16, nullptr, workspace, workspace_bytes, stream, false);
}

// ---- fused gate / up projection with SiLU(gate) * up as the epilogue (rows paired by is_prepack_w4_gate_up)
int is_prepack_w4_gate_up(const void* qweight, const int32_t* scale_i32, const float* scale_f32, const float* chan_scale,
                          int inter, int K, int group, void* qweight_packed, void* scales_packed,
                          float* chan_scale_packed, void* stream) {
    if (inter <= 0 || inter > (1 << 29)) return IS_ERR_INVALID_ARG;
    if (inter % 16 != 0) return IS_ERR_UNSUPPORTED;  // gate and up tiles alternate by 16 rows
    const int N = 2 * inter;
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    if ((scale_i32 == nullptr) == (scale_f32 == nullptr)) return IS_ERR_INVALID_ARG;  // exactly one kind of scales
    if ((chan_scale == nullptr) != (chan_scale_packed == nullptr)) return IS_ERR_INVALID_ARG;
    if (chan_scale != nullptr && ((reinterpret_cast<uintptr_t>(chan_scale) | reinterpret_cast<uintptr_t>(chan_scale_packed)) & 3u))
        return IS_ERR_INVALID_ARG;
    const void* scale = scale_i32 ? static_cast<const void*>(scale_i32) : static_cast<const void*>(scale_f32);
    if (!ok_ptr(qweight) || !ok_ptr(scale) || !ok_ptr(qweight_packed) || !ok_ptr(scales_packed)) return IS_ERR_INVALID_ARG;
    return hip_status(launch_prepack_w4(static_cast<const uint8_t*>(qweight), scale, scale_f32 != nullptr, N, K, group,
                                        static_cast<uint8_t*>(qweight_packed), static_cast<uint8_t*>(scales_packed),
                                        static_cast<hipStream_t>(stream), inter, chan_scale, chan_scale_packed));
}

size_t is_gemm_gate_up_silu_prepacked_workspace_bytes(int M, int inter, int K, int group) {
    if (M <= 0 || inter <= 0 || inter > (1 << 29) || inter % 16 != 0 || check_pk_shape(2 * inter, K, group) != IS_OK) return 0;
    const size_t gemm = is_gemm_prepacked_workspace_bytes(M, 2 * inter, K, group);
    // up to 64 token rows: the weight-streaming kernel writes the [M, 2 inter] fp16 tensor here, a second kernel reads it
    return !pk_takes_tile(M, 2 * inter, K) ? pad_256(gemm) + pad_256((size_t)M * 2 * inter * 2) : gemm;
}

static int gate_up_silu_common(const int8_t* xq, const float* a_scale, const void* wpack, const void* spack,
                               const float* chan_scale_packed, int M, int inter, int K, int group, int alpha_log2,
                               void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream,
                               bool int_scale) {
    if (M < 0 || inter <= 0 || inter > (1 << 29)) return IS_ERR_INVALID_ARG;
    if (inter % 16 != 0) return IS_ERR_UNSUPPORTED;
    const int N = 2 * inter;
    if (M == 0 || pk_takes_tile(M, N, K))
        return gemm_pk_common(xq, nullptr, a_scale, nullptr, wpack, spack, chan_scale_packed, M, N, K, group, alpha_log2,
                              out_fp16, acc_out, workspace, workspace_bytes, stream, int_scale, false, true);
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    const size_t need = is_gemm_gate_up_silu_prepacked_workspace_bytes(M, inter, K, group);
    if (!ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    if (workspace == nullptr || workspace_bytes < need) return IS_ERR_WORKSPACE;
    if (!ok_ptr(out_fp16)) return IS_ERR_INVALID_ARG;
    const size_t gemm = pad_256(is_gemm_prepacked_workspace_bytes(M, N, K, group));
    __half* gu = reinterpret_cast<__half*>(static_cast<unsigned char*>(workspace) + gemm);
    const int st = gemm_pk_common(xq, nullptr, a_scale, nullptr, wpack, spack, chan_scale_packed, M, N, K, group,
                                  alpha_log2, gu, acc_out, workspace, gemm, stream, int_scale);
    if (st != IS_OK) return st;
    return hip_status(launch_silu_mul_paired(gu, M, N, static_cast<__half*>(out_fp16), static_cast<hipStream_t>(stream)));
}

int is_gemm_w4a8_intscale_gate_up_silu_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                                 const void* scales_packed, const float* chan_scale_packed, int M,
                                                 int inter, int K, int group, int alpha_log2, void* out_fp16,
                                                 int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream) {
    return gate_up_silu_common(xq, a_scale, qweight_packed, scales_packed, chan_scale_packed, M, inter, K, group,
                               alpha_log2, out_fp16, acc_out, workspace, workspace_bytes, stream, true);
}

int is_gemm_w4a8_floatscale_gate_up_silu_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                                   const void* scales_packed, int M, int inter, int K, int group,
                                                   void* out_fp16, void* workspace, size_t workspace_bytes, void* stream) {
    return gate_up_silu_common(xq, a_scale, qweight_packed, scales_packed, nullptr, M, inter, K, group, 0, out_fp16,
                               nullptr, workspace, workspace_bytes, stream, false);
}

int is_prepare_activations_prepacked(const int8_t* xq, int M, int K, void* workspace, size_t workspace_bytes,
                                     void* stream) {
    if (M < 0 || K <= 0) return IS_ERR_INVALID_ARG;
    if (K % 128 != 0 || K > (1 << 20) || M > (1 << 20)) return IS_ERR_UNSUPPORTED;
    if (M > 0 && M <= 32) return IS_ERR_UNSUPPORTED;  // such calls take the weight-streaming kernel, which needs none
    if ((long long)((M + 15) / 16) * 16 * K >= (1LL << 31)) return IS_ERR_UNSUPPORTED;  // 32-bit offsets
    if (M == 0) return IS_OK;
    if (!ok_ptr(workspace) || workspace_bytes < gemm_tile_pk_min_workspace_bytes(M, K)) return IS_ERR_WORKSPACE;
    if (!ok_ptr(xq)) return IS_ERR_INVALID_ARG;
    return hip_status(launch_prepare_activations_pk(xq, M, K, workspace, static_cast<hipStream_t>(stream)));
}

int is_gemm_w4a8_intscale_prepacked_prepared(const float* a_scale, const void* qweight_packed, const void* scales_packed,
                                             const float* chan_scale, int M, int N, int K, int group, int alpha_log2,
                                             void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                             void* stream) {
    return gemm_pk_common(nullptr, nullptr, a_scale, nullptr, qweight_packed, scales_packed, chan_scale, M, N, K, group,
                          alpha_log2, out_fp16, acc_out, workspace, workspace_bytes, stream, true, false, false, true);
}

int is_gemm_w4a8_floatscale_prepacked_prepared(const float* a_scale, const void* qweight_packed,
                                               const void* scales_packed, int M, int N, int K, int group, void* out_fp16,
                                               void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_pk_common(nullptr, nullptr, a_scale, nullptr, qweight_packed, scales_packed, nullptr, M, N, K, group, 0,
                          out_fp16, nullptr, workspace, workspace_bytes, stream, false, false, false, true);
}

int is_gemm_w4a8_intscale_prepacked_noalloc(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                            const void* scales_packed, const float* chan_scale, int M, int N, int K,
                                            int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* stream) {
    if (M < 0) return IS_ERR_INVALID_ARG;
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    const size_t need = pk_takes_tile(M, N, K) ? gemm_tile_pk_min_workspace_bytes(M, K) : is_gemm_prepacked_workspace_bytes(M, N, K, group);
    if (need > (size_t)IS_NOALLOC_SCRATCH_BYTES) return IS_ERR_WORKSPACE;  // beyond the fixed scratch: use the other call
    void* ws = nullptr;
    if (need > 0) {
        const int st = static_scratch(&ws);
        if (st != IS_OK) return st;
    }
    // The array keeps what the last call left: the arrival counters of the K split are cleared on the stream first
    // (by a kernel, so that the call can be captured into a graph); everything else is written before it is read.
    return gemm_pk_common(xq, nullptr, a_scale, nullptr, qweight_packed, scales_packed, chan_scale, M, N, K, group,
                          alpha_log2, out_fp16, acc_out, ws, need > 0 ? (size_t)IS_NOALLOC_SCRATCH_BYTES : 0, stream, true,
                          /*fixed_scratch=*/true);
}

// ---- mixture-of-experts form on the kernel layout: num_experts weight sets, prepacked one by one, back to back
static int check_grouped_pk(int E, int M, int N, int K, int group) {
    if (E <= 0 || M < 0) return IS_ERR_INVALID_ARG;
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    if (E > kPkMaxExperts || M > (1 << 20)) return IS_ERR_UNSUPPORTED;
    if (((long long)(M + 15) / 16 + E) * 16 * K >= (1LL << 31)) return IS_ERR_UNSUPPORTED;  // 32-bit offsets
    return IS_OK;
}

size_t is_gemm_grouped_prepacked_workspace_bytes(int num_experts, int M_total, int N, int K, int group) {
    if (check_grouped_pk(num_experts, M_total, N, K, group) != IS_OK || M_total == 0) return 0;
    return gemm_tile_grouped_pk_workspace_bytes(num_experts, M_total, N, K);
}

static int gemm_grouped_pk_common(const int8_t* xq, const float* a_scale, const void* wpack, const void* spack,
                                  const float* chan_scale, const int32_t* row_offsets, int E, int M, int N, int K,
                                  int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                                  size_t workspace_bytes, void* stream, bool int_scale) {
    const int shape = check_grouped_pk(E, M, N, K, group);
    if (shape != IS_OK) return shape;
    if (int_scale && (alpha_log2 < 0 || alpha_log2 > 30)) return IS_ERR_INVALID_ARG;
    if (row_offsets == nullptr || (reinterpret_cast<uintptr_t>(row_offsets) & 3u)) return IS_ERR_INVALID_ARG;
    if (!ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    const size_t need = is_gemm_grouped_prepacked_workspace_bytes(E, M, N, K, group);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return IS_ERR_WORKSPACE;
    if (!ok_ptr(wpack) || !ok_ptr(spack) || !ok_opt(chan_scale)) return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (!ok_ptr(xq) || a_scale == nullptr || (reinterpret_cast<uintptr_t>(a_scale) & 3u)) return IS_ERR_INVALID_ARG;
    if (!ok_ptr(out_fp16) || !ok_opt(acc_out)) return IS_ERR_INVALID_ARG;
    PkArgs a;
    a.xq = xq;
    a.x_fp16 = nullptr;
    a.a_scale = a_scale;
    a.a_scale_out = nullptr;
    a.wpack = static_cast<const uint8_t*>(wpack);
    a.spack = static_cast<const uint8_t*>(spack);
    a.chan_scale = chan_scale;
    a.out = static_cast<__half*>(out_fp16);
    a.acc_out = acc_out;
    a.counters = nullptr;
    a.partials = nullptr;
    a.M = M;
    a.N = N;
    a.K = K;
    a.group = group;
    a.alpha_log2 = int_scale ? alpha_log2 : 0;
    return hip_status(launch_gemm_tile_grouped_pk(a, row_offsets, E, pk_weight_bytes(N, K), pk_scale_bytes(N, K, group),
                                                  int_scale, workspace, static_cast<hipStream_t>(stream)));
}

int is_gemm_w4a8_intscale_grouped_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                            const void* scales_packed, const float* chan_scale,
                                            const int32_t* row_offsets, int num_experts, int M_total, int N, int K,
                                            int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                                            size_t workspace_bytes, void* stream) {
    return gemm_grouped_pk_common(xq, a_scale, qweight_packed, scales_packed, chan_scale, row_offsets, num_experts,
                                  M_total, N, K, group, alpha_log2, out_fp16, acc_out, workspace, workspace_bytes, stream,
                                  true);
}

int is_gemm_w4a8_floatscale_grouped_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                              const void* scales_packed, const int32_t* row_offsets, int num_experts,
                                              int M_total, int N, int K, int group, void* out_fp16, void* workspace,
                                              size_t workspace_bytes, void* stream) {
    return gemm_grouped_pk_common(xq, a_scale, qweight_packed, scales_packed, nullptr, row_offsets, num_experts, M_total,
                                  N, K, group, 0, out_fp16, nullptr, workspace, workspace_bytes, stream, false);
}

size_t is_linear_prepacked_workspace_bytes(int M, int N, int K, int group) {
    if (M < 0 || check_pk_shape(N, K, group) != IS_OK) return 0;
    if (M == 0) return 0;
    return pad_256((size_t)M * K) + pad_256((size_t)M * 4) + is_gemm_prepacked_workspace_bytes(M, N, K, group);
}

static int linear_pk_common(const void* x_fp16, const void* wpack, const void* spack, const float* chan_scale, int M,
                            int N, int K, int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                            size_t workspace_bytes, void* stream, bool int_scale) {
    if (M < 0) return IS_ERR_INVALID_ARG;
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    const size_t need = is_linear_prepacked_workspace_bytes(M, N, K, group);
    if (!ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return IS_ERR_WORKSPACE;
    if (M == 0) return IS_OK;
    if (!ok_ptr(x_fp16)) return IS_ERR_INVALID_ARG;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int8_t* xq = reinterpret_cast<int8_t*>(ws);
    float* sa = reinterpret_cast<float*>(ws + pad_256((size_t)M * K));
    unsigned char* rest = ws + pad_256((size_t)M * K) + pad_256((size_t)M * 4);
    const size_t rest_bytes = workspace_bytes - (size_t)(rest - ws);
    PkPlan plan;
    if (M == 1 && pk_decode_plan(1, N, K, group, true, &plan))  // one token: quantised inside the GEMM kernel
        return gemm_pk_common(nullptr, x_fp16, nullptr, sa, wpack, spack, chan_scale, M, N, K, group, alpha_log2,
                              out_fp16, acc_out, rest, rest_bytes, stream, int_scale);
    if (M > 64 && gemm_tile_pk_takes_fp16(K))  // many tokens: the tiled kernel's preparation quantises on the way (a
                                               // workgroup per 8 rows: too few of them below that)
        return gemm_pk_common(nullptr, x_fp16, sa, sa, wpack, spack, chan_scale, M, N, K, group, alpha_log2, out_fp16,
                              acc_out, rest, rest_bytes, stream, int_scale);
    // the arguments of the GEMM are checked before the quantiser is enqueued
    if (!ok_ptr(wpack) || !ok_ptr(spack) || !ok_opt(chan_scale) || !ok_ptr(out_fp16) || !ok_opt(acc_out))
        return IS_ERR_INVALID_ARG;
    if (int_scale && (alpha_log2 < 0 || alpha_log2 > 30)) return IS_ERR_INVALID_ARG;
    if (!pk_takes_tile(M, N, K) && !pk_decode_plan(M, N, K, group, false, &plan)) return IS_ERR_UNSUPPORTED;
    const int st = hip_status(launch_quantize_act(static_cast<const __half*>(x_fp16), M, K, xq, sa,
                                                  static_cast<hipStream_t>(stream)));
    if (st != IS_OK) return st;
    return gemm_pk_common(xq, nullptr, sa, nullptr, wpack, spack, chan_scale, M, N, K, group, alpha_log2, out_fp16,
                          acc_out, rest, rest_bytes, stream, int_scale);
}

int is_linear_w4a8_intscale_prepacked(const void* x_fp16, const void* qweight_packed, const void* scales_packed,
                                      const float* chan_scale, int M, int N, int K, int group, int alpha_log2,
                                      void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                      void* stream) {
    if (K & 7) return IS_ERR_INVALID_ARG;
    return linear_pk_common(x_fp16, qweight_packed, scales_packed, chan_scale, M, N, K, group, alpha_log2, out_fp16,
                            acc_out, workspace, workspace_bytes, stream, true);
}

int is_linear_w4a8_floatscale_prepacked(const void* x_fp16, const void* qweight_packed, const void* scales_packed, int M,
                                        int N, int K, int group, void* out_fp16, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    if (K & 7) return IS_ERR_INVALID_ARG;
    return linear_pk_common(x_fp16, qweight_packed, scales_packed, nullptr, M, N, K, group, 0, out_fp16, nullptr,
                            workspace, workspace_bytes, stream, false);
}

int is_describe_prepacked(int M, int N, int K, int group, int int_scale, int fp16_in, char* names, size_t names_len) {
    if (names == nullptr || names_len == 0) return IS_ERR_INVALID_ARG;
    names[0] = '\0';
    if (M < 1) return IS_ERR_INVALID_ARG;
    const int shape = check_pk_shape(N, K, group);
    if (shape != IS_OK) return shape;
    if (pk_takes_tile(M, N, K)) {
        gemm_tile_pk_kernel_names(K, int_scale != 0, fp16_in != 0 && M > 64 && gemm_tile_pk_takes_fp16(K), names, names_len);
        return IS_OK;
    }
    PkPlan plan;
    const bool fused = fp16_in != 0 && M == 1 && pk_decode_plan(1, N, K, group, true, &plan);
    if (!fused && !pk_decode_plan(M, N, K, group, false, &plan)) return IS_ERR_UNSUPPORTED;
    pk_decode_kernel_name(plan, int_scale != 0, fused, names, names_len);
    return IS_OK;
}

int is_describe_grouped_prepacked(int num_experts, int M_total, int N, int K, int group, int int_scale, char* names,
                                  size_t names_len) {
    if (names == nullptr || names_len == 0) return IS_ERR_INVALID_ARG;
    names[0] = '\0';
    if (M_total < 1) return IS_ERR_INVALID_ARG;
    const int shape = check_grouped_pk(num_experts, M_total, N, K, group);
    if (shape != IS_OK) return shape;
    gemm_tile_grouped_pk_kernel_names(num_experts, M_total, int_scale != 0, names, names_len);
    return IS_OK;
}

// ---- fine-grained W8A8
static int check_w8_shape(int M, int N, int K, int group) {
    if (M < 0 || N <= 0 || K <= 0 || group <= 0 || K % group != 0) return IS_ERR_INVALID_ARG;
    if (group % 128 != 0) return IS_ERR_UNSUPPORTED;
    if (M > (1 << 20) || K > (1 << 20) || (long long)N * (K / group) * 4 >= (1LL << 31)) return IS_ERR_UNSUPPORTED;
    if ((long long)N * K >= (1LL << 31)) return IS_ERR_UNSUPPORTED;  // the kernel's weight offsets are 32-bit
    return IS_OK;
}

size_t is_gemm_w8a8_workspace_bytes(int M, int N, int K, int group) {
    return check_w8_shape(M, N, K, group) == IS_OK ? gemm_w8_workspace_bytes(1, M, N, K, group) : 0;
}

static int gemm_w8_common(const int8_t* xq, const float* a_scale, const int8_t* qweight8, const void* scale,
                          const float* chan_scale, int M, int N, int K, int group, int alpha_log2, void* out_fp16,
                          int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream, bool int_scale) {
    const int shape = check_w8_shape(M, N, K, group);
    if (shape != IS_OK) return shape;
    if (int_scale && (alpha_log2 < 0 || alpha_log2 > 30)) return IS_ERR_INVALID_ARG;
    if (!ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    if (workspace == nullptr || workspace_bytes < gemm_w8_workspace_bytes(1, M, N, K, group)) return IS_ERR_WORKSPACE;
    if (!ok_ptr(qweight8) || !ok_ptr(scale) || !ok_opt(chan_scale)) return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    if (!ok_ptr(xq) || a_scale == nullptr || (reinterpret_cast<uintptr_t>(a_scale) & 3u) || !ok_ptr(out_fp16) ||
        !ok_opt(acc_out))
        return IS_ERR_INVALID_ARG;
    GemmArgs a;
    a.xq = xq;
    a.a_scale = a_scale;
    a.qweight = reinterpret_cast<const uint8_t*>(qweight8);
    a.scale = scale;
    a.chan_scale = chan_scale;
    a.row_offsets = nullptr;
    a.out = static_cast<__half*>(out_fp16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.K = K;
    a.group = group;
    a.alpha_log2 = int_scale ? alpha_log2 : 0;
    a.num_experts = 1;
    a.w_bits = 8;
    // up to 64 token rows the layer is a weight stream: the bandwidth-bound general kernel; else the tiled kernel
    if (M <= 64 && !general_forced_off())
        return hip_status(launch_gemm_skinny(a, int_scale, static_cast<hipStream_t>(stream)));
    return hip_status(launch_gemm_w8(a, int_scale, workspace, static_cast<hipStream_t>(stream)));
}

int is_gemm_w8a8_intscale(const int8_t* xq, const float* a_scale, const int8_t* qweight8, const int32_t* scale_i32,
                          const float* chan_scale, int M, int N, int K, int group, int alpha_log2, void* out_fp16,
                          int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_w8_common(xq, a_scale, qweight8, scale_i32, chan_scale, M, N, K, group, alpha_log2, out_fp16, acc_out,
                          workspace, workspace_bytes, stream, true);
}

int is_gemm_w8a8_floatscale(const int8_t* xq, const float* a_scale, const int8_t* qweight8, const float* scale_f32, int M,
                            int N, int K, int group, void* out_fp16, void* workspace, size_t workspace_bytes,
                            void* stream) {
    return gemm_w8_common(xq, a_scale, qweight8, scale_f32, nullptr, M, N, K, group, 0, out_fp16, nullptr, workspace,
                          workspace_bytes, stream, false);
}

size_t is_gemm_safe_workspace_bytes(int M, int N, int K, int group) {
    if (check_gemm_shape(M, N, K, group) != IS_OK) return 0;
    // the derived float scales, then whatever the GEMM itself needs
    return (((size_t)N * (K / group) * 4 + 255) & ~(size_t)255) + is_gemm_workspace_bytes(M, N, K, group);
}

int is_gemm_w4a8_intscale_safe(const int8_t* xq, const float* a_scale, const void* qweight, const int32_t* scale_i32,
                               const float* chan_scale, int M, int N, int K, int group, int alpha_log2,
                               void* out_fp16, void* workspace, size_t workspace_bytes, void* stream) {
    const int shape = check_gemm_shape(M, N, K, group);
    if (shape != IS_OK) return shape;
    if (alpha_log2 < 0 || alpha_log2 > 30) return IS_ERR_INVALID_ARG;
    if (!ok_ptr(scale_i32) || !ok_opt(chan_scale) || !ok_opt(workspace)) return IS_ERR_INVALID_ARG;
    if (workspace == nullptr || workspace_bytes < is_gemm_safe_workspace_bytes(M, N, K, group)) return IS_ERR_WORKSPACE;
    const size_t scales_bytes = ((size_t)N * (K / group) * 4 + 255) & ~(size_t)255;
    float* derived = static_cast<float*>(workspace);
    // the arguments of the GEMM itself are checked before anything is enqueued
    if (!ok_ptr(qweight)) return IS_ERR_INVALID_ARG;
    if (M > 0 && (!ok_ptr(xq) || a_scale == nullptr || (reinterpret_cast<uintptr_t>(a_scale) & 3u) || !ok_ptr(out_fp16)))
        return IS_ERR_INVALID_ARG;
    if (M == 0) return IS_OK;
    const int st = hip_status(launch_derive_safe_scales(scale_i32, chan_scale, (size_t)N, K / group, alpha_log2, derived,
                                                        static_cast<hipStream_t>(stream)));
    if (st != IS_OK) return st;
    return gemm_common(xq, a_scale, qweight, derived, nullptr, nullptr, 1, M, N, K, group, 0, out_fp16, nullptr,
                       static_cast<unsigned char*>(workspace) + scales_bytes, workspace_bytes - scales_bytes, stream, false,
                       false);
}

int is_intscale_overflow_bound(const int32_t* scale_i32, int N, int K, int group, unsigned long long* bound_dev,
                               void* stream) {
    if (N <= 0 || K <= 0 || group <= 0 || K % group != 0) return IS_ERR_INVALID_ARG;
    if (!ok_ptr(scale_i32) || bound_dev == nullptr || (reinterpret_cast<uintptr_t>(bound_dev) & 7u))
        return IS_ERR_INVALID_ARG;
    return hip_status(launch_overflow_bound(scale_i32, N, K / group, group, bound_dev, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
