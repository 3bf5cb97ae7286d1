/*
 * intscale.h — C ABI of the fine-grained W4A8 linear layer with integer group scales on MI355X (gfx950).
 *
 * The layer follows the Integer Scale paper: int8 per-token activations times int4 weights quantised in groups
 * of `group` along K, where every float group scale s_g is replaced by the integer INT(s_g * alpha) so that the
 * per-group int32 partial sums are scaled and accumulated in int32 and converted to float once per output
 * (Eq. (2), Table 2 column "Ours").  The float-scale form (Eq. (1), Table 2 column "Atom") is exported as the
 * baseline, built on the same kernels.
 *
 * Conventions for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, 16-byte aligned, dense row-major.
 *     The library allocates nothing and never synchronises.  No result depends on an earlier call; the process state
 *     it does keep is housekeeping: the compute-unit count of the device (read once), which kernels have had their
 *     LDS limit raised on which device, the resolved address of the fixed scratch of the *_noalloc call, the routing
 *     override of is_set_kernel_route, and the environment switches INTSCALE_FORCE_KERNEL / INTSCALE_PK_SLABS /
 *     INTSCALE_PK_WAVES / INTSCALE_TILE_PARTS / INTSCALE_SKINNY_* (tests and experiments; unset in production), each
 *     read once per process, at its first use: no launch reads the environment.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Return value: IS_OK, or a negative IS_ERR_* code.  Arguments are validated before any HIP call; on an
 *     argument error nothing is enqueued and the outputs are untouched.
 *   - Notation: X is [M,K] (tokens x in-features), W is [N,K] (out-features x in-features, so the layer is
 *     X * W^T as in Eq. (1)); groups run along K; NG = K / group; alpha = 2^alpha_log2.
 *   - Rounding is round-half-to-even everywhere; the quantisers divide in IEEE fp32.
 *   - Group sizes.  The quantisers take any even group size that divides K (Appendix A.2).  The W4A8 GEMMs and linear
 *     calls on the canonical layouts (plain, grouped, overflow-safe) take multiples of 128, and 32 and 64; other sizes
 *     return IS_ERR_UNSUPPORTED.  Groups of 32 and 64 run one covering kernel for every M (one matrix instruction and
 *     one scale step per group; no workspace), not the tuned kernels: the paper measures group 128 only (Sec. 5.1,
 *     Table 1).  The calls on the kernel layout (is_prepack_w4 and *_prepacked) and W8A8 take multiples of 128 only.
 *   - Values the device computes stay on the device: the amplifier found by the heuristic search is written to a
 *     DEVICE int (alpha_log2_dev), not returned through a host pointer, because returning it would force a
 *     synchronisation inside the call; read it back when convenient.
 *
 * Canonical layouts
 *   qweight    uint8 [N, K/2]   byte j of row n = q[n,2j] in bits 0-3 | q[n,2j+1] in bits 4-7, two's-complement nibbles
 *   scale_f32  float [N, NG]    s[n,g] = max|w| over the group / 7                      (Appendix A.1, n = 4)
 *   scale_i32  int32 [N, NG]    INT(s * alpha) (RAW) or INT(s / c[n] * alpha) (NORM)    (Eq. (2))
 *   chan_scale float [N]        c[n]: 1 (RAW) or max_g s[n,g] (NORM)
 *   xq         int8  [M, K]     a_scale float [M]: s_a[m] = max|x| over the row / 127    (Appendix A.1, n = 8)
 *   out        fp16  [M, N]     acc int32 [M, N]
 */
#ifndef INTSCALE_H_
#define INTSCALE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IS_OK 0
#define IS_ERR_INVALID_ARG (-1) /* NULL / misaligned pointer, non-positive or inconsistent sizes, bad enum */
#define IS_ERR_UNSUPPORTED (-2) /* valid request outside what the kernels cover (see each function) */
#define IS_ERR_WORKSPACE (-3)   /* workspace_bytes < is_gemm_workspace_bytes(...) or workspace NULL while needed */
#define IS_ERR_HIP (-4)         /* a HIP call failed (no device, launch failure); see is_last_hip_error() */

#define IS_SCALE_RAW 0  /* IS = INT(s * alpha), c = 1: Eq. (2) as printed */
#define IS_SCALE_NORM 1 /* c[n] = max_g s[n,g]; IS = INT(s / c * alpha): scales normalised into (0,1] (Sec. 4.1) */

#define IS_ALPHA_HEURISTIC (-1) /* alpha_log2 value that selects the amplifier search of Sec. 4.1 / Listing 1 */
#define IS_ALPHA_LOG2_MAX 16

/*
 * Offline weight preparation: group-wise symmetric int4 quantisation (Appendix A.1, A.2; group size 128 in
 * Sec. 5) followed by the integer-scale derivation INT(s * alpha) (Eq. (2)).
 *   w_fp16        in   fp16 [N,K]
 *   group         even, divides K
 *   alpha_log2    0..16, or IS_ALPHA_HEURISTIC: the smallest i >= 0 with (smallest non-zero amplified value) * 2^i >= 1,
 *                 capped at 16 (Sec. 4.1); this needs alpha_log2_dev
 *   scale_mode    IS_SCALE_RAW or IS_SCALE_NORM
 *   qweight, scale_f32, scale_i32, chan_scale   out, canonical layouts above
 *   alpha_log2_dev  out, device int*, may be NULL unless the heuristic is requested: the log2 actually used
 * An all-zero group gets s = 0, q = 0, IS = 0.  Inputs must be finite.
 */
int is_quantize_weights_int4_group(const void* w_fp16, int N, int K, int group, int alpha_log2, int scale_mode,
                                   void* qweight, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                   int* alpha_log2_dev, void* stream);

/*
 * Online activation quantisation: per-token symmetric int8 (Appendix A.1 with n = 8; per-token in Sec. 5.1).
 *   x_fp16 in fp16 [M,K], K a multiple of 8;  xq out int8 [M,K];  a_scale out float [M].
 * M = 0 is a no-op.  An all-zero row gets s_a = 0 and codes 0.  Inputs must be finite.
 */
int is_quantize_act_int8_token(const void* x_fp16, int M, int K, int8_t* xq, float* a_scale, void* stream);

/*
 * The activation quantiser folded into the operator that produces the activation (the kernel fusion of Sec. 4.3 and
 * Sec. 5.2).  Each call returns exactly what its producer, an fp16 tensor and is_quantize_act_int8_token would,
 * without the fp16 tensor's trip through memory.  The producer's arithmetic is a fixed sequence of separately
 * rounded single-precision operations, because its fp16 value decides integer codes:
 *
 * RMSNorm:  y[m,k] = fp16( (x[m,k] * r[m]) * gamma[k] ),  r[m] = 1 / sqrt( float(sum_k x[m,k]^2 / K) + eps ),
 *           the sum of squares taken in double precision.
 *   x_fp16 in fp16 [M,K], K a multiple of 8;  gamma_fp16 in fp16 [K];  eps > 0 and finite;
 *   xq out int8 [M,K];  a_scale out float [M].
 *
 * SiLU * up:  h[m,i] = fp16( (g / (1 + e)) * u ),  g = gate_up[m,i], u = gate_up[m,inter+i], e = exp(-g) computed as
 *           t = clamp(-g, -87, 88), n = rint(t * log2 e), r = (t - n * 0.693145751953125) - n * 1.428606765330187e-06,
 *           the degree-6 Taylor polynomial of e^r by Horner's rule, times 2^n.
 *   gate_up_fp16 in fp16 [M, 2*inter] (gate half, then up half, of every row), inter a multiple of 8;
 *   xq out int8 [M,inter];  a_scale out float [M].
 *
 * M = 0 is a no-op.  A row whose products are all zero gets s_a = 0 and codes 0.  Inputs must be finite and the
 * fp16 results must not overflow.
 */
int is_rmsnorm_quantize_act_int8_token(const void* x_fp16, const void* gamma_fp16, float eps, int M, int K,
                                       int8_t* xq, float* a_scale, void* stream);
int is_silu_mul_quantize_act_int8_token(const void* gate_up_fp16, int M, int inter, int8_t* xq, float* a_scale,
                                        void* stream);

/*
 * Fine-grained W4A8 GEMM with integer scales (Eq. (2); Table 2 "Ours"):
 *   P[m,n,g] = sum_{k in group g} xq[m,k] * q[n,k]                    int32, exact
 *   acc[m,n] = sum_g P[m,n,g] * scale_i32[n,g]                        int32, wraps modulo 2^32
 *   out[m,n] = fp16( float(acc[m,n]) * a_scale[m] * chan_scale[n] * 2^-alpha_log2 )
 *   chan_scale   may be NULL (all ones)
 *   acc_out      may be NULL; otherwise receives the raw int32 accumulators [M,N]
 *   workspace    device scratch of at least is_gemm_workspace_bytes(M,N,K,group) bytes (may be NULL when that is 0)
 * Requirements: group a multiple of 128, or 32 or 64, dividing K (group = K gives the coarse-grained GEMM of
 * Table 2's first column); 0 <= alpha_log2 <= 30; N >= 1; M >= 0 (M = 0 is a no-op).
 * Any int32 scale is accepted and multiplied exactly modulo 2^32.
 */
int is_gemm_w4a8_intscale(const int8_t* xq, const float* a_scale, const void* qweight, const int32_t* scale_i32,
                          const float* chan_scale, int M, int N, int K, int group, int alpha_log2, void* out_fp16,
                          int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fine-grained W4A8 GEMM with float scales, the baseline (Eq. (1); Table 2 "Atom"):
 *   out[m,n] = fp16( a_scale[m] * sum_g float(P[m,n,g]) * scale_f32[n,g] )    accumulated in fp32
 * Same tiling, layouts and requirements as is_gemm_w4a8_intscale.
 */
int is_gemm_w4a8_floatscale(const int8_t* xq, const float* a_scale, const void* qweight, const float* scale_f32,
                            int M, int N, int K, int group, void* out_fp16, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * The linear layer on fp16 activations: is_quantize_act_int8_token followed by is_gemm_w4a8_intscale (or the
 * float-scale twin), behind one call and with the same results to the bit (Appendix A.1 per token, then Eq. (2) or
 * Eq. (1)).  For one token (M = 1, a decode step at batch 1) whose K the decode kernel covers, the quantiser runs
 * inside the GEMM kernel and no other kernel is launched; for more than 64 tokens with K <= 32768 the tiled kernel's
 * activation preparation quantises on the way; otherwise the two kernels run one after the other.
 *   x_fp16 in fp16 [M,K], K a multiple of 8;  the other arguments as for the GEMMs
 *   workspace    device scratch of at least is_linear_workspace_bytes(M,N,K,group) bytes (never 0 for M > 0): it
 *                receives the quantised activations [M,K], then (256-byte aligned) the token scales [M], then the
 *                GEMM's own workspace; the routes that quantise inside the GEMM write only the token scales
 */
size_t is_linear_workspace_bytes(int M, int N, int K, int group);
int is_linear_w4a8_intscale(const void* x_fp16, const void* qweight, const int32_t* scale_i32, const float* chan_scale,
                            int M, int N, int K, int group, int alpha_log2, void* out_fp16, int32_t* acc_out,
                            void* workspace, size_t workspace_bytes, void* stream);
int is_linear_w4a8_floatscale(const void* x_fp16, const void* qweight, const float* scale_f32, int M, int N, int K,
                              int group, void* out_fp16, void* workspace, size_t workspace_bytes, void* stream);

/* Scratch the two GEMMs above need for this shape (0 when they need none). Returns 0 for invalid shapes. */
size_t is_gemm_workspace_bytes(int M, int N, int K, int group);

/*
 * Kernel layout of a quantised weight matrix ("prepacked").  Sec. 4.2 converts the amplified scales to INT32 offline
 * and passes the weights through an "efficient weight processing" it does not describe; here that offline step
 * reorders both tensors into the order the gfx950 kernels consume them (same bytes, N padded to 16):
 *   qweight_packed   [ceil(N/16)] [K/128] blocks of 1 KB = 16 weight rows x 128 k; in a block, the 16 bytes at
 *                    (kb * 16 + r) * 16 hold row 16 t + r: byte j = q[n, 128 s + 16 kb + j] (bits 0-3) |
 *                    q[n, 128 s + 64 + 16 kb + j] (bits 4-7), two's-complement nibbles; rows past N are zero
 *   scales_packed    256-byte header (word 0: flags, bit 0 = some integer scale needs more than 24 signed bits,
 *                    bit 1 = float scales; words 1-3: N, K, group), then [ceil(N/16)] [K/group] [16 rows] 32-bit words
 * is_prepack_w4 takes the canonical qweight and exactly one of scale_i32 / scale_f32 (the other NULL); pack the same
 * weights twice to have both forms.  Sizes: is_prepack_w4_weight_bytes, is_prepack_w4_scale_bytes (0 for shapes that
 * are not covered).  Requirements: K and group multiples of 128 (IS_ERR_UNSUPPORTED otherwise: a 128-wide block has one
 * group scale per row), group dividing K, packed tensors below 2 GB.
 */
size_t is_prepack_w4_weight_bytes(int N, int K);
size_t is_prepack_w4_scale_bytes(int N, int K, int group);
int is_prepack_w4(const void* qweight, const int32_t* scale_i32, const float* scale_f32, int N, int K, int group,
                  void* qweight_packed, void* scales_packed, void* stream);

/*
 * The GEMMs of Eq. (2) and Eq. (1) on prepacked weights: same arithmetic and results as is_gemm_w4a8_intscale /
 * is_gemm_w4a8_floatscale (accumulators bit for bit; the float-scale sums in a different but fixed order).
 *   qweight_packed, scales_packed   from is_prepack_w4 (integer scales for the first, float scales for the second)
 *   workspace   at least is_gemm_prepacked_workspace_bytes(M,N,K,group) bytes.
 *               (Which kernel: the tiled one for M > 64, and for 33 <= M <= 64 when N * K >= 2^27; else the
 *               weight-streaming one.  Ask is_gemm_prepacked_workspace_bytes / is_describe_prepacked, do not guess.)
 *               M <= 64 (the weight-streaming kernel): 0 for most shapes; when it is not 0 the K dimension is split
 *               across workgroups and the first 64 KB of the workspace are arrival counters: they must be ZERO when a
 *               call starts and every call leaves them zero, so zero the workspace once after allocating it.
 *               M > 64 (the MFMA-bound tiled kernel): the activations re-ordered into MFMA operand blocks
 *               (ceil(M/16) * 16 * K bytes) and one zero-point correction per token row and K step, written by a
 *               preparation kernel of the call; when the last round of output tiles would leave most of the chip idle,
 *               also partial tiles (up to 64 MB) of a K split of that round, reduced exactly in int32 (the float-scale
 *               form adds its float partial sums in a fixed order).  No requirement on the contents.
 *               Calls sharing one workspace must not overlap.
 * Covered: M >= 1, N up to 16 * 256 * (compute units) rows when M <= 64, ceil(M/16) * 16 * K below 2^31 beyond
 * (IS_ERR_UNSUPPORTED otherwise).  M = 0 is a no-op.
 */
size_t is_gemm_prepacked_workspace_bytes(int M, int N, int K, int group);
int is_gemm_w4a8_intscale_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                    const void* scales_packed, const float* chan_scale, int M, int N, int K, int group,
                                    int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                                    size_t workspace_bytes, void* stream);
int is_gemm_w4a8_floatscale_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                      const void* scales_packed, int M, int N, int K, int group, void* out_fp16,
                                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Activations that several GEMMs share (the q / k / v or the gate / up projections of one layer input): the tiled
 * route's preparation of the quantised activations, done once, and the prepacked GEMMs on the prepared workspace,
 * which then launch the tiled kernel alone.  Same arithmetic and results as the calls above (Eq. (2) / Eq. (1)), bit
 * for bit.
 *   is_prepare_activations_prepacked   xq int8 [M,K] -> the front part of `workspace`, whose size depends on M and K
 *       only (MFMA operand blocks, zero-point corrections, zeroed arrival counters).  M > 32, K a multiple of
 *       128, ceil(M/16) * 16 * K below 2^31 (IS_ERR_UNSUPPORTED otherwise).
 *   is_gemm_w4a8_*_prepacked_prepared  as is_gemm_w4a8_*_prepacked without xq, on a workspace prepared for the same
 *       M and K; any number of calls, with any N and weights, may follow one preparation, one after the other on the
 *       same stream (each leaves the workspace prepared).  Only shapes that take the tiled kernel (M > 64, or
 *       33 <= M <= 64 with N * K >= 2^27): IS_ERR_UNSUPPORTED otherwise, use the ordinary call.
 *   workspace   the same buffer for all of them, at least is_gemm_prepacked_workspace_bytes(M, N, K, group) bytes of the
 *       widest N (less is accepted down to the size for N = 1: the last round's K split then uses what there is).
 */
int is_prepare_activations_prepacked(const int8_t* xq, int M, int K, void* workspace, size_t workspace_bytes,
                                     void* stream);
int is_gemm_w4a8_intscale_prepacked_prepared(const float* a_scale, const void* qweight_packed, const void* scales_packed,
                                             const float* chan_scale, int M, int N, int K, int group, int alpha_log2,
                                             void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                             void* stream);
int is_gemm_w4a8_floatscale_prepacked_prepared(const float* a_scale, const void* qweight_packed,
                                               const void* scales_packed, int M, int N, int K, int group, void* out_fp16,
                                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * is_gemm_w4a8_intscale_prepacked for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results, without the workspace: the
 * call uses a fixed scratch array inside the library (IS_NOALLOC_SCRATCH_BYTES of device memory per GPU, held until
 * the process ends) and allocates nothing, on the device or through any library.
 *   - Shapes whose is_gemm_prepacked_workspace_bytes(M,N,K,group) exceeds IS_NOALLOC_SCRATCH_BYTES return
 *     IS_ERR_WORKSPACE before anything is enqueued (covered: every M <= 64 shape, and tiled shapes up to about
 *     ceil(M/16) * 16 * K = 31 MiB; the tiled route splits its last round only as far as the rest of the scratch allows).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads)
 *     race on it; serialise them or give the overlapping ones the workspace form.
 *   - The first call on a device resolves the array's address (hipGetSymbolAddress); make that call outside a graph
 *     capture.  The K split's arrival counters are cleared by a small kernel of the call, not by a memset.
 */
#define IS_NOALLOC_SCRATCH_BYTES (32u << 20)
int is_gemm_w4a8_intscale_prepacked_noalloc(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                            const void* scales_packed, const float* chan_scale, int M, int N, int K,
                                            int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* stream);

/*
 * The linear layer on fp16 activations and prepacked weights: Appendix A.1 per token, then Eq. (2) / Eq. (1), with the
 * results of is_quantize_act_int8_token followed by the prepacked GEMM, to the bit.  One token (M = 1, K <= 32768) is
 * quantised inside the GEMM kernel (one launch); more than 64 tokens are quantised by the tiled kernel's preparation
 * pass; otherwise the quantiser runs first.
 *   workspace   at least is_linear_prepacked_workspace_bytes(M,N,K,group) bytes: quantised activations [M,K], token
 *               scales [M] (each padded to 256 bytes), then the GEMM's workspace, whose zero-counter rule applies.
 */
size_t is_linear_prepacked_workspace_bytes(int M, int N, int K, int group);
int is_linear_w4a8_intscale_prepacked(const void* x_fp16, const void* qweight_packed, const void* scales_packed,
                                      const float* chan_scale, int M, int N, int K, int group, int alpha_log2,
                                      void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                      void* stream);
int is_linear_w4a8_floatscale_prepacked(const void* x_fp16, const void* qweight_packed, const void* scales_packed, int M,
                                        int N, int K, int group, void* out_fp16, void* workspace,
                                        size_t workspace_bytes, void* stream);

/*
 * Mixture-of-experts form on the kernel layout (Sec. 5.4): as is_gemm_w4a8_*_grouped, with the `num_experts` weight
 * sets prepacked one by one by is_prepack_w4 and stored back to back: expert e's weights at qweight_packed +
 * e * is_prepack_w4_weight_bytes(N,K), its scales (header included) at scales_packed + e * is_prepack_w4_scale_bytes(
 * N,K,group).  chan_scale [E,N] (may be NULL), row_offsets device int32 [E+1] as for the canonical grouped calls.
 * Every row count takes the MFMA-bound tiled kernel with 128-row tiles per expert (the call is built for prefill-sized
 * batches; for a handful of rows per expert the canonical grouped call streams the weights better).  The workspace
 * (is_gemm_grouped_prepacked_workspace_bytes, contents arbitrary) receives the activations re-ordered into MFMA
 * operand blocks with every expert padded to whole 16-row tiles, the zero-point corrections and a table of the row
 * tiles.  Limits: num_experts <= 1024, (ceil(M_total/16) + num_experts) * 16 * K below 2^31.
 */
size_t is_gemm_grouped_prepacked_workspace_bytes(int num_experts, int M_total, int N, int K, int group);
int is_gemm_w4a8_intscale_grouped_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                            const void* scales_packed, const float* chan_scale,
                                            const int32_t* row_offsets, int num_experts, int M_total, int N, int K,
                                            int group, int alpha_log2, void* out_fp16, int32_t* acc_out, void* workspace,
                                            size_t workspace_bytes, void* stream);
int is_gemm_w4a8_floatscale_grouped_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                              const void* scales_packed, const int32_t* row_offsets, int num_experts,
                                              int M_total, int N, int K, int group, void* out_fp16, void* workspace,
                                              size_t workspace_bytes, void* stream);

/*
 * Fused gate / up projection of a gated feed-forward block with SiLU(gate) * up as the GEMM's epilogue (Sec. 4.2 names
 * kernel fusion around the GEMM; the LLaMA and Mixtral blocks of Sec. 5 are of this form).
 *   is_prepack_w4_gate_up: qweight [2 inter, K/2], scales [2 inter, K/group] and chan_scale [2 inter] (may be NULL,
 *     then chan_scale_packed must be NULL too) of the fused projection in canonical order, rows [0, inter) the gate's
 *     and [inter, 2 inter) the up's.  Writes the kernel layout of is_prepack_w4 with the rows paired: packed rows
 *     32 p .. 32 p + 15 are gate rows 16 p .. 16 p + 15, packed rows 32 p + 16 .. 32 p + 31 the up rows of the same
 *     outputs; chan_scale_packed [2 inter] receives the channel scales in that order.  Buffer sizes as for
 *     is_prepack_w4 with N = 2 inter.  inter must be a multiple of 16 (IS_ERR_UNSUPPORTED otherwise).
 *   is_gemm_w4a8_*_gate_up_silu_prepacked: out [M, inter] fp16, out[m, n] = fp16(SiLU(g) * u) with g, u the fp16
 *     results of the integer-scale (float-scale) GEMM of Eq. (2) (Eq. (1)) for gate row n and up row n: the value of
 *     the unfused sequence GEMM -> fp16 tensor -> SiLU * up, bit for bit, without the [M, 2 inter] tensor's trip
 *     through memory when M > 64 (the epilogue of the tiled kernel; for M <= 64 the weight-streaming kernel writes
 *     that tensor into the workspace and a second kernel reads it).  SiLU(g) = g / (1 + e^-g) in single precision,
 *     e^-g by the operation sequence stated in the oracle.  acc_out (may be NULL): [M, 2 inter] int32 accumulators
 *     in the packed row order.  workspace >= is_gemm_gate_up_silu_prepacked_workspace_bytes(M, inter, K, group),
 *     zero-filled once (same rules as the prepacked GEMM's).
 */
int is_prepack_w4_gate_up(const void* qweight, const int32_t* scale_i32, const float* scale_f32, const float* chan_scale,
                          int inter, int K, int group, void* qweight_packed, void* scales_packed,
                          float* chan_scale_packed, void* stream);
size_t is_gemm_gate_up_silu_prepacked_workspace_bytes(int M, int inter, int K, int group);
int is_gemm_w4a8_intscale_gate_up_silu_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                                 const void* scales_packed, const float* chan_scale_packed, int M,
                                                 int inter, int K, int group, int alpha_log2, void* out_fp16,
                                                 int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream);
int is_gemm_w4a8_floatscale_gate_up_silu_prepacked(const int8_t* xq, const float* a_scale, const void* qweight_packed,
                                                   const void* scales_packed, int M, int inter, int K, int group,
                                                   void* out_fp16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Which kernels the prepacked calls launch for a shape, as a kernel trace (rocprofv3 --kernel-trace) names them, in
 * launch order and separated by '\n' (the stand-alone activation quantiser of the linear call for 2 <= M <= 64, when
 * it runs, is not listed).  Host-only: nothing is launched.  int_scale: Eq. (2) or Eq. (1) form; fp16_in: the linear
 * call rather than the GEMM call.  Writes a NUL-terminated string of at most names_len bytes.
 */
int is_describe_prepacked(int M, int N, int K, int group, int int_scale, int fp16_in, char* names, size_t names_len);
/* The same for the grouped prepacked calls (the tile shape depends on the rows per expert on average). */
int is_describe_grouped_prepacked(int num_experts, int M_total, int N, int K, int group, int int_scale, char* names,
                                  size_t names_len);

/*
 * Mixture-of-experts form (Sec. 5.4 measures Mixtral 8x7B): one launch over `num_experts` weight sets.
 * Rows of xq are sorted by expert; rows [row_offsets[e], row_offsets[e+1]) use weight set e.
 *   qweight [E,N,K/2], scale_i32 / scale_f32 [E,N,NG], chan_scale [E,N] (may be NULL)
 *   row_offsets   device int32 [E+1], non-decreasing, row_offsets[0] = 0, row_offsets[E] = M_total
 *   M_total       number of rows of xq / out (the host does not read row_offsets)
 * Other arguments and requirements as for the plain GEMMs.
 */
int is_gemm_w4a8_intscale_grouped(const int8_t* xq, const float* a_scale, const void* qweight,
                                  const int32_t* scale_i32, const float* chan_scale, const int32_t* row_offsets,
                                  int num_experts, int M_total, int N, int K, int group, int alpha_log2,
                                  void* out_fp16, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                  void* stream);
int is_gemm_w4a8_floatscale_grouped(const int8_t* xq, const float* a_scale, const void* qweight,
                                    const float* scale_f32, const int32_t* row_offsets, int num_experts, int M_total,
                                    int N, int K, int group, void* out_fp16, void* workspace, size_t workspace_bytes,
                                    void* stream);
size_t is_gemm_grouped_workspace_bytes(int num_experts, int M_total, int N, int K, int group);

/*
 * Fine-grained W8A8 (int8 weights in groups along K; the paper's LLaMA-3 recipe uses it for the down-projection
 * layers, Sec. 5.5 / Table 5).  Same equations with n = 8 on the weight side (Appendix A.1):
 *   s = max|w| over the group / 127,  q = clamp(rne(w / s), -128, 127),  integer scales as for int4.
 *   qweight8   int8 [N, K], one code per byte, row-major; the other tensors as in the canonical layouts above
 * is_quantize_weights_int8_group takes the arguments and requirements of is_quantize_weights_int4_group.
 * The GEMMs compute Eq. (2) resp. Eq. (1) exactly as their W4A8 counterparts (a group's partial sum is at most 2^21
 * in magnitude, so the same integer scale step applies); group and K multiples of 128, any M >= 0, any N >= 1;
 * `workspace` of at least is_gemm_w8a8_workspace_bytes(M,N,K,group) bytes is always needed (transposed scales).
 */
int is_quantize_weights_int8_group(const void* w_fp16, int N, int K, int group, int alpha_log2, int scale_mode,
                                   int8_t* qweight8, float* scale_f32, int32_t* scale_i32, float* chan_scale,
                                   int* alpha_log2_dev, void* stream);
int is_gemm_w8a8_intscale(const int8_t* xq, const float* a_scale, const int8_t* qweight8, const int32_t* scale_i32,
                          const float* chan_scale, int M, int N, int K, int group, int alpha_log2, void* out_fp16,
                          int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream);
int is_gemm_w8a8_floatscale(const int8_t* xq, const float* a_scale, const int8_t* qweight8, const float* scale_f32, int M,
                            int N, int K, int group, void* out_fp16, void* workspace, size_t workspace_bytes,
                            void* stream);
size_t is_gemm_w8a8_workspace_bytes(int M, int N, int K, int group);

/*
 * Overflow risk of a layer (Sec. 5.6, the appendix on maximum activations, Limitations): the largest |accumulator|
 * the integer-scale GEMM can reach with these integer scales over all int8 activation codes and int4 weight codes,
 *   bound = max_n sum_g |scale_i32[n,g]| * group * 128 * 8
 * (a group's partial sum is at most group * 128 * 8 in magnitude).  The int32 accumulator cannot overflow iff
 * bound < 2^31.  A property of the weights alone: meant to be asked once, offline, per layer and amplifier.
 *   scale_i32   in   int32 [N, K/group]        bound_dev   out  device unsigned 64-bit integer, 8-byte aligned
 */
int is_intscale_overflow_bound(const int32_t* scale_i32, int N, int K, int group, unsigned long long* bound_dev,
                               void* stream);

/*
 * Overflow-safe form of the integer-scale GEMM, for layers whose bound is too large: the "degraded" kernel of the
 * Limitations section, which keeps the integer scales but takes the amplifier out group by group, so that nothing is
 * accumulated in 32 bits:
 *   out[m,n] = fp16( a_scale[m] * sum_g float(P[m,n,g]) * (float(scale_i32[n,g]) * chan_scale[n] * 2^-alpha_log2) )
 * accumulated in fp32 (the per-group conversions of Eq. (1) are back: this is the price).  Arguments as for
 * is_gemm_w4a8_intscale, without acc_out; workspace of at least is_gemm_safe_workspace_bytes(M,N,K,group) bytes
 * (never 0: it holds the derived scales).
 */
int is_gemm_w4a8_intscale_safe(const int8_t* xq, const float* a_scale, const void* qweight, const int32_t* scale_i32,
                               const float* chan_scale, int M, int N, int K, int group, int alpha_log2,
                               void* out_fp16, void* workspace, size_t workspace_bytes, void* stream);
size_t is_gemm_safe_workspace_bytes(int M, int N, int K, int group);

/*
 * Measurement aids (no part of the method): the two rates the GEMMs are priced against, as this chip delivers them.
 *   is_probe_stream_read  reads `bytes` bytes (a multiple of 16) at `src` (device) once, 16 bytes per lane
 *   is_probe_mfma_i8      every wave of a chip-filling launch issues `iters` rounds of 16 independent
 *                         v_mfma_i32_16x16x64_i8 on registers; *ops_out (host, may be NULL) = int8 operations done
 *   is_probe_mfma_i8_random  the same loop on operands that differ from one MFMA to the next (pseudo-random bytes):
 *                         the chip lowers its clock when the matrix pipe's inputs toggle, so this is the rate a real
 *                         contraction can reach, the one above the rate at the highest clock
 * `sink` is a device int the kernels may write (4-byte aligned).  Each enqueues one kernel on `stream`; time them with
 * events.  Errors as for the other calls.
 */
int is_probe_stream_read(const void* src, size_t bytes, int* sink, void* stream);
int is_probe_mfma_i8(int iters, int* sink, double* ops_out, void* stream);
int is_probe_mfma_i8_random(int iters, int* sink, double* ops_out, void* stream);

/*
 * For tests and experiments (not part of the method): which kernel the calls on the canonical layouts take.
 *   0  the library chooses by shape (the default);
 *   1  every call goes to the general kernel where it covers the shape;
 *   2  the W8A8 GEMMs go to the tiled kernel whatever M is;
 *   3  the prepacked calls of 33..64 token rows go to the tiled kernel whatever the size of the weights.
 * The setting is process-wide and starts from INTSCALE_FORCE_KERNEL=general|tiled (read once).  Returns the setting
 * that was in force before, or IS_ERR_INVALID_ARG.  Results do not depend on it (every route computes the same bits).
 */
int is_set_kernel_route(int route);

/* Human-readable name of a status code (static storage). */
const char* is_status_string(int status);
/* Text of the last HIP error this thread's calls ran into (static storage; "" if none). */
const char* is_last_hip_error(void);
/* Digest (16 hex digits) of the sources this library was compiled from; the Python binding rebuilds when it differs
 * from the digest of the sources beside it. */
const char* is_source_hash(void);

#ifdef __cplusplus
}
#endif
#endif /* INTSCALE_H_ */
