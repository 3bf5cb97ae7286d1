"""numpy front end of the CPU oracle (oracle_is.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module
and this module never imports the product package.

Every function takes and returns host numpy arrays in the canonical layouts
documented at the top of oracle_is.c.  fp16 inputs are widened to fp32 (exact)
before they reach the C code; fp16 outputs are produced by one correctly
rounded double -> half conversion (Eq. (2): the single FLOAT conversion and
the activation de-quantisation happen once per output).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import NamedTuple, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_is.c")
_LIB = os.path.join(_HERE, "liboracle_is.so")

SCALE_RAW = 0    # IS = round(s * alpha), c = 1                    (Eq. (2) as printed)
SCALE_NORM = 1   # c[n] = max_g s[n,g]; IS = round(s / c * alpha)  (scales normalised into (0,1], Sec. 4.1)


def build(force: bool = False) -> str:
    """Compile oracle_is.c with gcc (plain loops, OpenMP over rows). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-mavx2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.oracle_amplifier_log2.argtypes = [vp, ctypes.c_long]
        lib.oracle_amplifier_log2.restype = ci
        lib.oracle_quantize_weights_int4_group.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp]
        lib.oracle_quantize_weights_int4_group.restype = ci
        lib.oracle_quantize_act_int8_token.argtypes = [vp, ci, ci, vp, vp]
        lib.oracle_quantize_act_int8_token.restype = ci
        lib.oracle_group_partials.argtypes = [vp, vp, ci, ci, ci, ci, vp]
        lib.oracle_group_partials.restype = ci
        lib.oracle_gemm_w4a8_intscale.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp]
        lib.oracle_gemm_w4a8_intscale.restype = ci
        lib.oracle_gemm_w4a8_floatscale.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp]
        lib.oracle_gemm_w4a8_floatscale.restype = ci
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _check(status: int, what: str) -> None:
    if status != 0:
        raise ValueError(f"oracle {what}: invalid argument (status {status})")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


class QuantizedWeights(NamedTuple):
    qweight: np.ndarray      # uint8 [N, K/2]
    scale_f32: np.ndarray    # float32 [N, K/G]
    scale_i32: np.ndarray    # int32 [N, K/G]
    chan_scale: np.ndarray   # float32 [N]
    alpha_log2: int


def amplifier_log2(scales: np.ndarray) -> int:
    """Sec. 4.1 / Listing 1: log2 of the first power of two that lifts the smallest non-zero scale to >= 1."""
    s = _c(np.asarray(scales).reshape(-1), np.float32)
    return int(_load().oracle_amplifier_log2(_ptr(s), s.size))


def quantize_weights_int4_group(w: np.ndarray, group: int, alpha_log2: int, scale_mode: int = SCALE_RAW
                                ) -> QuantizedWeights:
    """Appendix A.1 (n = 4) per (row, group of `group` along K), then INT(s * alpha) of Eq. (2).

    alpha_log2 = -1 selects the heuristic amplifier of Sec. 4.1.
    """
    w32 = _c(w, np.float32)
    N, K = w32.shape
    if K % group != 0 or K % 2 != 0:
        raise ValueError("oracle quantize_weights: K must be even and a multiple of group")
    NG = K // group
    q = np.zeros((N, K // 2), dtype=np.uint8)
    s = np.zeros((N, NG), dtype=np.float32)
    si = np.zeros((N, NG), dtype=np.int32)
    c = np.zeros((N,), dtype=np.float32)
    a_out = ctypes.c_int(0)
    st = _load().oracle_quantize_weights_int4_group(_ptr(w32), N, K, group, alpha_log2, scale_mode, _ptr(q), _ptr(s),
                                                   _ptr(si), _ptr(c), ctypes.addressof(a_out))
    _check(st, "quantize_weights_int4_group")
    return QuantizedWeights(q, s, si, c, int(a_out.value))


def quantize_act_int8_token(x: np.ndarray):
    """Appendix A.1 (n = 8) per token row. Returns (xq int8 [M,K], a_scale float32 [M])."""
    x32 = _c(x, np.float32)
    M, K = x32.shape
    xq = np.zeros((M, K), dtype=np.int8)
    sa = np.zeros((M,), dtype=np.float32)
    _check(_load().oracle_quantize_act_int8_token(_ptr(x32), M, K, _ptr(xq), _ptr(sa)), "quantize_act_int8_token")
    return xq, sa


def unpack_int4(qweight: np.ndarray) -> np.ndarray:
    """Canonical packed bytes [N,K/2] -> int8 codes [N,K] (even k in the low nibble, two's complement)."""
    q = np.asarray(qweight, dtype=np.uint8)
    lo = (q & 0xF).astype(np.int16)
    hi = (q >> 4).astype(np.int16)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty((q.shape[0], q.shape[1] * 2), dtype=np.int8)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out


def pack_int4(q: np.ndarray) -> np.ndarray:
    """int codes [N,K] in [-8,7] -> canonical packed bytes [N,K/2]."""
    q = np.asarray(q).astype(np.int16)
    if q.min(initial=0) < -8 or q.max(initial=0) > 7:
        raise ValueError("int4 code out of range")
    u = (q & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


def group_partials(xq: np.ndarray, qweight: np.ndarray, group: int) -> np.ndarray:
    """P[m,n,g] = sum over group g of xq[m,k] * q[n,k]  (Table 2: C_g = A_g W_g). int32 [M,N,K/G]."""
    xq = _c(xq, np.int8)
    qweight = _c(qweight, np.uint8)
    M, K = xq.shape
    N = qweight.shape[0]
    p = np.zeros((M, N, K // group), dtype=np.int32)
    _check(_load().oracle_group_partials(_ptr(xq), _ptr(qweight), M, N, K, group, _ptr(p)), "group_partials")
    return p


class IntScaleResult(NamedTuple):
    acc: np.ndarray          # int32 [M,N], the wrapped 32-bit accumulators
    out: np.ndarray          # float64 [M,N], before the final rounding to fp16
    out_fp16: np.ndarray     # float16 [M,N]
    acc64: np.ndarray        # int64 [M,N], the sum without wrap
    max_prefix: np.ndarray   # int64 [M,N], max_g |prefix sum|


def gemm_w4a8_intscale(xq, a_scale, qweight, scale_i32, chan_scale, group: int, alpha_log2: int) -> IntScaleResult:
    """Eq. (2) with the Table 2 "Ours" recurrence; chan_scale may be None (c = 1)."""
    xq = _c(xq, np.int8)
    a_scale = _c(a_scale, np.float32)
    qweight = _c(qweight, np.uint8)
    scale_i32 = _c(scale_i32, np.int32)
    cs = None if chan_scale is None else _c(chan_scale, np.float32)
    M, K = xq.shape
    N = qweight.shape[0]
    if qweight.shape[1] * 2 != K or scale_i32.shape != (N, K // group) or a_scale.shape != (M,):
        raise ValueError("oracle gemm_w4a8_intscale: shape mismatch")
    if cs is not None and cs.shape != (N,):
        raise ValueError("oracle gemm_w4a8_intscale: chan_scale shape mismatch")
    acc = np.zeros((M, N), dtype=np.int32)
    out = np.zeros((M, N), dtype=np.float64)
    acc64 = np.zeros((M, N), dtype=np.int64)
    peak = np.zeros((M, N), dtype=np.int64)
    st = _load().oracle_gemm_w4a8_intscale(_ptr(xq), _ptr(a_scale), _ptr(qweight), _ptr(scale_i32), _ptr(cs), M, N, K,
                                          group, alpha_log2, _ptr(acc), _ptr(out), _ptr(acc64), _ptr(peak))
    _check(st, "gemm_w4a8_intscale")
    with np.errstate(over="ignore"):
        out16 = out.astype(np.float16)
    return IntScaleResult(acc, out, out16, acc64, peak)


class FloatScaleResult(NamedTuple):
    out: np.ndarray          # float64 [M,N]
    out_fp16: np.ndarray     # float16 [M,N]
    abs_sum: np.ndarray      # float64 [M,N], s_a * sum_g |P_g| s_g


def gemm_w4a8_floatscale(xq, a_scale, qweight, scale_f32, group: int) -> FloatScaleResult:
    """Eq. (1) with the Table 2 "Atom" recurrence, accumulated in double."""
    xq = _c(xq, np.int8)
    a_scale = _c(a_scale, np.float32)
    qweight = _c(qweight, np.uint8)
    scale_f32 = _c(scale_f32, np.float32)
    M, K = xq.shape
    N = qweight.shape[0]
    if qweight.shape[1] * 2 != K or scale_f32.shape != (N, K // group) or a_scale.shape != (M,):
        raise ValueError("oracle gemm_w4a8_floatscale: shape mismatch")
    out = np.zeros((M, N), dtype=np.float64)
    mag = np.zeros((M, N), dtype=np.float64)
    st = _load().oracle_gemm_w4a8_floatscale(_ptr(xq), _ptr(a_scale), _ptr(qweight), _ptr(scale_f32), M, N, K, group,
                                            _ptr(out), _ptr(mag))
    _check(st, "gemm_w4a8_floatscale")
    with np.errstate(over="ignore"):
        out16 = out.astype(np.float16)
    return FloatScaleResult(out, out16, mag)


def gemm_w4a8_intscale_grouped(xq, a_scale, qweight, scale_i32, chan_scale, row_offsets, group: int, alpha_log2: int):
    """Mixture-of-experts form (Sec. 5.4 measures Mixtral): rows [row_offsets[e], row_offsets[e+1]) of xq use the
    e-th weight set.  qweight [E,N,K/2], scale_i32 [E,N,K/G], chan_scale [E,N] or None.  Returns (acc, out_fp16)."""
    E = qweight.shape[0]
    M = xq.shape[0]
    N = qweight.shape[1]
    acc = np.zeros((M, N), dtype=np.int32)
    out16 = np.zeros((M, N), dtype=np.float16)
    for e in range(E):
        lo, hi = int(row_offsets[e]), int(row_offsets[e + 1])
        if hi <= lo:
            continue
        r = gemm_w4a8_intscale(xq[lo:hi], a_scale[lo:hi], qweight[e], scale_i32[e],
                               None if chan_scale is None else chan_scale[e], group, alpha_log2)
        acc[lo:hi] = r.acc
        out16[lo:hi] = r.out_fp16
    return acc, out16


def gemm_w4a8_floatscale_grouped(xq, a_scale, qweight, scale_f32, row_offsets, group: int):
    """Float-scale twin of gemm_w4a8_intscale_grouped. Returns (out float64, abs_sum float64)."""
    E = qweight.shape[0]
    M = xq.shape[0]
    N = qweight.shape[1]
    out = np.zeros((M, N), dtype=np.float64)
    mag = np.zeros((M, N), dtype=np.float64)
    for e in range(E):
        lo, hi = int(row_offsets[e]), int(row_offsets[e + 1])
        if hi <= lo:
            continue
        r = gemm_w4a8_floatscale(xq[lo:hi], a_scale[lo:hi], qweight[e], scale_f32[e], group)
        out[lo:hi] = r.out
        mag[lo:hi] = r.abs_sum
    return out, mag


def overflow_safe_scale_bound(K: int, group: int) -> int:
    """Largest integer scale for which no input can overflow the 32-bit accumulator:
    |acc| <= (K/G) * G * 128 * 8 * IS_max < 2^31  (|xq| <= 128, |q| <= 8)."""
    return (2 ** 31 - 1) // (K * 128 * 8)


def layer_overflow_bound(scale_i32: np.ndarray, group: int) -> int:
    """Largest |accumulator| the integer-scale GEMM of Eq. (2) can reach with these integer scales, over all int8
    activation codes and int4 weight codes: max_n sum_g |IS[n,g]| * G * 128 * 8 (a group's partial sum is at most
    G * 128 * 8 in magnitude, reached by xq = -128, q = -8).  The 32-bit accumulator cannot overflow iff this is
    below 2^31 (the overflow risk the paper's Sec. 5.6 and Limitations discuss).  Python integer."""
    IS = np.abs(np.asarray(scale_i32).astype(np.int64))
    return int(IS.sum(axis=1).max()) * group * 128 * 8 if IS.size else 0


class SafeResult(NamedTuple):
    out: np.ndarray          # float64 [M,N], before the final rounding to fp16
    out_fp16: np.ndarray     # float16 [M,N]
    abs_sum: np.ndarray      # float64 [M,N], s_a * c / alpha * sum_g |P_g * IS_g|


def gemm_w4a8_intscale_safe(xq, a_scale, qweight, scale_i32, chan_scale, group: int, alpha_log2: int) -> SafeResult:
    """The overflow-safe ("degraded") form the paper's Limitations section names: the integer scales are kept but
    the amplifier is taken out group by group, so nothing accumulates in 32 bits:
        out[m,n] = s_a[m] * sum_g P[m,n,g] * (IS[n,g] * c[n] / alpha)
    Here the sum is exact (64-bit integers; it cannot wrap for any int32 scales and K < 2^20) and rounded once."""
    r = gemm_w4a8_intscale(xq, a_scale, qweight, scale_i32, chan_scale, group, alpha_log2)
    M, N = r.acc64.shape
    sa = _c(a_scale, np.float32).astype(np.float64)[:, None]
    c = np.ones((1, N)) if chan_scale is None else _c(chan_scale, np.float32).astype(np.float64)[None, :]
    factor = sa * c / float(2 ** alpha_log2)
    out = r.acc64.astype(np.float64) * factor
    p = group_partials(xq, qweight, group).astype(np.int64)
    mag = np.abs(p * np.asarray(scale_i32).astype(np.int64)[None, :, :]).sum(axis=2).astype(np.float64) * factor
    with np.errstate(over="ignore"):
        out16 = out.astype(np.float16)
    return SafeResult(out, out16, mag)


# ---------------------------------------------------------------------------------------------------------------------
# Fine-grained W8A8 (int8 weights; the paper's LLaMA-3 recipe uses it for down-projection layers, Sec. 5.5 / Table 5).
# Same equations with n = 8 on the weight side; written out in numpy (int64 / float64), no blocking.
# ---------------------------------------------------------------------------------------------------------------------
class QuantizedWeights8(NamedTuple):
    qweight: np.ndarray      # int8 [N,K]
    scale_f32: np.ndarray    # float32 [N,K/G], s = max|w| / 127
    scale_i32: np.ndarray    # int32 [N,K/G]
    chan_scale: np.ndarray   # float32 [N]
    alpha_log2: int


def quantize_weights_int8_group(w: np.ndarray, group: int, alpha_log2: int, scale_mode: int = SCALE_RAW
                                ) -> QuantizedWeights8:
    """Appendix A.1 with n = 8 on every (row, group): s = max|w| / 127, q = clamp(rne(w / s), -128, 127), both in
    IEEE fp32; then INT(s * alpha) of Eq. (2) (RAW) or INT(s / c * alpha) with c[n] = max_g s[n,g] (NORM);
    alpha_log2 = -1 runs the amplifier search of Sec. 4.1."""
    w32 = np.asarray(w).astype(np.float32)
    N, K = w32.shape
    if K % group or group <= 0 or not (-1 <= alpha_log2 <= 16) or scale_mode not in (SCALE_RAW, SCALE_NORM):
        raise ValueError("oracle quantize_weights_int8_group: bad arguments")
    NG = K // group
    wg = w32.reshape(N, NG, group)
    amax = np.abs(wg).max(axis=2).astype(np.float32)
    s = (amax / np.float32(127.0)).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.rint((wg / s[:, :, None]).astype(np.float32))
    q = np.where(s[:, :, None] > 0, np.clip(r, -128.0, 127.0), 0.0).astype(np.int8).reshape(N, K)
    if scale_mode == SCALE_NORM:
        c = s.max(axis=1).astype(np.float32)
        with np.errstate(divide="ignore", invalid="ignore"):
            amplified = np.where(c[:, None] > 0, (s / c[:, None]).astype(np.float32), np.float32(0)).astype(np.float32)
    else:
        c = np.ones(N, np.float32)
        amplified = s
    a = amplifier_log2(amplified) if alpha_log2 < 0 else alpha_log2
    IS = np.rint(np.ldexp(amplified, a).astype(np.float32)).astype(np.int32)
    return QuantizedWeights8(q, s, IS, c, a)


def group_partials_w8(xq: np.ndarray, q8: np.ndarray, group: int) -> np.ndarray:
    """P[m,n,g] = sum over group g of xq[m,k] * q[n,k], int64 [M,N,K/G] (|P| <= G * 128 * 128)."""
    M, K = xq.shape
    N = q8.shape[0]
    xg = np.asarray(xq).astype(np.int64).reshape(M, K // group, group)
    qg = np.asarray(q8).astype(np.int64).reshape(N, K // group, group)
    return np.einsum("mgk,ngk->mng", xg, qg)


def gemm_w8a8_intscale(xq, a_scale, q8, scale_i32, chan_scale, group: int, alpha_log2: int) -> IntScaleResult:
    """Eq. (2) / Table 2 "Ours" with int8 weights: acc = sum_g P_g * IS_g in int32 (wrapping), one conversion."""
    p = group_partials_w8(xq, q8, group)
    terms = p * np.asarray(scale_i32).astype(np.int64)[None, :, :]
    acc64 = terms.sum(axis=2)
    peak = np.abs(np.cumsum(terms, axis=2)).max(axis=2)
    acc = ((acc64 + 2 ** 31) % 2 ** 32 - 2 ** 31).astype(np.int32)
    N = acc.shape[1]
    sa = _c(a_scale, np.float32).astype(np.float64)[:, None]
    c = np.ones((1, N)) if chan_scale is None else _c(chan_scale, np.float32).astype(np.float64)[None, :]
    out = acc.astype(np.float64) * sa * c / float(2 ** alpha_log2)
    with np.errstate(over="ignore"):
        out16 = out.astype(np.float16)
    return IntScaleResult(acc, out, out16, acc64, peak)


def gemm_w8a8_floatscale(xq, a_scale, q8, scale_f32, group: int) -> FloatScaleResult:
    """Eq. (1) / Table 2 "Atom" with int8 weights, accumulated in double."""
    p = group_partials_w8(xq, q8, group).astype(np.float64)
    s = _c(scale_f32, np.float32).astype(np.float64)[None, :, :]
    sa = _c(a_scale, np.float32).astype(np.float64)[:, None]
    out = (p * s).sum(axis=2) * sa
    mag = (np.abs(p) * s).sum(axis=2) * sa
    with np.errstate(over="ignore"):
        out16 = out.astype(np.float16)
    return FloatScaleResult(out, out16, mag)


# ---------------------------------------------------------------------------------------------------------
# Activation quantisation folded into the operator that produces the activation ("kernel fusion", Sec. 4.3 and
# Sec. 5.2): the result is DEFINED as the unfused pipeline, producer -> fp16 tensor -> Appendix A.1 quantiser,
# so that fusing changes no code.  The producers are written as a fixed sequence of separately rounded
# single-precision operations (stated in each docstring), because their fp16 result decides integer codes.
# ---------------------------------------------------------------------------------------------------------
def rmsnorm_fp16(x: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm of fp16 rows: y = fp16( (x * r) * gamma ), r = 1 / sqrt(mean(x^2) + eps).

    Sum of squares in double (every fp16 square is exact there), mean rounded once to single, then single
    precision: add eps, square root, reciprocal, the two products in the order written, one rounding to fp16.
    """
    x16 = np.asarray(x, dtype=np.float16)
    g32 = np.asarray(gamma, dtype=np.float16).astype(np.float32)
    M, K = x16.shape
    ss = np.zeros((M,), dtype=np.float64)
    x64 = x16.astype(np.float64)
    for m in range(M):
        ss[m] = np.sum(x64[m] * x64[m])
    mean = (ss / np.float64(K)).astype(np.float32)
    r = np.float32(1.0) / np.sqrt(mean + np.float32(eps), dtype=np.float32)
    x32 = x16.astype(np.float32)
    y = (x32 * r[:, None]) * g32[None, :]
    return y.astype(np.float16)


def rmsnorm_quantize_act_int8_token(x: np.ndarray, gamma: np.ndarray, eps: float):
    """RMSNorm, then Appendix A.1 (n = 8) per token row on its fp16 output. Returns (xq, a_scale)."""
    return quantize_act_int8_token(rmsnorm_fp16(x, gamma, eps))


def exp_f32(t: np.ndarray) -> np.ndarray:
    """e^t in single precision by a stated sequence of separately rounded operations.

    t is clamped to [-87, 88]; n = rint(t * log2(e)); r = (t - n * ln2_hi) - n * ln2_lo; the degree-6 Taylor
    polynomial of e^r in Horner form (multiply, then add, each rounded); the result is scaled by 2^n exactly.
    """
    f = np.float32
    t = np.minimum(np.maximum(np.asarray(t, dtype=np.float32), f(-87.0)), f(88.0))
    n = np.rint(t * f(1.4426950408889634))
    r = (t - n * f(0.693145751953125)) - n * f(1.428606765330187e-06)
    p = f(1.0 / 720.0)
    for c in (1.0 / 120.0, 1.0 / 24.0, 1.0 / 6.0, 0.5, 1.0, 1.0):
        p = p * r + f(c)
    return np.ldexp(p, n.astype(np.int32)).astype(np.float32)


def silu_f32(g: np.ndarray) -> np.ndarray:
    """SiLU(g) = g / (1 + e^-g) in single precision: exp_f32, one addition, one division."""
    g = np.asarray(g, dtype=np.float32)
    return g / (np.float32(1.0) + exp_f32(-g))


def silu_mul_fp16(gate_up: np.ndarray) -> np.ndarray:
    """h = fp16( SiLU(gate) * up ) for gate_up = [gate | up] along the last axis (fp16 [M, 2I] -> fp16 [M, I])."""
    gu = np.asarray(gate_up, dtype=np.float16).astype(np.float32)
    inter = gu.shape[1] // 2
    if gu.shape[1] != 2 * inter:
        raise ValueError("oracle silu_mul: the last axis must hold gate and up halves of equal length")
    return (silu_f32(gu[:, :inter]) * gu[:, inter:]).astype(np.float16)


def silu_mul_quantize_act_int8_token(gate_up: np.ndarray):
    """SiLU(gate) * up, then Appendix A.1 (n = 8) per token row on its fp16 output. Returns (xq, a_scale)."""
    return quantize_act_int8_token(silu_mul_fp16(gate_up))
