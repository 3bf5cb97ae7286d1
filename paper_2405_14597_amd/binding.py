"""Thin Python binding of libintscale.so (the C ABI declared in include/intscale.h).

Argument marshalling only: torch supplies device memory and the stream, every step of the layer runs in the
library's HIP kernels.  There is no CPU or PyTorch fallback: if the library is missing and cannot be built, or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

from . import build as _build

IS_OK = 0
IS_ERR_INVALID_ARG = -1
IS_ERR_UNSUPPORTED = -2
IS_ERR_WORKSPACE = -3
IS_ERR_HIP = -4
IS_SCALE_RAW = 0
IS_SCALE_NORM = 1
IS_ALPHA_HEURISTIC = -1

EXPORTED_SYMBOLS = (
    "is_quantize_weights_int4_group",
    "is_quantize_act_int8_token",
    "is_rmsnorm_quantize_act_int8_token",
    "is_silu_mul_quantize_act_int8_token",
    "is_gemm_w4a8_intscale",
    "is_gemm_w4a8_floatscale",
    "is_gemm_workspace_bytes",
    "is_linear_workspace_bytes",
    "is_linear_w4a8_intscale",
    "is_linear_w4a8_floatscale",
    "is_gemm_w4a8_intscale_grouped",
    "is_gemm_w4a8_floatscale_grouped",
    "is_gemm_grouped_workspace_bytes",
    "is_quantize_weights_int8_group",
    "is_gemm_w8a8_intscale",
    "is_gemm_w8a8_floatscale",
    "is_gemm_w8a8_workspace_bytes",
    "is_intscale_overflow_bound",
    "is_gemm_w4a8_intscale_safe",
    "is_gemm_safe_workspace_bytes",
    "is_prepack_w4_weight_bytes",
    "is_prepack_w4_scale_bytes",
    "is_prepack_w4",
    "is_gemm_prepacked_workspace_bytes",
    "is_gemm_w4a8_intscale_prepacked",
    "is_gemm_w4a8_floatscale_prepacked",
    "is_gemm_w4a8_intscale_prepacked_noalloc",
    "is_prepare_activations_prepacked",
    "is_gemm_w4a8_intscale_prepacked_prepared",
    "is_gemm_w4a8_floatscale_prepacked_prepared",
    "is_linear_prepacked_workspace_bytes",
    "is_linear_w4a8_intscale_prepacked",
    "is_linear_w4a8_floatscale_prepacked",
    "is_gemm_grouped_prepacked_workspace_bytes",
    "is_gemm_w4a8_intscale_grouped_prepacked",
    "is_gemm_w4a8_floatscale_grouped_prepacked",
    "is_prepack_w4_gate_up",
    "is_gemm_gate_up_silu_prepacked_workspace_bytes",
    "is_gemm_w4a8_intscale_gate_up_silu_prepacked",
    "is_gemm_w4a8_floatscale_gate_up_silu_prepacked",
    "is_describe_prepacked",
    "is_describe_grouped_prepacked",
    "is_source_hash",
    "is_probe_stream_read",
    "is_probe_mfma_i8",
    "is_probe_mfma_i8_random",
    "is_set_kernel_route",
    "is_status_string",
    "is_last_hip_error",
)


class IntScaleError(RuntimeError):
    def __init__(self, fn: str, status: int, detail: str = ""):
        self.status = status
        super().__init__(f"{fn} failed: {status_string(status)}" + (f" ({detail})" if detail else ""))


_lib = None


def library_path() -> str:
    return _build.LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libintscale.so; build it first if none is there, or if the one there was compiled from other sources than
    the ones beside it (the library carries a digest of its sources)."""
    global _lib
    if _lib is not None:
        return _lib
    if "INTSCALE_LIBRARY" in os.environ:      # somebody else's build: loaded as it is
        if not os.path.exists(_build.LIB_PATH):
            raise IntScaleError("load_library", IS_ERR_INVALID_ARG, f"INTSCALE_LIBRARY={_build.LIB_PATH} does not exist")
    elif _build.needs_build():
        _build.build_library(force=True)
    # The library and torch must share ONE HIP runtime (device pointers and streams cross between them), so torch's
    # runtime is loaded first and libintscale.so's libamdhip64 dependency resolves to it.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.is_quantize_weights_int4_group.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.is_quantize_weights_int4_group.restype = ci
    lib.is_quantize_act_int8_token.argtypes = [vp, ci, ci, vp, vp, vp]
    lib.is_quantize_act_int8_token.restype = ci
    lib.is_rmsnorm_quantize_act_int8_token.argtypes = [vp, vp, ctypes.c_float, ci, ci, vp, vp, vp]
    lib.is_rmsnorm_quantize_act_int8_token.restype = ci
    lib.is_silu_mul_quantize_act_int8_token.argtypes = [vp, ci, ci, vp, vp, vp]
    lib.is_silu_mul_quantize_act_int8_token.restype = ci
    lib.is_gemm_w4a8_intscale.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_gemm_w4a8_intscale.restype = ci
    lib.is_gemm_w4a8_floatscale.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w4a8_floatscale.restype = ci
    lib.is_gemm_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.is_gemm_workspace_bytes.restype = sz
    lib.is_linear_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.is_linear_workspace_bytes.restype = sz
    lib.is_linear_w4a8_intscale.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_linear_w4a8_intscale.restype = ci
    lib.is_linear_w4a8_floatscale.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_linear_w4a8_floatscale.restype = ci
    lib.is_gemm_w4a8_intscale_grouped.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_gemm_w4a8_intscale_grouped.restype = ci
    lib.is_gemm_w4a8_floatscale_grouped.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w4a8_floatscale_grouped.restype = ci
    lib.is_gemm_grouped_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.is_gemm_grouped_workspace_bytes.restype = sz
    lib.is_quantize_weights_int8_group.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.is_quantize_weights_int8_group.restype = ci
    lib.is_gemm_w8a8_intscale.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_gemm_w8a8_intscale.restype = ci
    lib.is_gemm_w8a8_floatscale.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w8a8_floatscale.restype = ci
    lib.is_gemm_w8a8_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.is_gemm_w8a8_workspace_bytes.restype = sz
    lib.is_intscale_overflow_bound.argtypes = [vp, ci, ci, ci, vp, vp]
    lib.is_intscale_overflow_bound.restype = ci
    lib.is_gemm_w4a8_intscale_safe.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w4a8_intscale_safe.restype = ci
    lib.is_gemm_safe_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.is_gemm_safe_workspace_bytes.restype = sz
    lib.is_prepack_w4_weight_bytes.argtypes = [ci, ci]
    lib.is_prepack_w4_weight_bytes.restype = sz
    lib.is_prepack_w4_scale_bytes.argtypes = [ci, ci, ci]
    lib.is_prepack_w4_scale_bytes.restype = sz
    lib.is_prepack_w4.argtypes = [vp, vp, vp, ci, ci, ci, vp, vp, vp]
    lib.is_prepack_w4.restype = ci
    lib.is_gemm_prepacked_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.is_gemm_prepacked_workspace_bytes.restype = sz
    lib.is_gemm_w4a8_intscale_prepacked.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_gemm_w4a8_intscale_prepacked.restype = ci
    lib.is_gemm_w4a8_floatscale_prepacked.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w4a8_floatscale_prepacked.restype = ci
    lib.is_prepack_w4_gate_up.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.is_prepack_w4_gate_up.restype = ci
    lib.is_gemm_gate_up_silu_prepacked_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.is_gemm_gate_up_silu_prepacked_workspace_bytes.restype = sz
    lib.is_gemm_w4a8_intscale_gate_up_silu_prepacked.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_gemm_w4a8_intscale_gate_up_silu_prepacked.restype = ci
    lib.is_gemm_w4a8_floatscale_gate_up_silu_prepacked.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w4a8_floatscale_gate_up_silu_prepacked.restype = ci
    lib.is_gemm_w4a8_intscale_prepacked_noalloc.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp]
    lib.is_gemm_w4a8_intscale_prepacked_noalloc.restype = ci
    lib.is_prepare_activations_prepacked.argtypes = [vp, ci, ci, vp, sz, vp]
    lib.is_prepare_activations_prepacked.restype = ci
    lib.is_gemm_w4a8_intscale_prepacked_prepared.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_gemm_w4a8_intscale_prepacked_prepared.restype = ci
    lib.is_gemm_w4a8_floatscale_prepacked_prepared.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w4a8_floatscale_prepacked_prepared.restype = ci
    lib.is_gemm_grouped_prepacked_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.is_gemm_grouped_prepacked_workspace_bytes.restype = sz
    lib.is_gemm_w4a8_intscale_grouped_prepacked.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, sz,
                                                            vp]
    lib.is_gemm_w4a8_intscale_grouped_prepacked.restype = ci
    lib.is_gemm_w4a8_floatscale_grouped_prepacked.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_gemm_w4a8_floatscale_grouped_prepacked.restype = ci
    lib.is_linear_prepacked_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.is_linear_prepacked_workspace_bytes.restype = sz
    lib.is_linear_w4a8_intscale_prepacked.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.is_linear_w4a8_intscale_prepacked.restype = ci
    lib.is_linear_w4a8_floatscale_prepacked.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.is_linear_w4a8_floatscale_prepacked.restype = ci
    lib.is_probe_stream_read.argtypes = [vp, sz, vp, vp]
    lib.is_probe_stream_read.restype = ci
    lib.is_probe_mfma_i8.argtypes = [ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.is_probe_mfma_i8.restype = ci
    lib.is_probe_mfma_i8_random.argtypes = [ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.is_probe_mfma_i8_random.restype = ci
    lib.is_set_kernel_route.argtypes = [ci]
    lib.is_set_kernel_route.restype = ci
    lib.is_status_string.argtypes = [ci]
    lib.is_status_string.restype = ctypes.c_char_p
    lib.is_last_hip_error.argtypes = []
    lib.is_last_hip_error.restype = ctypes.c_char_p
    lib.is_source_hash.argtypes = []
    lib.is_source_hash.restype = ctypes.c_char_p
    lib.is_describe_prepacked.argtypes = [ci, ci, ci, ci, ci, ci, ctypes.c_char_p, sz]
    lib.is_describe_prepacked.restype = ci
    lib.is_describe_grouped_prepacked.argtypes = [ci, ci, ci, ci, ci, ci, ctypes.c_char_p, sz]
    lib.is_describe_grouped_prepacked.restype = ci
    _lib = lib
    return lib


KERNEL_ROUTES = {"auto": 0, "general": 1, "tiled": 2, "tiled64": 3}


def is_set_kernel_route(route) -> str:
    """Routing override for tests and experiments ("auto", "general", "tiled", "tiled64"); returns the one in force before."""
    code = KERNEL_ROUTES[route] if isinstance(route, str) else int(route)
    before = load_library().is_set_kernel_route(code)
    _check("is_set_kernel_route", before if before < 0 else 0)
    return {v: k for k, v in KERNEL_ROUTES.items()}[before]


def status_string(status: int) -> str:
    return load_library().is_status_string(int(status)).decode()


def last_hip_error() -> str:
    return load_library().is_last_hip_error().decode()


def _check(fn: str, status: int) -> None:
    if status != IS_OK:
        raise IntScaleError(fn, status, last_hip_error() if status == IS_ERR_HIP else "")


# --------------------------------------------------------------------------------------------------------------
# torch-tensor level.  torch is imported lazily so that the symbol/ABI checks work without it.
# --------------------------------------------------------------------------------------------------------------
def _torch():
    import torch
    return torch


def _stream_handle(stream) -> int:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _p(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _require(t, dtype, shape, name):
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name}: expected contiguous cuda tensor {dtype} {tuple(shape)}, got {t.dtype} "
                         f"{tuple(t.shape)} on {t.device}")


class QuantizedWeights(NamedTuple):
    qweight: "object"      # uint8 [N, K/2] (or [E,N,K/2])
    scale_f32: "object"    # float32 [N, K/G]
    scale_i32: "object"    # int32 [N, K/G]
    chan_scale: "object"   # float32 [N]
    alpha_log2_dev: "object"  # int32 [1] on the device


def is_quantize_weights_int4_group(w, group: int, alpha_log2: int, scale_mode: int = IS_SCALE_RAW, stream=None
                                   ) -> QuantizedWeights:
    torch = _torch()
    N, K = w.shape
    _require(w, torch.float16, (N, K), "w")
    if group <= 0 or K % group != 0:
        raise IntScaleError("is_quantize_weights_int4_group", IS_ERR_INVALID_ARG)
    dev = w.device
    q = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    s = torch.empty((N, K // group), dtype=torch.float32, device=dev)
    si = torch.empty((N, K // group), dtype=torch.int32, device=dev)
    c = torch.empty((N,), dtype=torch.float32, device=dev)
    a_dev = torch.empty((4,), dtype=torch.int32, device=dev)
    st = load_library().is_quantize_weights_int4_group(_p(w), N, K, group, alpha_log2, scale_mode, _p(q), _p(s), _p(si),
                                                      _p(c), _p(a_dev), _stream_handle(stream))
    _check("is_quantize_weights_int4_group", st)
    return QuantizedWeights(q, s, si, c, a_dev[:1])


def is_quantize_act_int8_token(x, xq=None, a_scale=None, stream=None):
    torch = _torch()
    M, K = x.shape
    _require(x, torch.float16, (M, K), "x")
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if a_scale is None:
        a_scale = torch.empty((M,), dtype=torch.float32, device=x.device)
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    st = load_library().is_quantize_act_int8_token(_p(x), M, K, _p(xq), _p(a_scale), _stream_handle(stream))
    _check("is_quantize_act_int8_token", st)
    return xq, a_scale


def is_rmsnorm_quantize_act_int8_token(x, gamma, eps: float, xq=None, a_scale=None, stream=None):
    torch = _torch()
    M, K = x.shape
    _require(x, torch.float16, (M, K), "x")
    _require(gamma, torch.float16, (K,), "gamma")
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if a_scale is None:
        a_scale = torch.empty((M,), dtype=torch.float32, device=x.device)
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    st = load_library().is_rmsnorm_quantize_act_int8_token(_p(x), _p(gamma), float(eps), M, K, _p(xq), _p(a_scale),
                                                           _stream_handle(stream))
    _check("is_rmsnorm_quantize_act_int8_token", st)
    return xq, a_scale


def is_silu_mul_quantize_act_int8_token(gate_up, xq=None, a_scale=None, stream=None):
    torch = _torch()
    M, two_inter = gate_up.shape
    inter = two_inter // 2
    _require(gate_up, torch.float16, (M, 2 * inter), "gate_up")
    if xq is None:
        xq = torch.empty((M, inter), dtype=torch.int8, device=gate_up.device)
    if a_scale is None:
        a_scale = torch.empty((M,), dtype=torch.float32, device=gate_up.device)
    _require(xq, torch.int8, (M, inter), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    st = load_library().is_silu_mul_quantize_act_int8_token(_p(gate_up), M, inter, _p(xq), _p(a_scale),
                                                            _stream_handle(stream))
    _check("is_silu_mul_quantize_act_int8_token", st)
    return xq, a_scale


def is_gemm_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_gemm_workspace_bytes(M, N, K, group))


def is_gemm_grouped_workspace_bytes(E: int, M_total: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_gemm_grouped_workspace_bytes(E, M_total, N, K, group))


def _workspace(nbytes: int, device, workspace):
    torch = _torch()
    if workspace is not None:
        return workspace, workspace.numel() * workspace.element_size()
    if nbytes == 0:
        return None, 0
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=device)
    return ws, nbytes


def _release_workspace(ws, workspace, stream) -> None:
    """A workspace this module allocated goes back to torch's allocator when the call returns, while the kernels may
    still be queued: tell the allocator which stream uses it, so the block is not handed out on another stream early."""
    if ws is not None and workspace is None and stream is not None and hasattr(stream, "cuda_stream"):
        ws.record_stream(stream)


def is_gemm_w4a8_intscale(xq, a_scale, qweight, scale_i32, chan_scale, group: int, alpha_log2: int, out=None,
                          acc_out=None, want_acc: bool = False, workspace=None, stream=None):
    """Returns (out fp16 [M,N], acc int32 [M,N] or None)."""
    torch = _torch()
    M, K = xq.shape
    N = qweight.shape[0]
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(qweight, torch.uint8, (N, K // 2), "qweight")
    _require(scale_i32, torch.int32, (N, K // group), "scale_i32")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    ws, ws_bytes = _workspace(is_gemm_workspace_bytes(M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_intscale(_p(xq), _p(a_scale), _p(qweight), _p(scale_i32), _p(chan_scale), M, N, K,
                                             group, alpha_log2, _p(out), _p(acc_out), _p(ws), ws_bytes,
                                             _stream_handle(stream))
    _check("is_gemm_w4a8_intscale", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


def is_gemm_w4a8_floatscale(xq, a_scale, qweight, scale_f32, group: int, out=None, workspace=None, stream=None):
    torch = _torch()
    M, K = xq.shape
    N = qweight.shape[0]
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(qweight, torch.uint8, (N, K // 2), "qweight")
    _require(scale_f32, torch.float32, (N, K // group), "scale_f32")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _workspace(is_gemm_workspace_bytes(M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_floatscale(_p(xq), _p(a_scale), _p(qweight), _p(scale_f32), M, N, K, group,
                                               _p(out), _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_gemm_w4a8_floatscale", st)
    _release_workspace(ws, workspace, stream)
    return out


def is_linear_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_linear_workspace_bytes(M, N, K, group))


def is_linear_w4a8_intscale(x, qweight, scale_i32, chan_scale, group: int, alpha_log2: int, out=None, acc_out=None,
                            want_acc: bool = False, workspace=None, stream=None):
    """fp16 activations in: quantiser + integer-scale GEMM behind one call. Returns (out fp16 [M,N], acc or None)."""
    torch = _torch()
    M, K = x.shape
    N = qweight.shape[0]
    _require(x, torch.float16, (M, K), "x")
    _require(qweight, torch.uint8, (N, K // 2), "qweight")
    _require(scale_i32, torch.int32, (N, K // group), "scale_i32")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=x.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    ws, ws_bytes = _workspace(is_linear_workspace_bytes(M, N, K, group), x.device, workspace)
    st = load_library().is_linear_w4a8_intscale(_p(x), _p(qweight), _p(scale_i32), _p(chan_scale), M, N, K, group,
                                               alpha_log2, _p(out), _p(acc_out), _p(ws), ws_bytes,
                                               _stream_handle(stream))
    _check("is_linear_w4a8_intscale", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


def is_linear_w4a8_floatscale(x, qweight, scale_f32, group: int, out=None, workspace=None, stream=None):
    torch = _torch()
    M, K = x.shape
    N = qweight.shape[0]
    _require(x, torch.float16, (M, K), "x")
    _require(qweight, torch.uint8, (N, K // 2), "qweight")
    _require(scale_f32, torch.float32, (N, K // group), "scale_f32")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _workspace(is_linear_workspace_bytes(M, N, K, group), x.device, workspace)
    st = load_library().is_linear_w4a8_floatscale(_p(x), _p(qweight), _p(scale_f32), M, N, K, group, _p(out), _p(ws),
                                                 ws_bytes, _stream_handle(stream))
    _check("is_linear_w4a8_floatscale", st)
    _release_workspace(ws, workspace, stream)
    return out


def is_quantize_weights_int8_group(w, group: int, alpha_log2: int, scale_mode: int = IS_SCALE_RAW, stream=None
                                   ) -> QuantizedWeights:
    """Fine-grained W8A8 weights: qweight is int8 [N,K]."""
    torch = _torch()
    N, K = w.shape
    _require(w, torch.float16, (N, K), "w")
    if group <= 0 or K % group != 0:
        raise IntScaleError("is_quantize_weights_int8_group", IS_ERR_INVALID_ARG)
    dev = w.device
    q = torch.empty((N, K), dtype=torch.int8, device=dev)
    s = torch.empty((N, K // group), dtype=torch.float32, device=dev)
    si = torch.empty((N, K // group), dtype=torch.int32, device=dev)
    c = torch.empty((N,), dtype=torch.float32, device=dev)
    a_dev = torch.empty((4,), dtype=torch.int32, device=dev)
    st = load_library().is_quantize_weights_int8_group(_p(w), N, K, group, alpha_log2, scale_mode, _p(q), _p(s), _p(si),
                                                      _p(c), _p(a_dev), _stream_handle(stream))
    _check("is_quantize_weights_int8_group", st)
    return QuantizedWeights(q, s, si, c, a_dev[:1])


def is_gemm_w8a8_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_gemm_w8a8_workspace_bytes(M, N, K, group))


def is_gemm_w8a8_intscale(xq, a_scale, qweight8, scale_i32, chan_scale, group: int, alpha_log2: int, out=None,
                          acc_out=None, want_acc: bool = False, workspace=None, stream=None):
    """Returns (out fp16 [M,N], acc int32 [M,N] or None)."""
    torch = _torch()
    M, K = xq.shape
    N = qweight8.shape[0]
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(qweight8, torch.int8, (N, K), "qweight8")
    _require(scale_i32, torch.int32, (N, K // group), "scale_i32")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    ws, ws_bytes = _workspace(is_gemm_w8a8_workspace_bytes(M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w8a8_intscale(_p(xq), _p(a_scale), _p(qweight8), _p(scale_i32), _p(chan_scale), M, N, K,
                                             group, alpha_log2, _p(out), _p(acc_out), _p(ws), ws_bytes,
                                             _stream_handle(stream))
    _check("is_gemm_w8a8_intscale", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


def is_gemm_w8a8_floatscale(xq, a_scale, qweight8, scale_f32, group: int, out=None, workspace=None, stream=None):
    torch = _torch()
    M, K = xq.shape
    N = qweight8.shape[0]
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(qweight8, torch.int8, (N, K), "qweight8")
    _require(scale_f32, torch.float32, (N, K // group), "scale_f32")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _workspace(is_gemm_w8a8_workspace_bytes(M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w8a8_floatscale(_p(xq), _p(a_scale), _p(qweight8), _p(scale_f32), M, N, K, group,
                                               _p(out), _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_gemm_w8a8_floatscale", st)
    _release_workspace(ws, workspace, stream)
    return out


def is_gemm_safe_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_gemm_safe_workspace_bytes(M, N, K, group))


def is_gemm_w4a8_intscale_safe(xq, a_scale, qweight, scale_i32, chan_scale, group: int, alpha_log2: int, out=None,
                               workspace=None, stream=None):
    torch = _torch()
    M, K = xq.shape
    N = qweight.shape[0]
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(qweight, torch.uint8, (N, K // 2), "qweight")
    _require(scale_i32, torch.int32, (N, K // group), "scale_i32")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _workspace(is_gemm_safe_workspace_bytes(M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_intscale_safe(_p(xq), _p(a_scale), _p(qweight), _p(scale_i32), _p(chan_scale), M,
                                                  N, K, group, alpha_log2, _p(out), _p(ws), ws_bytes,
                                                  _stream_handle(stream))
    _check("is_gemm_w4a8_intscale_safe", st)
    _release_workspace(ws, workspace, stream)
    return out


def is_intscale_overflow_bound(scale_i32, group: int, bound=None, stream=None):
    """Returns a device tensor holding the layer's worst-case |accumulator| (int64 view of the unsigned 64-bit value)."""
    torch = _torch()
    N, NG = scale_i32.shape
    _require(scale_i32, torch.int32, (N, NG), "scale_i32")
    if bound is None:
        bound = torch.empty((1,), dtype=torch.int64, device=scale_i32.device)
    _require(bound, torch.int64, (1,), "bound")
    st = load_library().is_intscale_overflow_bound(_p(scale_i32), N, NG * group, group, _p(bound), _stream_handle(stream))
    _check("is_intscale_overflow_bound", st)
    return bound


def is_gemm_w4a8_intscale_grouped(xq, a_scale, qweight, scale_i32, chan_scale, row_offsets, group: int,
                                  alpha_log2: int, out=None, acc_out=None, want_acc: bool = False, workspace=None,
                                  stream=None):
    torch = _torch()
    M, K = xq.shape
    E, N = qweight.shape[0], qweight.shape[1]
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(qweight, torch.uint8, (E, N, K // 2), "qweight")
    _require(scale_i32, torch.int32, (E, N, K // group), "scale_i32")
    _require(row_offsets, torch.int32, (E + 1,), "row_offsets")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (E, N), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    ws, ws_bytes = _workspace(is_gemm_grouped_workspace_bytes(E, M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_intscale_grouped(_p(xq), _p(a_scale), _p(qweight), _p(scale_i32), _p(chan_scale),
                                                     _p(row_offsets), E, M, N, K, group, alpha_log2, _p(out),
                                                     _p(acc_out), _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_gemm_w4a8_intscale_grouped", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


def is_gemm_w4a8_floatscale_grouped(xq, a_scale, qweight, scale_f32, row_offsets, group: int, out=None,
                                    workspace=None, stream=None):
    torch = _torch()
    M, K = xq.shape
    E, N = qweight.shape[0], qweight.shape[1]
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(qweight, torch.uint8, (E, N, K // 2), "qweight")
    _require(scale_f32, torch.float32, (E, N, K // group), "scale_f32")
    _require(row_offsets, torch.int32, (E + 1,), "row_offsets")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _workspace(is_gemm_grouped_workspace_bytes(E, M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_floatscale_grouped(_p(xq), _p(a_scale), _p(qweight), _p(scale_f32),
                                                       _p(row_offsets), E, M, N, K, group, _p(out), _p(ws), ws_bytes,
                                                       _stream_handle(stream))
    _check("is_gemm_w4a8_floatscale_grouped", st)
    _release_workspace(ws, workspace, stream)
    return out


def is_probe_stream_read(src, sink, stream=None) -> int:
    """Enqueues one streaming read of the whole tensor `src`; returns the bytes read."""
    nbytes = (src.numel() * src.element_size()) // 16 * 16
    _check("is_probe_stream_read", load_library().is_probe_stream_read(_p(src), nbytes, _p(sink), _stream_handle(stream)))
    return nbytes


def is_probe_mfma_i8(iters: int, sink, stream=None) -> float:
    """Enqueues the int8 MFMA loop; returns the int8 operations it performs."""
    ops = ctypes.c_double(0.0)
    _check("is_probe_mfma_i8", load_library().is_probe_mfma_i8(iters, _p(sink), ctypes.byref(ops), _stream_handle(stream)))
    return float(ops.value)


def is_probe_mfma_i8_random(iters: int, sink, stream=None) -> float:
    """The same loop on operands that change from one MFMA to the next; returns the int8 operations it performs."""
    ops = ctypes.c_double(0.0)
    _check("is_probe_mfma_i8_random",
           load_library().is_probe_mfma_i8_random(iters, _p(sink), ctypes.byref(ops), _stream_handle(stream)))
    return float(ops.value)



# --------------------------------------------------------------------------------------------------------------
# prepacked weights (kernel layout)
# --------------------------------------------------------------------------------------------------------------
class PackedWeights(NamedTuple):
    wpack: "object"    # uint8, kernel layout of the int4 weights
    spack: "object"    # uint8, header + kernel layout of the group scales (integer or float)
    N: int
    K: int
    group: int
    float_scales: bool


def is_prepack_w4(qweight, scale, group: int, stream=None) -> PackedWeights:
    """Canonical qweight [N,K/2] + scale_i32 or scale_f32 [N,K/group] -> kernel layout."""
    torch = _torch()
    lib = load_library()
    N, K2 = qweight.shape
    K = 2 * K2
    _require(qweight, torch.uint8, (N, K2), "qweight")
    if scale.dtype not in (torch.int32, torch.float32):
        raise ValueError("scale: int32 or float32 expected")
    _require(scale, scale.dtype, (N, K // group), "scale")
    wb, sb = int(lib.is_prepack_w4_weight_bytes(N, K)), int(lib.is_prepack_w4_scale_bytes(N, K, group))
    if wb == 0 or sb == 0:
        raise IntScaleError("is_prepack_w4", IS_ERR_UNSUPPORTED)
    wpack = torch.empty((wb,), dtype=torch.uint8, device=qweight.device)
    spack = torch.empty((sb,), dtype=torch.uint8, device=qweight.device)
    is_float = scale.dtype == torch.float32
    st = lib.is_prepack_w4(_p(qweight), None if is_float else _p(scale), _p(scale) if is_float else None, N, K, group,
                           _p(wpack), _p(spack), _stream_handle(stream))
    _check("is_prepack_w4", st)
    return PackedWeights(wpack, spack, N, K, group, is_float)


def is_gemm_prepacked_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_gemm_prepacked_workspace_bytes(M, N, K, group))


def is_linear_prepacked_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_linear_prepacked_workspace_bytes(M, N, K, group))


class PackedExperts(NamedTuple):
    wpack: "object"    # uint8 [E, weight bytes]: every expert's weights in the kernel layout, back to back
    spack: "object"    # uint8 [E, scale bytes]: every expert's scales (header included)
    E: int
    N: int
    K: int
    group: int
    float_scales: bool


def is_prepack_w4_experts(qweight, scale, group: int, stream=None) -> PackedExperts:
    """qweight [E,N,K/2] + scale_i32 or scale_f32 [E,N,K/group] -> every expert prepacked by is_prepack_w4, back to back."""
    torch = _torch()
    lib = load_library()
    E, N, K2 = qweight.shape
    K = 2 * K2
    _require(qweight, torch.uint8, (E, N, K2), "qweight")
    if scale.dtype not in (torch.int32, torch.float32):
        raise ValueError("scale: int32 or float32 expected")
    _require(scale, scale.dtype, (E, N, K // group), "scale")
    wb, sb = int(lib.is_prepack_w4_weight_bytes(N, K)), int(lib.is_prepack_w4_scale_bytes(N, K, group))
    if wb == 0 or sb == 0:
        raise IntScaleError("is_prepack_w4", IS_ERR_UNSUPPORTED)
    wpack = torch.empty((E, wb), dtype=torch.uint8, device=qweight.device)
    spack = torch.empty((E, sb), dtype=torch.uint8, device=qweight.device)
    is_float = scale.dtype == torch.float32
    for e in range(E):
        st = lib.is_prepack_w4(_p(qweight[e]), None if is_float else _p(scale[e]), _p(scale[e]) if is_float else None, N, K,
                               group, _p(wpack[e]), _p(spack[e]), _stream_handle(stream))
        _check("is_prepack_w4", st)
    return PackedExperts(wpack, spack, E, N, K, group, is_float)


def is_gemm_grouped_prepacked_workspace_bytes(E: int, M: int, N: int, K: int, group: int) -> int:
    return int(load_library().is_gemm_grouped_prepacked_workspace_bytes(E, M, N, K, group))


def is_gemm_w4a8_intscale_grouped_prepacked(xq, a_scale, packed: PackedExperts, chan_scale, row_offsets, alpha_log2: int,
                                            out=None, acc_out=None, want_acc: bool = False, workspace=None, stream=None):
    """Mixture-of-experts form on prepacked experts. Returns (out fp16 [M,N], acc or None)."""
    torch = _torch()
    M, K = xq.shape
    E, N, group = packed.E, packed.N, packed.group
    if K != packed.K or packed.float_scales:
        raise ValueError("packed experts: K mismatch or float scales")
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(row_offsets, torch.int32, (E + 1,), "row_offsets")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (E, N), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    ws, ws_bytes = _workspace(is_gemm_grouped_prepacked_workspace_bytes(E, M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_intscale_grouped_prepacked(
        _p(xq), _p(a_scale), _p(packed.wpack), _p(packed.spack), _p(chan_scale), _p(row_offsets), E, M, N, K, group,
        alpha_log2, _p(out), _p(acc_out), _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_gemm_w4a8_intscale_grouped_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


def is_gemm_w4a8_floatscale_grouped_prepacked(xq, a_scale, packed: PackedExperts, row_offsets, out=None, workspace=None,
                                              stream=None):
    torch = _torch()
    M, K = xq.shape
    E, N, group = packed.E, packed.N, packed.group
    if K != packed.K or not packed.float_scales:
        raise ValueError("packed experts: K mismatch or integer scales")
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    _require(row_offsets, torch.int32, (E + 1,), "row_offsets")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _workspace(is_gemm_grouped_prepacked_workspace_bytes(E, M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_floatscale_grouped_prepacked(
        _p(xq), _p(a_scale), _p(packed.wpack), _p(packed.spack), _p(row_offsets), E, M, N, K, group, _p(out), _p(ws),
        ws_bytes, _stream_handle(stream))
    _check("is_gemm_w4a8_floatscale_grouped_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out


def is_describe_prepacked(M: int, N: int, K: int, group: int, int_scale: bool = True, fp16_in: bool = False):
    """Names of the kernels the prepacked GEMM (or, fp16_in, linear) call launches for this shape, in launch order, as a
    kernel trace shows them.  Host-only."""
    buf = ctypes.create_string_buffer(512)
    st = load_library().is_describe_prepacked(M, N, K, group, int(int_scale), int(fp16_in), buf, len(buf))
    _check("is_describe_prepacked", st)
    return buf.value.decode().split("\n")


def is_describe_grouped_prepacked(num_experts: int, M_total: int, N: int, K: int, group: int, int_scale: bool = True):
    """The same for the grouped prepacked GEMM call."""
    buf = ctypes.create_string_buffer(512)
    st = load_library().is_describe_grouped_prepacked(num_experts, M_total, N, K, group, int(int_scale), buf, len(buf))
    _check("is_describe_grouped_prepacked", st)
    return buf.value.decode().split("\n")


def _zero_workspace(nbytes: int, device, workspace):
    """The prepacked GEMMs want their arrival counters zero: a fresh workspace is zero-filled."""
    torch = _torch()
    if workspace is not None:
        return workspace, workspace.numel() * workspace.element_size()
    if nbytes == 0:
        return None, 0
    return torch.zeros((nbytes,), dtype=torch.uint8, device=device), nbytes


def is_gemm_w4a8_intscale_prepacked(xq, a_scale, packed: PackedWeights, chan_scale, alpha_log2: int, out=None,
                                    acc_out=None, want_acc: bool = False, workspace=None, stream=None):
    """Returns (out fp16 [M,N], acc int32 [M,N] or None)."""
    torch = _torch()
    M, K = xq.shape
    N, group = packed.N, packed.group
    if K != packed.K or packed.float_scales:
        raise ValueError("packed weights: K mismatch or float scales")
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    ws, ws_bytes = _zero_workspace(is_gemm_prepacked_workspace_bytes(M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_intscale_prepacked(_p(xq), _p(a_scale), _p(packed.wpack), _p(packed.spack),
                                                       _p(chan_scale), M, N, K, group, alpha_log2, _p(out), _p(acc_out),
                                                       _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_gemm_w4a8_intscale_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


class PackedGateUp(NamedTuple):
    packed: PackedWeights   # the fused projection, N = 2 * inter, gate / up rows paired by 16-row tile
    chan_scale: "object"    # float32 [2 * inter] in the packed row order, or None
    inter: int


def is_prepack_w4_gate_up(qweight, scale, chan_scale, group: int, stream=None) -> PackedGateUp:
    """Canonical fused gate_up projection (rows [0, inter) gate, [inter, 2 inter) up) -> kernel layout with the rows of
    gate and up paired, for the GEMMs with the SiLU(gate) * up epilogue."""
    torch = _torch()
    lib = load_library()
    N, K2 = qweight.shape
    K, inter = 2 * K2, N // 2
    if N != 2 * inter:
        raise ValueError("qweight: an even number of rows (gate and up) expected")
    _require(qweight, torch.uint8, (N, K2), "qweight")
    if scale.dtype not in (torch.int32, torch.float32):
        raise ValueError("scale: int32 or float32 expected")
    _require(scale, scale.dtype, (N, K // group), "scale")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    wb, sb = int(lib.is_prepack_w4_weight_bytes(N, K)), int(lib.is_prepack_w4_scale_bytes(N, K, group))
    if wb == 0 or sb == 0:
        raise IntScaleError("is_prepack_w4_gate_up", IS_ERR_UNSUPPORTED)
    wpack = torch.empty((wb,), dtype=torch.uint8, device=qweight.device)
    spack = torch.empty((sb,), dtype=torch.uint8, device=qweight.device)
    cpack = None if chan_scale is None else torch.empty((N,), dtype=torch.float32, device=qweight.device)
    is_float = scale.dtype == torch.float32
    st = lib.is_prepack_w4_gate_up(_p(qweight), None if is_float else _p(scale), _p(scale) if is_float else None,
                                   _p(chan_scale), inter, K, group, _p(wpack), _p(spack), _p(cpack), _stream_handle(stream))
    _check("is_prepack_w4_gate_up", st)
    return PackedGateUp(PackedWeights(wpack, spack, N, K, group, is_float), cpack, inter)


def is_gemm_gate_up_silu_prepacked_workspace_bytes(M: int, inter: int, K: int, group: int) -> int:
    return int(load_library().is_gemm_gate_up_silu_prepacked_workspace_bytes(M, inter, K, group))


def is_gemm_w4a8_intscale_gate_up_silu_prepacked(xq, a_scale, gate_up: PackedGateUp, alpha_log2: int, out=None,
                                                 acc_out=None, want_acc: bool = False, workspace=None, stream=None):
    """Returns (out fp16 [M, inter] = SiLU(gate) * up, acc int32 [M, 2 inter] in the packed row order or None)."""
    torch = _torch()
    M, K = xq.shape
    packed, inter = gate_up.packed, gate_up.inter
    if K != packed.K or packed.float_scales:
        raise ValueError("packed weights: K mismatch or float scales")
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    if out is None:
        out = torch.empty((M, inter), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, inter), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, 2 * inter), dtype=torch.int32, device=xq.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, 2 * inter), "acc_out")
    ws, ws_bytes = _zero_workspace(is_gemm_gate_up_silu_prepacked_workspace_bytes(M, inter, K, packed.group), xq.device,
                                   workspace)
    st = load_library().is_gemm_w4a8_intscale_gate_up_silu_prepacked(
        _p(xq), _p(a_scale), _p(packed.wpack), _p(packed.spack), _p(gate_up.chan_scale), M, inter, K, packed.group,
        alpha_log2, _p(out), _p(acc_out), _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_gemm_w4a8_intscale_gate_up_silu_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


def is_gemm_w4a8_floatscale_gate_up_silu_prepacked(xq, a_scale, gate_up: PackedGateUp, out=None, workspace=None,
                                                   stream=None):
    torch = _torch()
    M, K = xq.shape
    packed, inter = gate_up.packed, gate_up.inter
    if K != packed.K or not packed.float_scales:
        raise ValueError("packed weights: K mismatch or integer scales")
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    if out is None:
        out = torch.empty((M, inter), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, inter), "out")
    ws, ws_bytes = _zero_workspace(is_gemm_gate_up_silu_prepacked_workspace_bytes(M, inter, K, packed.group), xq.device,
                                   workspace)
    st = load_library().is_gemm_w4a8_floatscale_gate_up_silu_prepacked(
        _p(xq), _p(a_scale), _p(packed.wpack), _p(packed.spack), M, inter, K, packed.group, _p(out), _p(ws), ws_bytes,
        _stream_handle(stream))
    _check("is_gemm_w4a8_floatscale_gate_up_silu_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out


IS_NOALLOC_SCRATCH_BYTES = 32 << 20


def is_gemm_w4a8_intscale_prepacked_noalloc(xq, a_scale, packed: PackedWeights, chan_scale, alpha_log2: int, out,
                                            acc_out=None, stream=None):
    """The prepacked integer-scale GEMM on the library's fixed scratch: nothing is allocated, here or in the library, so
    `out` (fp16 [M,N]) and, if wanted, `acc_out` (int32 [M,N]) come from the caller.  Calls that overlap on one GPU
    race on the scratch."""
    torch = _torch()
    M, K = xq.shape
    N, group = packed.N, packed.group
    if K != packed.K or packed.float_scales:
        raise ValueError("packed weights: K mismatch or float scales")
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    _require(out, torch.float16, (M, N), "out")
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    st = load_library().is_gemm_w4a8_intscale_prepacked_noalloc(_p(xq), _p(a_scale), _p(packed.wpack), _p(packed.spack),
                                                               _p(chan_scale), M, N, K, group, alpha_log2, _p(out),
                                                               _p(acc_out), _stream_handle(stream))
    _check("is_gemm_w4a8_intscale_prepacked_noalloc", st)
    return out, acc_out


def is_prepare_activations_prepacked(xq, workspace, stream=None):
    """The tiled route's preparation of quantised activations [M,K] into `workspace` (a uint8 tensor the caller keeps
    for the *_prepared GEMMs that follow; size it with is_gemm_prepacked_workspace_bytes of the widest N)."""
    torch = _torch()
    M, K = xq.shape
    _require(xq, torch.int8, (M, K), "xq")
    st = load_library().is_prepare_activations_prepacked(_p(xq), M, K, _p(workspace), workspace.numel(),
                                                         _stream_handle(stream))
    _check("is_prepare_activations_prepacked", st)
    return workspace


def is_gemm_w4a8_intscale_prepacked_prepared(a_scale, packed: PackedWeights, chan_scale, alpha_log2: int, workspace,
                                             out=None, acc_out=None, want_acc=False, stream=None):
    """The prepacked integer-scale GEMM on a workspace is_prepare_activations_prepacked has filled (tiled kernel only)."""
    torch = _torch()
    M = a_scale.shape[0]
    N, K, group = packed.N, packed.K, packed.group
    if packed.float_scales:
        raise ValueError("packed weights: float scales")
    _require(a_scale, torch.float32, (M,), "a_scale")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a_scale.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=a_scale.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    st = load_library().is_gemm_w4a8_intscale_prepacked_prepared(
        _p(a_scale), _p(packed.wpack), _p(packed.spack), _p(chan_scale), M, N, K, group, alpha_log2, _p(out),
        _p(acc_out), _p(workspace), workspace.numel(), _stream_handle(stream))
    _check("is_gemm_w4a8_intscale_prepacked_prepared", st)
    return out, acc_out


def is_gemm_w4a8_floatscale_prepacked_prepared(a_scale, packed: PackedWeights, workspace, out=None, stream=None):
    torch = _torch()
    M = a_scale.shape[0]
    N, K, group = packed.N, packed.K, packed.group
    if not packed.float_scales:
        raise ValueError("packed weights: integer scales")
    _require(a_scale, torch.float32, (M,), "a_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a_scale.device)
    _require(out, torch.float16, (M, N), "out")
    st = load_library().is_gemm_w4a8_floatscale_prepacked_prepared(
        _p(a_scale), _p(packed.wpack), _p(packed.spack), M, N, K, group, _p(out), _p(workspace), workspace.numel(),
        _stream_handle(stream))
    _check("is_gemm_w4a8_floatscale_prepacked_prepared", st)
    return out


def is_gemm_w4a8_floatscale_prepacked(xq, a_scale, packed: PackedWeights, out=None, workspace=None, stream=None):
    torch = _torch()
    M, K = xq.shape
    N, group = packed.N, packed.group
    if K != packed.K or not packed.float_scales:
        raise ValueError("packed weights: K mismatch or integer scales")
    _require(xq, torch.int8, (M, K), "xq")
    _require(a_scale, torch.float32, (M,), "a_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _zero_workspace(is_gemm_prepacked_workspace_bytes(M, N, K, group), xq.device, workspace)
    st = load_library().is_gemm_w4a8_floatscale_prepacked(_p(xq), _p(a_scale), _p(packed.wpack), _p(packed.spack), M, N,
                                                         K, group, _p(out), _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_gemm_w4a8_floatscale_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out


def is_linear_w4a8_intscale_prepacked(x, packed: PackedWeights, chan_scale, alpha_log2: int, out=None, acc_out=None,
                                      want_acc: bool = False, workspace=None, stream=None):
    """fp16 activations in, prepacked weights. Returns (out fp16 [M,N], acc or None)."""
    torch = _torch()
    M, K = x.shape
    N, group = packed.N, packed.group
    if K != packed.K or packed.float_scales:
        raise ValueError("packed weights: K mismatch or float scales")
    _require(x, torch.float16, (M, K), "x")
    if chan_scale is not None:
        _require(chan_scale, torch.float32, (N,), "chan_scale")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _require(out, torch.float16, (M, N), "out")
    if acc_out is None and want_acc:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=x.device)
    if acc_out is not None:
        _require(acc_out, torch.int32, (M, N), "acc_out")
    ws, ws_bytes = _zero_workspace(is_linear_prepacked_workspace_bytes(M, N, K, group), x.device, workspace)
    st = load_library().is_linear_w4a8_intscale_prepacked(_p(x), _p(packed.wpack), _p(packed.spack), _p(chan_scale), M, N,
                                                         K, group, alpha_log2, _p(out), _p(acc_out), _p(ws), ws_bytes,
                                                         _stream_handle(stream))
    _check("is_linear_w4a8_intscale_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out, acc_out


def is_linear_w4a8_floatscale_prepacked(x, packed: PackedWeights, out=None, workspace=None, stream=None):
    torch = _torch()
    M, K = x.shape
    N, group = packed.N, packed.group
    if K != packed.K or not packed.float_scales:
        raise ValueError("packed weights: K mismatch or integer scales")
    _require(x, torch.float16, (M, K), "x")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _require(out, torch.float16, (M, N), "out")
    ws, ws_bytes = _zero_workspace(is_linear_prepacked_workspace_bytes(M, N, K, group), x.device, workspace)
    st = load_library().is_linear_w4a8_floatscale_prepacked(_p(x), _p(packed.wpack), _p(packed.spack), M, N, K, group,
                                                           _p(out), _p(ws), ws_bytes, _stream_handle(stream))
    _check("is_linear_w4a8_floatscale_prepacked", st)
    _release_workspace(ws, workspace, stream)
    return out
