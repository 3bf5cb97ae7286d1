"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header declares, and
rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

import paper_2405_14597_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "intscale.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(is_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree():
    names = declared_functions()
    assert set(names) == set(P.EXPORTED_SYMBOLS)
    lib = ctypes.CDLL(P.library_path())
    for n in names:
        assert hasattr(lib, n), f"libintscale.so does not export {n}"


def test_status_strings():
    assert P.status_string(P.IS_OK) == "IS_OK"
    assert P.status_string(P.IS_ERR_INVALID_ARG) == "IS_ERR_INVALID_ARG"
    assert P.status_string(P.IS_ERR_UNSUPPORTED) == "IS_ERR_UNSUPPORTED"
    assert P.status_string(P.IS_ERR_WORKSPACE) == "IS_ERR_WORKSPACE"
    assert P.status_string(P.IS_ERR_HIP) == "IS_ERR_HIP"
    assert P.status_string(-99) == "IS_ERR_UNKNOWN"


A = 0x10000  # a fake, 16-byte aligned "device pointer": validation must fail before it is ever dereferenced


def gemm_is(lib, xq=A, sa=A, qw=A, sc=A, cs=None, M=8, N=16, K=256, G=128, a=10, out=A, acc=None, ws=None, wsb=0):
    return lib.is_gemm_w4a8_intscale(xq, sa, qw, sc, cs, M, N, K, G, a, out, acc, ws, wsb, None)


def test_gemm_argument_validation():
    lib = P.load_library()
    bad = P.IS_ERR_INVALID_ARG
    assert gemm_is(lib, xq=None) == bad
    assert gemm_is(lib, sa=None) == bad
    assert gemm_is(lib, qw=None) == bad
    assert gemm_is(lib, sc=None) == bad
    assert gemm_is(lib, out=None) == bad
    assert gemm_is(lib, xq=A + 4) == bad            # misaligned
    assert gemm_is(lib, cs=A + 8) == bad
    assert gemm_is(lib, M=-1) == bad
    assert gemm_is(lib, N=0) == bad
    assert gemm_is(lib, K=0) == bad
    assert gemm_is(lib, K=200) == bad               # K not a multiple of group
    assert gemm_is(lib, a=-1) == bad
    assert gemm_is(lib, a=31) == bad
    assert gemm_is(lib, K=192, G=96) == P.IS_ERR_UNSUPPORTED   # neither a multiple of 128 nor 32 or 64
    assert gemm_is(lib, K=192, G=64, M=0) == P.IS_OK and gemm_is(lib, K=96, G=32, M=0) == P.IS_OK
    assert gemm_is(lib, K=192, G=64, sc=None) == bad
    # groups of 32 and 64 run a kernel that needs no workspace, whatever M is
    assert lib.is_gemm_workspace_bytes(4096, 16, 256, 64) == 0 and lib.is_gemm_workspace_bytes(4096, 16, 256, 128) > 0
    assert lib.is_gemm_grouped_workspace_bytes(2, 4096, 16, 256, 32) == 0
    assert gemm_is(lib, M=0) == P.IS_OK             # empty batch: nothing to do, nothing launched
    assert lib.is_gemm_workspace_bytes(8, 16, 256, 128) == 0


def test_floatscale_and_grouped_argument_validation():
    lib = P.load_library()
    bad = P.IS_ERR_INVALID_ARG
    assert lib.is_gemm_w4a8_floatscale(A, A, A, None, 8, 16, 256, 128, A, None, 0, None) == bad
    assert lib.is_gemm_w4a8_floatscale(A, A, A, A, 8, 16, 100, 128, A, None, 0, None) == bad
    assert lib.is_gemm_w4a8_intscale_grouped(A, A, A, A, None, None, 4, 8, 16, 256, 128, 10, A, None, None, 0, None) == bad
    assert lib.is_gemm_w4a8_intscale_grouped(A, A, A, A, None, A, 0, 8, 16, 256, 128, 10, A, None, None, 0, None) == bad
    assert lib.is_gemm_w4a8_floatscale_grouped(A, A, A, A, A + 2, 4, 8, 16, 256, 128, A, None, 0, None) == bad


def test_overflow_entry_points_argument_validation():
    lib = P.load_library()
    bad = P.IS_ERR_INVALID_ARG
    assert lib.is_intscale_overflow_bound(None, 16, 256, 128, A, None) == bad
    assert lib.is_intscale_overflow_bound(A, 16, 256, 128, None, None) == bad
    assert lib.is_intscale_overflow_bound(A, 16, 256, 128, A + 4, None) == bad      # 8-byte alignment of the result
    assert lib.is_intscale_overflow_bound(A, 0, 256, 128, A, None) == bad
    assert lib.is_intscale_overflow_bound(A, 16, 250, 128, A, None) == bad
    need = lib.is_gemm_safe_workspace_bytes(8, 16, 256, 128)
    assert need >= 16 * 2 * 4 and lib.is_gemm_safe_workspace_bytes(8, 16, 250, 128) == 0
    safe = lambda **kw: lib.is_gemm_w4a8_intscale_safe(
        kw.get("xq", A), kw.get("sa", A), kw.get("q", A), kw.get("si", A), kw.get("c", None), kw.get("M", 8), 16,
        kw.get("K", 256), 128, kw.get("a", 10), kw.get("out", A), kw.get("ws", A), kw.get("wsb", need), None)
    assert safe(si=None) == bad and safe(q=None) == bad and safe(xq=None) == bad and safe(out=None) == bad
    assert safe(a=31) == bad and safe(K=250) == bad and safe(c=A + 4) == bad
    assert safe(ws=None) == P.IS_ERR_WORKSPACE and safe(wsb=need - 1) == P.IS_ERR_WORKSPACE


def test_quantizer_argument_validation():
    lib = P.load_library()
    bad = P.IS_ERR_INVALID_ARG
    q = lambda **kw: lib.is_quantize_weights_int4_group(
        kw.get("w", A), kw.get("N", 16), kw.get("K", 256), kw.get("G", 128), kw.get("a", 10), kw.get("mode", 0),
        kw.get("q", A), kw.get("s", A), kw.get("si", A), kw.get("c", A), kw.get("adev", None), None)
    assert q(w=None) == bad and q(q=None) == bad and q(s=None) == bad and q(si=None) == bad and q(c=None) == bad
    assert q(N=0) == bad and q(K=255) == bad and q(G=100) == bad and q(G=0) == bad
    assert q(a=17) == bad and q(a=-2) == bad and q(mode=2) == bad
    assert q(a=-1, adev=None) == bad                # the amplifier search needs somewhere to put its result
    x = lambda **kw: lib.is_quantize_act_int8_token(kw.get("x", A), kw.get("M", 4), kw.get("K", 256), kw.get("xq", A),
                                                    kw.get("sa", A), None)
    assert x(x=None) == bad and x(xq=None) == bad and x(sa=None) == bad
    assert x(K=100) == bad and x(M=-1) == bad
    assert x(M=0) == P.IS_OK


def test_fused_producer_argument_validation():
    lib = P.load_library()
    bad = P.IS_ERR_INVALID_ARG
    n = lambda **kw: lib.is_rmsnorm_quantize_act_int8_token(kw.get("x", A), kw.get("g", A), kw.get("eps", 1e-5),
                                                            kw.get("M", 4), kw.get("K", 256), kw.get("xq", A),
                                                            kw.get("sa", A), None)
    assert n(x=None) == bad and n(g=None) == bad and n(xq=None) == bad and n(sa=None) == bad and n(sa=A + 2) == bad
    assert n(K=100) == bad and n(K=0) == bad and n(M=-1) == bad
    assert n(eps=0.0) == bad and n(eps=-1e-5) == bad and n(eps=float("inf")) == bad and n(eps=float("nan")) == bad
    assert n(M=0) == P.IS_OK
    s = lambda **kw: lib.is_silu_mul_quantize_act_int8_token(kw.get("gu", A), kw.get("M", 4), kw.get("I", 256),
                                                             kw.get("xq", A), kw.get("sa", A), None)
    assert s(gu=None) == bad and s(xq=None) == bad and s(sa=None) == bad
    assert s(I=100) == bad and s(I=0) == bad and s(M=-1) == bad
    assert s(M=0) == P.IS_OK


def test_linear_argument_validation():
    lib = P.load_library()
    bad = P.IS_ERR_INVALID_ARG
    need = lib.is_linear_workspace_bytes(8, 16, 256, 128)
    assert need >= 8 * 256 + 8 * 4 and lib.is_linear_workspace_bytes(8, 16, 250, 128) == 0
    assert lib.is_linear_workspace_bytes(0, 16, 256, 128) == 0
    lin = lambda **kw: lib.is_linear_w4a8_intscale(
        kw.get("x", A), kw.get("q", A), kw.get("si", A), kw.get("c", None), kw.get("M", 8), 16, kw.get("K", 256), 128,
        kw.get("a", 10), kw.get("out", A), None, kw.get("ws", A), kw.get("wsb", need), None)
    assert lin(x=None) == bad and lin(q=None) == bad and lin(si=None) == bad and lin(out=None) == bad
    assert lin(a=31) == bad and lin(K=250) == bad and lin(c=A + 4) == bad and lin(M=-1) == bad
    assert lin(ws=None) == P.IS_ERR_WORKSPACE and lin(wsb=need - 1) == P.IS_ERR_WORKSPACE
    assert lin(M=0, ws=None, wsb=0) == P.IS_OK
    assert lib.is_linear_w4a8_floatscale(A, A, None, 8, 16, 256, 128, A, A, need, None) == bad


def test_w8a8_rejects_weights_of_2gib_and_more():
    """The W8A8 kernels index the int8 weights with 32-bit offsets: N * K >= 2^31 must be refused, not wrapped."""
    lib = P.load_library()
    call = lambda N, K: lib.is_gemm_w8a8_intscale(A, A, A, A, None, 8, N, K, 128, 10, A, None, None, 0, None)
    assert call(1 << 16, 1 << 15) == P.IS_ERR_UNSUPPORTED          # exactly 2^31 weights
    assert call(1 << 17, 1 << 15) == P.IS_ERR_UNSUPPORTED
    assert lib.is_gemm_w8a8_workspace_bytes(8, 1 << 16, 1 << 15, 128) == 0
    assert call(1 << 16, (1 << 15) - 128) != P.IS_ERR_UNSUPPORTED  # just below: passes the shape check


def test_prepacked_argument_validation():
    lib = P.load_library()
    bad, uns = P.IS_ERR_INVALID_ARG, P.IS_ERR_UNSUPPORTED
    assert lib.is_prepack_w4_weight_bytes(16, 256) == 2048 and lib.is_prepack_w4_weight_bytes(17, 256) == 4096
    assert lib.is_prepack_w4_scale_bytes(16, 256, 128) == 256 + 2 * 64
    assert lib.is_prepack_w4_weight_bytes(16, 200) == 0 and lib.is_prepack_w4_scale_bytes(16, 256, 64) == 0
    pre = lambda **kw: lib.is_prepack_w4(kw.get("q", A), kw.get("si", A), kw.get("sf", None), 16, kw.get("K", 256),
                                         kw.get("G", 128), kw.get("wp", A), kw.get("sp", A), None)
    assert pre(q=None) == bad and pre(wp=None) == bad and pre(sp=None) == bad
    assert pre(si=None) == bad and pre(sf=A) == bad            # exactly one kind of scales
    assert pre(G=64) == uns and pre(K=192, G=64) == uns and pre(K=250) == bad
    gemm = lambda **kw: lib.is_gemm_w4a8_intscale_prepacked(
        kw.get("xq", A), kw.get("sa", A), kw.get("wp", A), kw.get("sp", A), kw.get("c", None), kw.get("M", 8), 16,
        kw.get("K", 256), kw.get("G", 128), kw.get("a", 10), kw.get("out", A), None, kw.get("ws", None),
        kw.get("wsb", 0), None)
    assert gemm(xq=None) == bad and gemm(sa=None) == bad and gemm(wp=None) == bad and gemm(sp=None) == bad
    assert gemm(out=None) == bad and gemm(a=31) == bad and gemm(M=-1) == bad and gemm(c=A + 4) == bad
    assert gemm(G=64) == uns and gemm(M=0) == P.IS_OK
    need = lib.is_gemm_prepacked_workspace_bytes(128, 16, 256, 128)   # tiled route: prepared activations
    assert need >= 128 * 256
    assert gemm(M=128, ws=None) == P.IS_ERR_WORKSPACE and gemm(M=128, ws=A, wsb=need - 1) == P.IS_ERR_WORKSPACE
    lneed = lib.is_linear_prepacked_workspace_bytes(8, 16, 256, 128)
    lin = lambda **kw: lib.is_linear_w4a8_intscale_prepacked(
        kw.get("x", A), kw.get("wp", A), kw.get("sp", A), None, kw.get("M", 8), 16, kw.get("K", 256), 128, 10,
        kw.get("out", A), None, kw.get("ws", A), kw.get("wsb", lneed), None)
    assert lneed >= 8 * 256 + 8 * 4
    assert lin(x=None) == bad and lin(wp=None) == bad and lin(out=None) == bad and lin(K=250) == bad
    assert lin(ws=None) == P.IS_ERR_WORKSPACE and lin(wsb=lneed - 1) == P.IS_ERR_WORKSPACE
    assert lin(M=0, ws=None, wsb=0) == P.IS_OK


def test_grouped_prepacked_argument_validation():
    lib = P.load_library()
    bad, uns = P.IS_ERR_INVALID_ARG, P.IS_ERR_UNSUPPORTED
    need = lib.is_gemm_grouped_prepacked_workspace_bytes(4, 300, 48, 1024, 128)
    # activations padded per expert to 16-row tiles, corrections, table
    assert need >= (300 // 16 + 4) * 16 * 1024
    assert lib.is_gemm_grouped_prepacked_workspace_bytes(4, 0, 48, 1024, 128) == 0
    assert lib.is_gemm_grouped_prepacked_workspace_bytes(0, 300, 48, 1024, 128) == 0
    assert lib.is_gemm_grouped_prepacked_workspace_bytes(4, 300, 48, 1000, 128) == 0
    call = lambda **kw: lib.is_gemm_w4a8_intscale_grouped_prepacked(
        kw.get("xq", A), kw.get("sa", A), kw.get("wp", A), kw.get("sp", A), kw.get("c", None), kw.get("off", A),
        kw.get("E", 4), kw.get("M", 300), 48, kw.get("K", 1024), kw.get("G", 128), kw.get("a", 10), kw.get("out", A), None,
        kw.get("ws", A), kw.get("wsb", need), None)
    assert call(xq=None) == bad and call(sa=None) == bad and call(wp=None) == bad and call(sp=None) == bad
    assert call(off=None) == bad and call(off=A + 2) == bad and call(out=None) == bad and call(a=31) == bad
    assert call(E=0) == bad and call(M=-1) == bad and call(K=1000) == bad and call(c=A + 4) == bad
    assert call(G=64) == uns and call(E=2000) == uns
    assert call(ws=None) == P.IS_ERR_WORKSPACE and call(wsb=need - 1) == P.IS_ERR_WORKSPACE
    assert call(M=0, ws=None, wsb=0) == P.IS_OK
    assert lib.is_gemm_w4a8_floatscale_grouped_prepacked(A, A, A, A, None, 4, 300, 48, 1024, 128, A, A, need, None) == bad


def test_noalloc_argument_validation():
    """The entry point without a workspace checks shapes and the size of its fixed scratch before any HIP call."""
    lib = P.load_library()
    bad = P.IS_ERR_INVALID_ARG
    call = lambda **kw: lib.is_gemm_w4a8_intscale_prepacked_noalloc(
        kw.get("xq", A), kw.get("sa", A), kw.get("wp", A), kw.get("sp", A), None, kw.get("M", 8), kw.get("N", 16),
        kw.get("K", 256), kw.get("G", 128), kw.get("a", 10), kw.get("out", A), None, None)
    assert call(M=-1) == bad and call(K=250) == bad and call(G=64) == P.IS_ERR_UNSUPPORTED
    assert call(xq=None) == bad and call(wp=None) == bad and call(out=None) == bad and call(a=31) == bad
    assert call(M=0) == P.IS_OK
    assert lib.is_gemm_prepacked_workspace_bytes(2048, 256, 28672, 128) > P.IS_NOALLOC_SCRATCH_BYTES
    assert call(M=2048, N=256, K=28672) == P.IS_ERR_WORKSPACE


def test_shared_preparation_argument_validation():
    """The preparation of shared activations and the GEMMs on a prepared workspace check shapes, route and workspace
    before any HIP call: only shapes of the tiled route have a preparation."""
    lib = P.load_library()
    bad, unsup = P.IS_ERR_INVALID_ARG, P.IS_ERR_UNSUPPORTED
    big = 1 << 30
    prep = lambda **kw: lib.is_prepare_activations_prepacked(kw.get("xq", A), kw.get("M", 128), kw.get("K", 256),
                                                             kw.get("ws", A), kw.get("wsb", big), None)
    assert prep(M=-1) == bad and prep(K=0) == bad and prep(K=200) == unsup and prep(M=32) == unsup and prep(M=1) == unsup
    assert prep(M=0) == P.IS_OK
    assert prep(ws=None) == P.IS_ERR_WORKSPACE and prep(wsb=1024) == P.IS_ERR_WORKSPACE and prep(xq=None) == bad
    assert prep(M=1 << 20, K=1 << 12) == unsup      # 32-bit offsets
    gemm = lambda **kw: lib.is_gemm_w4a8_intscale_prepacked_prepared(
        kw.get("sa", A), kw.get("wp", A), kw.get("sp", A), None, kw.get("M", 128), kw.get("N", 16), kw.get("K", 256),
        kw.get("G", 128), kw.get("a", 10), kw.get("out", A), None, kw.get("ws", A), kw.get("wsb", big), None)
    assert gemm(M=64) == unsup and gemm(M=8) == unsup                      # the weight-streaming kernel's shapes
    assert gemm(M=-1) == bad and gemm(G=64) == unsup and gemm(a=31) == bad
    assert gemm(ws=None) == P.IS_ERR_WORKSPACE and gemm(wsb=64) == P.IS_ERR_WORKSPACE
    assert gemm(sa=None) == bad and gemm(wp=None) == bad and gemm(out=None) == bad
    assert gemm(M=0) == P.IS_OK
    fs = lib.is_gemm_w4a8_floatscale_prepacked_prepared
    assert fs(A, A, A, 64, 16, 256, 128, A, A, big, None) == unsup and fs(None, A, A, 128, 16, 256, 128, A, A, big, None) == bad


def test_gate_up_silu_argument_validation():
    lib = P.load_library()
    bad, uns = P.IS_ERR_INVALID_ARG, P.IS_ERR_UNSUPPORTED
    pre = lambda **kw: lib.is_prepack_w4_gate_up(kw.get("q", A), kw.get("si", A), kw.get("sf", None), kw.get("c", None),
                                                 kw.get("inter", 16), kw.get("K", 256), kw.get("G", 128), kw.get("wp", A),
                                                 kw.get("sp", A), kw.get("cp", None), None)
    assert pre(q=None) == bad and pre(wp=None) == bad and pre(sp=None) == bad and pre(si=None) == bad and pre(sf=A) == bad
    assert pre(c=A) == bad and pre(cp=A) == bad          # channel scales in and out go together
    assert pre(inter=0) == bad and pre(inter=24) == uns and pre(G=64) == uns and pre(K=250) == bad
    wsb = lib.is_gemm_gate_up_silu_prepacked_workspace_bytes
    assert wsb(8, 24, 256, 128) == 0 and wsb(8, 16, 256, 64) == 0 and wsb(0, 16, 256, 128) == 0
    # up to 64 token rows: the [M, 2 inter] fp16 tensor on top of the GEMM's own workspace
    assert wsb(8, 16, 256, 128) == lib.is_gemm_prepacked_workspace_bytes(8, 32, 256, 128) + 8 * 32 * 2
    assert wsb(128, 16, 256, 128) == lib.is_gemm_prepacked_workspace_bytes(128, 32, 256, 128)
    gemm = lambda **kw: lib.is_gemm_w4a8_intscale_gate_up_silu_prepacked(
        kw.get("xq", A), kw.get("sa", A), kw.get("wp", A), kw.get("sp", A), kw.get("c", None), kw.get("M", 8),
        kw.get("inter", 16), kw.get("K", 256), kw.get("G", 128), kw.get("a", 10), kw.get("out", A), None, kw.get("ws", A),
        kw.get("wsb", 1 << 20), None)
    assert gemm(inter=0) == bad and gemm(inter=24) == uns and gemm(M=-1) == bad and gemm(G=64) == uns
    assert gemm(ws=None) == P.IS_ERR_WORKSPACE and gemm(wsb=100) == P.IS_ERR_WORKSPACE and gemm(out=None) == bad
    assert gemm(M=128, ws=None, wsb=0) == P.IS_ERR_WORKSPACE and gemm(M=128, xq=None) == bad and gemm(M=128, a=31) == bad
    assert gemm(M=0, ws=None, wsb=0) == P.IS_OK
    fs = lib.is_gemm_w4a8_floatscale_gate_up_silu_prepacked
    assert fs(A, A, A, A, 8, 24, 256, 128, A, A, 1 << 20, None) == uns
    assert fs(A, A, A, A, 128, 16, 256, 128, None, A, 1 << 20, None) == bad


def test_describe_prepacked_names_the_kernels():
    one = P.is_describe_prepacked(1, 8192, 8192, 128, True, True)
    assert len(one) == 1 and one[0].startswith("gemm_decode_pk_kernel<1, ") and one[0].endswith("true, true>")
    dec = P.is_describe_prepacked(32, 8192, 8192, 128, False, False)
    assert dec[0].startswith("gemm_decode_pk_kernel<2, ") and dec[0].endswith("false, false>")
    til = P.is_describe_prepacked(2048, 8192, 8192, 128, True, True)
    assert til == ["quantize_prepare_rows_pk_kernel", "gemm_tile_pk_kernel<true>"]
    assert P.is_describe_prepacked(2048, 8192, 8192, 128, False, False)[0] == "prepare_activations_pk_kernel"
    with pytest.raises(P.IntScaleError):
        P.is_describe_prepacked(8, 16, 256, 64)
    lib = P.load_library()
    buf = ctypes.create_string_buffer(8)
    assert lib.is_describe_prepacked(1, 16, 256, 128, 1, 0, buf, 8) == P.IS_OK and len(buf.value) <= 7   # truncated, terminated
    assert lib.is_describe_prepacked(1, 16, 256, 128, 1, 0, None, 8) == P.IS_ERR_INVALID_ARG
    grp = P.is_describe_grouped_prepacked(8, 1024, 14336, 4096, 128, True)
    assert grp == ["prepare_activations_grouped_pk_kernel", "gemm_tile_grouped_pk_kernel<true>"]
    assert P.is_describe_grouped_prepacked(8, 1024, 14336, 4096, 128, False)[1] == "gemm_tile_grouped_pk_kernel<false>"
    assert lib.is_describe_grouped_prepacked(0, 16, 256, 128, 128, 1, buf, 8) == P.IS_ERR_INVALID_ARG
    assert lib.is_describe_grouped_prepacked(2, 16, 256, 128, 64, 1, buf, 8) == P.IS_ERR_UNSUPPORTED


def test_kernel_route_override_is_a_host_setting():
    """The routing override of the tests is a call, not an environment read on the launch path: it returns the setting
    in force before, rejects unknown routes and leaves the setting alone when it does."""
    lib = P.load_library()
    first = P.is_set_kernel_route("general")
    try:
        assert P.is_set_kernel_route("tiled") == "general"
        assert lib.is_set_kernel_route(4) == P.IS_ERR_INVALID_ARG and lib.is_set_kernel_route(-1) == P.IS_ERR_INVALID_ARG
        assert P.is_set_kernel_route("auto") == "tiled"
    finally:
        P.is_set_kernel_route(first)
    assert P.is_set_kernel_route(first) == first


def test_library_carries_the_digest_of_its_sources():
    from paper_2405_14597_amd import build
    assert P.load_library().is_source_hash().decode() == build.source_hash() == build.built_hash()
    assert not build.needs_build()


def test_missing_device_is_reported_not_hidden():
    """With valid arguments the call reaches HIP; without a GPU that must surface as IS_ERR_HIP, never as success."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = P.load_library()
    assert gemm_is(lib) == P.IS_ERR_HIP
    assert P.last_hip_error() != ""
