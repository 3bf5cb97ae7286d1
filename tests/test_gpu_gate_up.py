"""GPU parity of the fused gate / up projection with SiLU(gate) * up as the GEMM's epilogue (kernel fusion around the
GEMM, Sec. 4.2), through the C ABI, against the CPU oracle: the paired kernel layout against its definition, int32
accumulators bit for bit, the fp16 result within the stated tolerance of the oracle's unfused sequence (integer-scale
GEMM of Eq. (2) -> fp16 -> SiLU * up) and bit for bit equal to that sequence applied to the library's own GEMM output,
in both regimes (weight-streaming kernel + second kernel up to 64 token rows, tiled kernel's epilogue above), with
the K range of the last round's tiles cut into parts, and the float-scale twin (Eq. (1)).
"""
import numpy as np
import pytest

from oracle import oracle as O
from test_gpu_parity import dev, host
from test_gpu_prepacked import packed_layout_numpy

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

G = 128


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_14597_amd as pkg
    pkg.load_library()
    return pkg


def paired_rows(inter):
    """Canonical row (gate rows, then up rows) of every packed row: tiles of 16 gate rows and 16 up rows alternate."""
    n = np.arange(2 * inter)
    t = n // 16
    return np.where(t % 2 == 1, inter, 0) + (t // 2) * 16 + n % 16


def make(rng, M, inter, K, wide=False):
    N = 2 * inter
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    sa = (rng.random(M) * 0.02 + 0.001).astype(np.float32)
    qw = O.pack_int4(rng.integers(-8, 8, size=(N, K)).astype(np.int8))
    IS = rng.integers(0, 1025, size=(N, K // G)).astype(np.int32)
    if wide:
        IS[3, 0] = 2 ** 25
    s = (rng.random((N, K // G)) * 0.01).astype(np.float32)
    c = (rng.random(N) * 0.01 + 0.001).astype(np.float32)
    return xq, sa, qw, IS, s, c


@pytest.mark.parametrize("inter,K", [(16, 128), (48, 1024), (272, 512)])
def test_gate_up_prepack_pairs_the_rows(P, inter, K):
    rng = np.random.default_rng(inter + K)
    _, _, qw, IS, s, c = make(rng, 1, inter, K)
    rows = paired_rows(inter)
    for scale in (IS, s):
        gu = P.is_prepack_w4_gate_up(dev(qw), dev(scale), dev(c), G)
        w_ref, s_ref = packed_layout_numpy(qw[rows], scale[rows], G)        # the plain layout of the permuted matrix
        assert np.array_equal(host(gu.packed.wpack), w_ref)
        body = host(gu.packed.spack)[256:].view(scale.dtype)
        assert np.array_equal(body, s_ref)
        header = host(gu.packed.spack)[:256].view(np.int32)
        assert header[0] & 4 and header[1] == 2 * inter and header[2] == K and header[3] == G and header[4] == inter
        assert np.array_equal(host(gu.chan_scale), c[rows])
    assert P.is_prepack_w4_gate_up(dev(qw), dev(IS), None, G).chan_scale is None


def reference(xq, sa, qw, IS, c, inter, a=10):
    """The oracle's unfused sequence on the canonical fused projection: (acc [M, 2 inter], h fp16 [M, inter])."""
    r = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, a)
    return r.acc, O.silu_mul_fp16(r.out.astype(np.float16))


@pytest.mark.parametrize("M,inter,K,wide", [(1, 48, 256, False), (24, 272, 1024, False), (64, 16, 128, True),
                                             (65, 48, 1024, False), (130, 272, 512, True), (300, 144, 256, False),
                                             (256, 4096, 1024, False)])
def test_gate_up_silu_intscale(P, M, inter, K, wide):
    rng = np.random.default_rng(9000 + M + inter + K)
    xq, sa, qw, IS, _, c = make(rng, M, inter, K, wide)
    rows = paired_rows(inter)
    acc_ref, h_ref = reference(xq, sa, qw, IS, c, inter)
    gu = P.is_prepack_w4_gate_up(dev(qw), dev(IS), dev(c), G)
    ws = torch.full((max(16, P.is_gemm_gate_up_silu_prepacked_workspace_bytes(M, inter, K, G)),), 0, dtype=torch.uint8,
                    device="cuda:0")
    h, acc = P.is_gemm_w4a8_intscale_gate_up_silu_prepacked(dev(xq), dev(sa), gu, 10, want_acc=True, workspace=ws)
    assert np.array_equal(host(acc), acc_ref[:, rows]), "int32 accumulators (packed row order)"
    h2, _ = P.is_gemm_w4a8_intscale_gate_up_silu_prepacked(dev(xq), dev(sa), gu, 10, workspace=ws)   # 16-byte stores
    assert np.array_equal(host(h2).view(np.uint16), host(h).view(np.uint16))
    got, want = host(h).astype(np.float64), h_ref.astype(np.float64)
    # g and u may each sit one fp16 step from the oracle's (fp32 epilogue against the oracle's double), the product then
    # within a few: the stated tolerance of the fp16 outputs
    assert np.all(np.abs(got - want) <= 1e-2 * np.abs(want) + 2.0 ** -24)
    # bit for bit the unfused sequence on the library's own fp16 GEMM output (the plain GEMM call on the paired rows)
    wsg = torch.zeros((max(16, P.is_gemm_prepacked_workspace_bytes(M, 2 * inter, K, G)),), dtype=torch.uint8, device="cuda:0")
    plain, _ = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), gu.packed, gu.chan_scale, 10, workspace=wsg)
    canonical = np.empty((M, 2 * inter), np.float16)
    canonical[:, rows] = host(plain)
    assert np.array_equal(host(h).view(np.uint16), O.silu_mul_fp16(canonical).view(np.uint16))


@pytest.mark.parametrize("M,inter,K,wide", [(40, 272, 1024, False), (64, 48, 256, True), (33, 4096, 512, False)])
def test_gate_up_silu_33_to_64_rows_on_the_tiled_kernel(P, M, inter, K, wide):
    """The route large projections take at 33..64 rows: the tiled kernel's 64-row instance with the fused epilogue."""
    before = P.is_set_kernel_route("tiled64")
    try:
        test_gate_up_silu_intscale(P, M, inter, K, wide)
    finally:
        P.is_set_kernel_route(before)


@pytest.mark.parametrize("M,inter,K", [(8, 48, 256), (200, 272, 1024)])
def test_gate_up_silu_floatscale(P, M, inter, K):
    rng = np.random.default_rng(9100 + M + inter)
    xq, sa, qw, _, s, _ = make(rng, M, inter, K)
    rows = paired_rows(inter)
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, G)
    gu = P.is_prepack_w4_gate_up(dev(qw), dev(s), None, G)
    h = host(P.is_gemm_w4a8_floatscale_gate_up_silu_prepacked(dev(xq), dev(sa), gu))
    plain = host(P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), gu.packed))
    canonical = np.empty((M, 2 * inter), np.float16)
    canonical[:, rows] = plain
    assert np.array_equal(h.view(np.uint16), O.silu_mul_fp16(canonical).view(np.uint16))
    # against the oracle's float-scale result: its outputs carry the summation-order tolerance of Eq. (1); where gate and
    # up both lie within one fp16 step of the oracle's the product does too
    g_ref, u_ref = fs.out[:, :inter], fs.out[:, inter:]
    want = O.silu_mul_fp16(np.concatenate([g_ref, u_ref], axis=1).astype(np.float16)).astype(np.float64)
    tol = 2e-2 * np.abs(want) + 1e-4 * (np.abs(u_ref) * fs.abs_sum[:, :inter] + np.abs(g_ref) * fs.abs_sum[:, inter:]) + 1e-7
    assert np.all(np.abs(h.astype(np.float64) - want) <= tol)


def test_gate_up_silu_arguments(P):
    rng = np.random.default_rng(5)
    xq, sa, qw, IS, _, c = make(rng, 70, 48, 256)
    gu = P.is_prepack_w4_gate_up(dev(qw), dev(IS), dev(c), G)
    lib = P.load_library()
    out = torch.empty((70, 48), dtype=torch.float16, device="cuda:0")
    need = P.is_gemm_gate_up_silu_prepacked_workspace_bytes(70, 48, 256, G)
    ws = torch.zeros((need,), dtype=torch.uint8, device="cuda:0")
    args = lambda inter, nbytes: (dev(xq).data_ptr(), dev(sa).data_ptr(), gu.packed.wpack.data_ptr(), gu.packed.spack.data_ptr(),
                                  gu.chan_scale.data_ptr(), 70, inter, 256, G, 10, out.data_ptr(), None, ws.data_ptr(), nbytes, None)
    assert lib.is_gemm_w4a8_intscale_gate_up_silu_prepacked(*args(48, need - 1)) == P.IS_ERR_WORKSPACE
    assert lib.is_gemm_w4a8_intscale_gate_up_silu_prepacked(*args(40, need)) == P.IS_ERR_UNSUPPORTED
    assert lib.is_gemm_w4a8_intscale_gate_up_silu_prepacked(*args(0, need)) == P.IS_ERR_INVALID_ARG
    empty, _ = P.is_gemm_w4a8_intscale_gate_up_silu_prepacked(torch.empty((0, 256), dtype=torch.int8, device="cuda:0"),
                                                              torch.empty((0,), dtype=torch.float32, device="cuda:0"), gu, 10)
    assert empty.shape == (0, 48)
