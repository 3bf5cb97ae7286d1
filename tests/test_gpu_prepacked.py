"""GPU parity of the prepacked route (kernel layout of the weights + the weight-streaming decode kernel) against the
CPU oracle, through the C ABI: the packed layout byte for byte against its definition written out in numpy, int32
accumulators bit-exact, fp16 outputs within the stated tolerance, for every token-tile count, every number of token
rows kept in LDS, with and without the K split across workgroups, ragged N, wide scales, wide groups, the float-scale
twin, and the one-call linear layer on fp16 activations.
"""
import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O
from test_gpu_parity import check_fs, check_out, dev, host, rand_quantised

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


def packed_layout_numpy(qweight, scale, group):
    """The kernel layout as include/intscale.h defines it, element by element."""
    N, K2 = qweight.shape
    K = 2 * K2
    q = O.unpack_int4(qweight).astype(np.int64) & 0xF          # two's-complement nibbles [N,K]
    n16, steps = (N + 15) // 16, K // 128
    qp = np.zeros((n16 * 16, K), np.int64)
    qp[:N] = q
    w = np.zeros((n16, steps, 4, 16, 16), np.uint8)             # [tile][step][kb][row][byte]
    for kb in range(4):
        for j in range(16):
            lo = qp[:, np.arange(steps) * 128 + 16 * kb + j]           # [rows, steps]
            hi = qp[:, np.arange(steps) * 128 + 64 + 16 * kb + j]
            b = (lo | (hi << 4)).astype(np.uint8).reshape(n16, 16, steps)
            w[:, :, kb, :, j] = b.transpose(0, 2, 1)
    NG = K // group
    sp = np.zeros((n16 * 16, NG), scale.dtype)
    sp[:N] = scale
    s = sp.reshape(n16, 16, NG).transpose(0, 2, 1)                # [tile][group][row]
    return w.reshape(-1), np.ascontiguousarray(s).reshape(-1)


@pytest.mark.parametrize("N,K,group", [(16, 128, 128), (40, 1024, 128), (272, 4096, 256), (100, 1536, 512)])
def test_prepack_layout(P, N, K, group):
    rng = np.random.default_rng(N + K)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    qw = O.pack_int4(q)
    IS = rng.integers(-2 ** 20, 2 ** 20, size=(N, K // group)).astype(np.int32)
    s = rng.random((N, K // group)).astype(np.float32)
    for scale, is_float in ((IS, False), (s, True)):
        pk = P.is_prepack_w4(dev(qw), dev(scale), group)
        w_ref, s_ref = packed_layout_numpy(qw, scale, group)
        assert np.array_equal(host(pk.wpack), w_ref)
        sp = host(pk.spack)
        header = sp[:256].view(np.int32)
        assert header[0] == (2 if is_float else 0) and tuple(header[1:4]) == (N, K, group)
        assert np.array_equal(sp[256:].view(scale.dtype), s_ref)
    wide = IS.copy()
    wide[N // 2, 0] = 2 ** 23
    assert host(P.is_prepack_w4(dev(qw), dev(wide), group).spack)[:4].view(np.int32)[0] == 1
    wide[N // 2, 0] = -2 ** 23
    assert host(P.is_prepack_w4(dev(qw), dev(wide), group).spack)[:4].view(np.int32)[0] == 0


# (M, N, K): one, two and four token tiles; 1, 2, 4, 8, 16 token rows kept in LDS; fewer blocks than waves; row tiles
# shared by several waves and whole tiles inside one wave; many tiles per workgroup; K split across workgroups
# (K = 11008 at 16 rows, 8192 and 28672 at 32 rows, 4096 and 11008 at 64 rows); ragged N
PK_SHAPES = [(1, 16, 128), (1, 4096, 4096), (1, 100, 20480), (2, 4200, 1024), (3, 272, 2048), (5, 8208, 512),
             (8, 4096, 4096), (9, 40, 1024), (16, 272, 1024), (16, 5008, 11008), (16, 12288, 256), (17, 40, 1024),
             (24, 4120, 1024), (32, 4360, 8192), (32, 528, 28672), (33, 100, 2048), (48, 2064, 3584), (64, 4096, 1024),
             (64, 48, 11008), (64, 8208, 4096), (40, 4200, 1024), (1, 22016, 4096), (16, 22016, 4096), (7, 1, 256)]


@pytest.mark.parametrize("M,N,K", PK_SHAPES)
def test_prepacked_gemm_intscale_bit_exact_acc(P, M, N, K):
    rng = np.random.default_rng(1500 + M + N + K)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
    pk = P.is_prepack_w4(dev(qw), dev(IS), G)
    out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")
    ref1 = O.gemm_w4a8_intscale(xq, sa, qw, IS, None, G, 7)
    out1, acc1 = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, None, 7)
    assert acc1 is None
    check_out(host(out1), ref1.out)


@pytest.mark.parametrize("M,N,K", PK_SHAPES)
def test_prepacked_gemm_floatscale(P, M, N, K):
    rng = np.random.default_rng(2500 + M + N + K)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, G)
    pk = P.is_prepack_w4(dev(qw), dev(s), G)
    out = P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), pk)
    check_fs(host(out), fs, f"M{M} N{N} K{K}")


@pytest.mark.parametrize("M,K", [(16, 4096), (64, 4096), (32, 8192)])
def test_prepacked_extreme_codes_and_wide_scales(P, M, K):
    """All codes at -128 / -8, negative and wider-than-24-bit integer scales, wrap-around; with and without K split."""
    N = 32
    xq = np.full((M, K), -128, np.int8)
    q = np.full((N, K), -8, np.int8)
    xq[1::2] = 127
    q[::3] = 7
    rng = np.random.default_rng(5)
    sa = np.ones(M, np.float32)
    for IS in (np.full((N, K // G), 511, np.int32), np.full((N, K // G), 40000, np.int32),
               rng.integers(-2 ** 31, 2 ** 31, size=(N, K // G), dtype=np.int64).astype(np.int32),
               rng.integers(-2 ** 23, 2 ** 23, size=(N, K // G), dtype=np.int64).astype(np.int32)):
        ref = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, None, G, 10)
        pk = P.is_prepack_w4(dev(O.pack_int4(q)), dev(IS), G)
        out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, None, 10, want_acc=True)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out)


@pytest.mark.parametrize("M", [3, 40])
@pytest.mark.parametrize("group", [256, 384, 1536])
def test_prepacked_wider_groups(P, M, group):
    """Several K steps share a scale (group = K is the coarse-grained GEMM, Table 2's first column)."""
    N, K = 80, 1536
    rng = np.random.default_rng(group + M)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    IS = rng.integers(0, 300, size=(N, K // group)).astype(np.int32)
    s = rng.random((N, K // group)).astype(np.float32) * 0.01
    sa = rng.random(M).astype(np.float32)
    qw = O.pack_int4(q)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, None, group, 8)
    out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), P.is_prepack_w4(dev(qw), dev(IS), group), None, 8,
                                                 want_acc=True)
    assert np.array_equal(host(acc), ref.acc)
    check_out(host(out), ref.out)
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, group)
    check_fs(host(P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), P.is_prepack_w4(dev(qw), dev(s), group))), fs)


def test_prepacked_split_k_workspace_reuse(P):
    """The arrival counters of the K split are left zero: one zeroed workspace serves call after call, of different
    shapes, and the results do not change from call to call."""
    shapes = [(64, 2064, 4096), (32, 528, 8192), (64, 48, 11008), (64, 2064, 4096)]
    need = max(P.is_gemm_prepacked_workspace_bytes(M, N, K, G) for M, N, K in shapes)
    assert need > 0
    ws = torch.zeros((need,), dtype=torch.uint8, device="cuda:0")
    for rep, (M, N, K) in enumerate(shapes):
        rng = np.random.default_rng(300 + M + N + K)
        xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
        ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
        pk = P.is_prepack_w4(dev(qw), dev(IS), G)
        for _ in range(2):
            out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10, want_acc=True, workspace=ws)
            assert np.array_equal(host(acc), ref.acc), f"call {rep}"
            check_out(host(out), ref.out)
        fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, G)
        pkf = P.is_prepack_w4(dev(qw), dev(s), G)
        a = P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), pkf, workspace=ws)
        b = P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), pkf, workspace=ws)
        check_fs(host(a), fs)
        assert torch.equal(a, b), "float-scale partials are added in a fixed order"
    torch.cuda.synchronize()
    assert int(ws[: 64 * 1024].view(torch.int32).abs().max()) == 0


LINEAR_PK_SHAPES = [(1, 4096, 4096), (1, 12288, 4096), (1, 4096, 11008), (1, 272, 12288), (1, 40, 1024), (1, 16, 128),
                    (1, 64, 28672), (1, 4360, 13312), (1, 48, 40960), (8, 4096, 4096), (64, 48, 11008), (33, 300, 1024)]


@pytest.mark.parametrize("M,N,K", LINEAR_PK_SHAPES)
def test_prepacked_linear_fp16_activations(P, M, N, K):
    rng = np.random.default_rng(7500 + M + N + K)
    _, qw, IS, s, _, c = rand_quantised(rng, 1, N, K)
    x = S.activations_outlier(M, K, 77 + K % 13)
    xq_ref, sa_ref = O.quantize_act_int8_token(x)
    ref = O.gemm_w4a8_intscale(xq_ref, sa_ref, qw, IS, c, G, 10)
    out, acc = P.is_linear_w4a8_intscale_prepacked(dev(x), P.is_prepack_w4(dev(qw), dev(IS), G), dev(c), 10,
                                                   want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")
    fs = O.gemm_w4a8_floatscale(xq_ref, sa_ref, qw, s, G)
    out_fs = P.is_linear_w4a8_floatscale_prepacked(dev(x), P.is_prepack_w4(dev(qw), dev(s), G))
    check_fs(host(out_fs), fs, f"M{M} N{N} K{K}")


def test_prepacked_linear_token_scale_and_zero_token(P):
    """The one-kernel route writes the token's scale where the two-kernel route does; an all-zero token gives scale 0
    and an all-zero output."""
    N, K = 512, 4096
    rng = np.random.default_rng(7100)
    _, qw, IS, s, _, c = rand_quantised(rng, 1, N, K)
    pk = P.is_prepack_w4(dev(qw), dev(IS), G)
    x = S.activations_student_t(1, K, 5)
    _, sa_ref = O.quantize_act_int8_token(x)
    ws = torch.zeros((P.is_linear_prepacked_workspace_bytes(1, N, K, G),), dtype=torch.uint8, device="cuda:0")
    P.is_linear_w4a8_intscale_prepacked(dev(x), pk, dev(c), 10, workspace=ws)
    off = (K + 255) // 256 * 256
    assert np.array_equal(host(ws[off:off + 4]).view(np.float32), sa_ref)
    out, acc = P.is_linear_w4a8_intscale_prepacked(dev(np.zeros((1, K), np.float16)), pk, dev(c), 10, want_acc=True)
    assert not host(acc).any() and not host(out).any()


# more than 64 token rows: the tiled kernel on the prepacked layout (ragged row and column tiles, one and many K steps,
# N not a multiple of 8: element-wise epilogue; several tiles per XCD)
TILE_PK_SHAPES = [(65, 256, 128), (129, 300, 1024), (256, 512, 2048), (300, 700, 1152), (513, 257, 512), (128, 256, 4096),
                  (1000, 1040, 256), (70, 16, 384)]


@pytest.mark.parametrize("M,N,K", TILE_PK_SHAPES)
def test_prepacked_tiled_gemm(P, M, N, K):
    rng = np.random.default_rng(3500 + M + N + K)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    xq[0], xq[1] = -128, 127                 # extreme codes on both sides
    q = O.unpack_int4(qw)
    q[0], q[1] = -8, 7
    qw = O.pack_int4(q)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
    pk = P.is_prepack_w4(dev(qw), dev(IS), G)
    out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")
    out1, _ = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10)   # the staged epilogue
    check_out(host(out1), ref.out, f"M{M} N{N} K{K} (no accumulator export)")
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, G)
    out_fs = P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), P.is_prepack_w4(dev(qw), dev(s), G))
    check_fs(host(out_fs), fs, f"M{M} N{N} K{K}")


@pytest.fixture
def tiled64(P):
    """Sends the prepacked calls of 33..64 rows to the tiled kernel whatever the size of the weights."""
    before = P.is_set_kernel_route("tiled64")
    yield
    P.is_set_kernel_route(before)


# 33..64 token rows on the tiled kernel's 64-row instance (the route large weight matrices take): ragged rows and
# columns, one and many K steps, a K range cut into parts (few tile columns), N not a multiple of 8
@pytest.mark.parametrize("M,N,K", [(33, 300, 1024), (64, 520, 2048), (48, 256, 128), (40, 1040, 4096), (64, 100, 11008),
                                   (57, 4104, 512)])
def test_prepacked_33_to_64_rows_on_the_tiled_kernel(P, tiled64, M, N, K):
    assert P.is_describe_prepacked(M, N, K, G)[-1] == "gemm_tile_pk_kernel<true>"
    rng = np.random.default_rng(3900 + M + N + K)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    xq[0], xq[M - 1] = -128, 127
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
    pk = P.is_prepack_w4(dev(qw), dev(IS), G)
    out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")
    out1, _ = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10)   # the staged epilogue
    check_out(host(out1), ref.out, f"M{M} N{N} K{K} (no accumulator export)")
    out_na = torch.empty((M, N), dtype=torch.float16, device="cuda:0")
    acc_na = torch.empty((M, N), dtype=torch.int32, device="cuda:0")
    P.is_gemm_w4a8_intscale_prepacked_noalloc(dev(xq), dev(sa), pk, dev(c), 10, out_na, acc_na)   # the fixed scratch
    assert np.array_equal(host(acc_na), ref.acc) and np.array_equal(host(out_na), host(out))
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, G)
    out_fs = P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), P.is_prepack_w4(dev(qw), dev(s), G))
    check_fs(host(out_fs), fs, f"M{M} N{N} K{K}")
    # the linear call on fp16 activations: stand-alone quantiser, then the same kernels
    x = S.activations_outlier(M, K, 31 + K % 7)
    xq_ref, sa_ref = O.quantize_act_int8_token(x)
    ref_l = O.gemm_w4a8_intscale(xq_ref, sa_ref, qw, IS, c, G, 10)
    out_l, acc_l = P.is_linear_w4a8_intscale_prepacked(dev(x), pk, dev(c), 10, want_acc=True)
    assert np.array_equal(host(acc_l), ref_l.acc), "linear call: int32 accumulators differ"
    check_out(host(out_l), ref_l.out, f"linear M{M} N{N} K{K}")


@pytest.mark.parametrize("M,K", [(130, 1024), (2048, 2048), (65, 128), (300, 4096)])
def test_prepacked_gemms_on_shared_prepared_activations(P, M, K):
    """One preparation of the activations, then GEMMs with several weight sets of different widths on the prepared
    workspace (last rounds with and without a K split, so the arrival counters are used and left zero in turn): the
    accumulators and outputs of the ordinary prepacked call, bit for bit, and the oracle's accumulators."""
    rng = np.random.default_rng(4100 + M + K)
    widths = [520, 16, 4104, 256, 520]
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    sa = (rng.random(M).astype(np.float32) + 0.1)
    ws = torch.empty(max(P.is_gemm_prepacked_workspace_bytes(M, n, K, G) for n in widths), dtype=torch.uint8, device="cuda:0")
    ws.random_(0, 256)
    P.is_prepare_activations_prepacked(dev(xq), ws)
    for i, N in enumerate(widths):
        _, qw, IS, s, _, c = rand_quantised(np.random.default_rng(4200 + N + i), 1, N, K)
        pk = P.is_prepack_w4(dev(qw), dev(IS), G)
        out, acc = P.is_gemm_w4a8_intscale_prepacked_prepared(dev(sa), pk, dev(c), 10, ws, want_acc=i % 2 == 0)
        ref_out, ref_acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10, want_acc=True)
        assert torch.equal(out, ref_out), f"N {N}"
        if acc is not None:
            assert torch.equal(acc, ref_acc), f"N {N}"
            assert np.array_equal(host(acc), O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10).acc)
        pf = P.is_prepack_w4(dev(qw), dev(s), G)
        assert torch.equal(P.is_gemm_w4a8_floatscale_prepacked_prepared(dev(sa), pf, ws),
                           P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), pf)), f"float scales, N {N}"


def test_prepacked_33_to_64_rows_random_shapes_match_the_canonical_call(P, tiled64):
    """Random shapes of 33..64 rows on the tiled kernel's 64-row instance (a wide scale now and then), each twice on a
    workspace of arbitrary contents, accumulators and fp16 outputs against the canonical call's, which the tests of
    test_gpu_parity.py and test_gpu_configs.py hold to the oracle."""
    rng = np.random.default_rng(20240598)
    for case in range(80):
        M = int(rng.integers(33, 65))
        N = int(rng.choice([16, 48, 200, 256, 264, 520, 1024, 2056, 4096]))
        K = int(rng.choice([128, 256, 1024, 2048, 4096, 11008, 14336]))
        q = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda:0")
        si = torch.randint(0, 1025, (N, K // G), dtype=torch.int32, device="cuda:0")
        if rng.random() < 0.3:
            si[0, 0] = 2 ** 25
        c = torch.rand((N,), device="cuda:0") + 0.5
        xq = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda:0")
        sa = torch.rand(M, device="cuda:0") + 0.1
        ref_out, ref = P.is_gemm_w4a8_intscale(xq, sa, q, si, c, G, 10, want_acc=True)
        pk = P.is_prepack_w4(q, si, G)
        ws = torch.empty(max(16, P.is_gemm_prepacked_workspace_bytes(M, N, K, G)), dtype=torch.uint8, device="cuda:0")
        for it in range(2):
            ws.random_(0, 256)
            out, acc = P.is_gemm_w4a8_intscale_prepacked(xq, sa, pk, c, 10, want_acc=it == 0, workspace=ws)
            if it == 0:
                assert torch.equal(acc, ref), f"case {case}: M {M}, N {N}, K {K}"
            assert torch.equal(out, ref_out), f"case {case}: M {M}, N {N}, K {K} (fp16 outputs, pass {it})"


@pytest.mark.parametrize("M,N,K", [(64, 8192, 28672), (40, 28672, 8192)])
def test_prepacked_33_to_64_rows_on_large_weights_take_the_tiled_kernel(P, M, N, K):
    """From 2^27 weights on the library itself picks the tiled kernel for 33..64 rows (the LLaMA-2-70B gate and down
    projections), and the weight-streaming kernel below (its qkv projection)."""
    assert P.is_describe_prepacked(M, N, K, G)[-1] == "gemm_tile_pk_kernel<true>"
    assert P.is_describe_prepacked(M, 10240, 8192, G)[-1].startswith("gemm_decode_pk_kernel<4, ")
    assert P.is_describe_prepacked(32, N, K, G)[-1].startswith("gemm_decode_pk_kernel<2, ")
    rng = np.random.default_rng(3950 + M)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
    pk = P.is_prepack_w4(dev(qw), dev(IS), G)
    out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")


@pytest.mark.parametrize("M,N,K,group", [(200, 300, 1024, 128), (129, 520, 2048, 256), (130, 80, 1536, 1536),
                                         (129, 300, 6144, 384)])
def test_prepacked_tiled_wide_scales_and_groups(P, M, N, K, group):
    """Scales beyond 24 bits (the 32-bit multiply instance, bit-exact modulo 2^32), groups of several K steps (the last:
    K parts of the last round's tiles that begin inside a group)."""
    rng = np.random.default_rng(77 + M)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sa = rng.random(M).astype(np.float32)
    qw = O.pack_int4(q)
    for IS in (rng.integers(-2 ** 31, 2 ** 31, size=(N, K // group), dtype=np.int64).astype(np.int32),
               np.where(rng.random((N, K // group)) < 0.05, 2 ** 24, 5).astype(np.int32),
               rng.integers(0, 1025, size=(N, K // group)).astype(np.int32)):
        ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, None, group, 10)
        out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), P.is_prepack_w4(dev(qw), dev(IS), group), None, 10,
                                                     want_acc=True)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out)


def test_prepacked_tiled_workspace_contents_do_not_matter(P):
    """The tiled route writes what it reads of its workspace (its preparation kernel also clears the arrival counters
    of the K split of the last round): a workspace full of ones, used twice, gives the same bits."""
    M, N, K = 300, 520, 4096
    assert P.is_gemm_prepacked_workspace_bytes(M, N, K, G) > (M + 15) // 16 * 16 * K + 2 ** 20   # partial tiles in it
    rng = np.random.default_rng(4100)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
    pk = P.is_prepack_w4(dev(qw), dev(IS), G)
    ws = torch.full((P.is_gemm_prepacked_workspace_bytes(M, N, K, G),), 0xFF, dtype=torch.uint8, device="cuda:0")
    for _ in range(2):
        out, acc = P.is_gemm_w4a8_intscale_prepacked(dev(xq), dev(sa), pk, dev(c), 10, want_acc=True, workspace=ws)
        assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
        check_out(host(out), ref.out)
    pkf = P.is_prepack_w4(dev(qw), dev(s), G)
    a = P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), pkf, workspace=ws)
    b = P.is_gemm_w4a8_floatscale_prepacked(dev(xq), dev(sa), pkf, workspace=ws)
    assert torch.equal(a, b)          # float partial sums are added in part order, whoever arrives last
    check_fs(host(a), O.gemm_w4a8_floatscale(xq, sa, qw, s, G))


@pytest.mark.parametrize("M,N,K", [(130, 512, 4096), (70, 272, 8192), (200, 256, 14336), (66, 128, 28672), (257, 40, 2048),
                                   (70, 48, 40960), (72, 32, 256), (89, 16, 128), (300, 48, 1152)])
def test_prepacked_tiled_linear_fp16(P, M, N, K):
    """More than 64 fp16 tokens: the tiled kernel's preparation quantises on the way (a workgroup per 8 token rows: row
    maxima, then the rounding into the kernel layout; rows longer than the registers hold are read twice).  Fewer K
    steps than waves, 8-row halves past M, an all-zero row."""
    rng = np.random.default_rng(7600 + M + N + K)
    _, qw, IS, s, _, c = rand_quantised(rng, 1, N, K)
    x = S.activations_student_t(M, K, 78 + K % 13)
    x[M // 2] = 0
    xq_ref, sa_ref = O.quantize_act_int8_token(x)
    ref = O.gemm_w4a8_intscale(xq_ref, sa_ref, qw, IS, c, G, 10)
    out, acc = P.is_linear_w4a8_intscale_prepacked(dev(x), P.is_prepack_w4(dev(qw), dev(IS), G), dev(c), 10,
                                                   want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")
    fs = O.gemm_w4a8_floatscale(xq_ref, sa_ref, qw, s, G)
    check_fs(host(P.is_linear_w4a8_floatscale_prepacked(dev(x), P.is_prepack_w4(dev(qw), dev(s), G))), fs)


# mixture-of-experts form on prepacked experts: experts without rows, with a few rows (padded to a 16-row tile), with
# several row tiles, with exactly one or two full tiles; ragged tile columns; a wide-scale expert among narrow ones.  The
# row counts cover the kernel's four instances per table entry (1..16, 17..32, 33..64, 65..128 rows), alone and with the
# K range cut into parts (K >= 2048 here).
@pytest.mark.parametrize("counts,N,K", [([5, 0, 17, 64, 1, 0, 33, 8], 48, 1024), ([0, 0, 3], 48, 512), ([130, 2], 48, 1024),
                                        ([0, 300, 0, 129, 70], 520, 1024), ([128, 128, 128], 256, 2048),
                                        ([0, 0, 0, 270], 48, 1024), ([257, 1, 1], 264, 4096), ([16, 15, 17, 1], 272, 128),
                                        ([400], 48, 1024), ([700, 500], 264, 512), ([0, 900], 48, 2048)])
def test_prepacked_grouped_gemm(P, counts, N, K):
    E = len(counts)
    rng = np.random.default_rng(sum(counts) + N)
    M = sum(counts)
    off = np.zeros(E + 1, np.int32)
    off[1:] = np.cumsum(counts)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    sa = (rng.random(M) + 0.01).astype(np.float32)
    q = np.stack([O.pack_int4(rng.integers(-8, 8, size=(N, K)).astype(np.int8)) for _ in range(E)])
    IS = rng.integers(0, 1025, size=(E, N, K // G)).astype(np.int32)
    IS[E - 1, 0, 0] = 2 ** 25                     # the last expert needs 32-bit multiplies, the others do not
    s = (rng.random((E, N, K // G)) * 0.01).astype(np.float32)
    c = (rng.random((E, N)) + 0.01).astype(np.float32)
    acc_ref, out_ref = O.gemm_w4a8_intscale_grouped(xq, sa, q, IS, c, off, G, 10)
    pk = P.is_prepack_w4_experts(dev(q), dev(IS), G)
    ws = torch.full((P.is_gemm_grouped_prepacked_workspace_bytes(E, M, N, K, G),), 0xFF, dtype=torch.uint8, device="cuda:0")
    for _ in range(2):                            # the workspace's contents do not matter
        out, acc = P.is_gemm_w4a8_intscale_grouped_prepacked(dev(xq), dev(sa), pk, dev(c), dev(off), 10, want_acc=True,
                                                             workspace=ws)
        assert np.array_equal(host(acc), acc_ref)
        assert np.array_equal(host(out), out_ref) or np.allclose(host(out).astype(np.float64), out_ref.astype(np.float64),
                                                                 rtol=2e-3, atol=2.0 ** -24)
    out2, _ = P.is_gemm_w4a8_intscale_grouped_prepacked(dev(xq), dev(sa), pk, dev(c), dev(off), 10)   # staged epilogue
    assert np.allclose(host(out2).astype(np.float64), out_ref.astype(np.float64), rtol=2e-3, atol=2.0 ** -24)
    fs_ref, fs_mag = O.gemm_w4a8_floatscale_grouped(xq, sa, q, s, off, G)
    fs = host(P.is_gemm_w4a8_floatscale_grouped_prepacked(dev(xq), dev(sa), P.is_prepack_w4_experts(dev(q), dev(s), G),
                                                          dev(off))).astype(np.float64)
    assert np.all(np.abs(fs - fs_ref) <= 1e-2 * np.abs(fs_ref) + 2e-5 * fs_mag + 2.0 ** -24)


def test_prepacked_grouped_random_shapes_match_the_canonical_call(P):
    """Many random expert row counts (all four row-count instances of the kernel, K ranges cut or not, a wide-scale expert now
    and then), each twice on a workspace of arbitrary contents: the accumulators of the prepacked grouped call against
    those of the canonical grouped call, which the tests above and test_gpu_configs.py hold to the oracle."""
    rng = np.random.default_rng(20240597)
    for case in range(120):
        E = int(rng.integers(1, 13))
        counts = rng.integers(0, [20, 70, 140, 300][int(rng.integers(0, 4))] + 1, size=E)
        if counts.sum() == 0:
            counts[0] = 5
        M = int(counts.sum())
        N = int(rng.choice([16, 48, 200, 256, 264, 520, 1024]))
        K = int(rng.choice([128, 256, 1024, 2048, 4096]))
        off = torch.tensor(np.concatenate([[0], np.cumsum(counts)]).astype(np.int32), device="cuda:0")
        q = torch.randint(0, 256, (E, N, K // 2), dtype=torch.uint8, device="cuda:0")
        si = torch.randint(0, 1025, (E, N, K // G), dtype=torch.int32, device="cuda:0")
        if rng.random() < 0.3:
            si[int(rng.integers(0, E)), 0, 0] = 2 ** 25
        xq = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda:0")
        sa = torch.rand(M, device="cuda:0") + 0.1
        _, ref = P.is_gemm_w4a8_intscale_grouped(xq, sa, q, si, None, off, G, 10, want_acc=True)
        pk = P.is_prepack_w4_experts(q, si, G)
        ws = torch.empty(max(16, P.is_gemm_grouped_prepacked_workspace_bytes(E, M, N, K, G)), dtype=torch.uint8, device="cuda:0")
        for _ in range(2):
            ws.random_(0, 256)
            _, acc = P.is_gemm_w4a8_intscale_grouped_prepacked(xq, sa, pk, None, off, 10, want_acc=True, workspace=ws)
            assert torch.equal(acc, ref), f"case {case}: rows per expert {counts.tolist()}, N {N}, K {K}"


def test_prepacked_grouped_empty(P):
    E, N, K = 3, 48, 256
    pk = P.is_prepack_w4_experts(torch.zeros((E, N, K // 2), dtype=torch.uint8, device="cuda:0"),
                                 torch.ones((E, N, K // G), dtype=torch.int32, device="cuda:0"), G)
    off = torch.zeros(E + 1, dtype=torch.int32, device="cuda:0")
    out, _ = P.is_gemm_w4a8_intscale_grouped_prepacked(torch.empty((0, K), dtype=torch.int8, device="cuda:0"),
                                                       torch.empty((0,), dtype=torch.float32, device="cuda:0"), pk, None,
                                                       off, 10)
    assert out.shape == (0, N)
    assert P.is_gemm_grouped_prepacked_workspace_bytes(E, 0, N, K, G) == 0


def test_prepacked_empty_and_unsupported(P):
    rng = np.random.default_rng(3)
    xq, qw, IS, s, sa, c = rand_quantised(rng, 1, 16, 128)
    pk = P.is_prepack_w4(dev(qw), dev(IS), G)
    e8 = torch.empty((0, 128), dtype=torch.int8, device="cuda:0")
    e32 = torch.empty((0,), dtype=torch.float32, device="cuda:0")
    out, _ = P.is_gemm_w4a8_intscale_prepacked(e8, e32, pk, None, 10)
    assert out.shape == (0, 16)
