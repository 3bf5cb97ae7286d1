"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on the same seeded
inputs.  Integer results (codes, integer scales, int32 accumulators) must be bit-exact; fp16 outputs must satisfy
|gpu - ref| <= 1e-2 |ref| + 2^-24 (the tolerance the target states; the observed error is checked against the much
smaller bound that one fp16 rounding plus three fp32 roundings allow).
"""
import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O

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


@pytest.fixture(params=["auto", "general"])
def kernel(request, P):
    """Runs a test twice: with the library's own kernel choice, and with everything forced onto the general kernel."""
    before = P.is_set_kernel_route(request.param)
    yield request.param
    P.is_set_kernel_route(before)


@pytest.fixture
def route_setting(P):
    """A function that sets the library's routing override for the rest of the test."""
    before = P.is_set_kernel_route("auto")
    yield P.is_set_kernel_route
    P.is_set_kernel_route(before)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.detach().cpu().numpy()


def check_out(got16, ref64, what=""):
    got = got16.astype(np.float64)
    big = np.abs(ref64) > 65000.0      # at the edge of (or beyond) the fp16 range: same sign, saturated or inf
    if np.any(big):
        assert bool(np.all(np.sign(got[big]) == np.sign(ref64[big]))) and bool(np.all(np.abs(got[big]) > 64900.0)), what
    err = np.abs(got[~big] - ref64[~big])
    ref = np.abs(ref64[~big])
    ok = bool(np.all(err <= 1e-2 * ref + 2.0 ** -24))
    assert ok, f"{what}: fp16 output outside 1e-2 relative (max abs err {err.max()})"
    # derived bound: half an fp16 ulp (2^-11 relative, 2^-25 absolute in the subnormal range) plus fp32 slack
    ok = bool(np.all(err <= (2.0 ** -11 + 2.0 ** -20) * ref + 2.0 ** -24))
    assert ok, f"{what}: more than one fp16 rounding (max abs err {err.max()})"


def check_fs(got16, fs, what=""):
    got = got16.astype(np.float64)
    err = np.abs(got - fs.out)
    # fp32 accumulation over K/G terms in a different order than the oracle's double sum
    tol = 1e-2 * np.abs(fs.out) + 2e-5 * fs.abs_sum + 2.0 ** -24
    ok = bool(np.all(err <= tol))
    assert ok, f"{what}: float-scale output outside tolerance (max abs err {err.max()})"


def rand_quantised(rng, M, N, K, is_lo=0, is_hi=1025):
    xq = rng.integers(-128, 128, size=(M, K), dtype=np.int64).astype(np.int8)
    q = rng.integers(-8, 8, size=(N, K), dtype=np.int64).astype(np.int8)
    IS = rng.integers(is_lo, is_hi, size=(N, K // G), dtype=np.int64).astype(np.int32)
    s = (rng.random((N, K // G)) * 0.02 + 1e-4).astype(np.float32)
    sa = (rng.random(M) * 0.1 + 1e-3).astype(np.float32)
    c = (rng.random(N) * 0.05 + 1e-3).astype(np.float32)
    return xq, O.pack_int4(q), IS, s, sa, c


# ------------------------------------------------------------------------------------------------ quantisers
@pytest.mark.parametrize("M,K,kind", [(1, 4096, "outlier"), (8, 4096, "outlier"), (33, 11008, "outlier"),
                                      (64, 1024, "student"), (5, 8, "outlier"), (130, 28672, "student"),
                                      # few rows spread over 512 / 1024 lanes, many rows with 2 / 8 / 16 chunks per
                                      # lane, rows too long for registers
                                      (20, 8192, "outlier"), (300, 4096, "outlier"), (260, 11008, "student"),
                                      (257, 28672, "outlier"), (3, 40000, "outlier"), (300, 40000, "student")])
def test_act_quantizer_bit_exact(P, M, K, kind):
    x = S.activations_outlier(M, K, 11) if kind == "outlier" else S.activations_student_t(M, K, 12)
    if M > 2:
        x[1] = 0          # an all-zero token row
        x[2, 0] = 60000   # a large outlier
    xq_ref, sa_ref = O.quantize_act_int8_token(x)
    xq, sa = P.is_quantize_act_int8_token(dev(x))
    assert np.array_equal(host(xq), xq_ref)
    assert np.array_equal(host(sa), sa_ref)


def test_act_quantizer_empty(P):
    x = torch.empty((0, 4096), dtype=torch.float16, device="cuda:0")
    xq, sa = P.is_quantize_act_int8_token(x)
    assert xq.shape == (0, 4096) and sa.shape == (0,)


@pytest.mark.parametrize("N,K,group,alpha,mode", [
    (96, 1024, 128, 10, 0), (96, 1024, 128, 10, 1), (272, 4096, 128, 6, 0), (272, 4096, 128, 12, 1),
    (33, 2048, 32, 8, 1), (17, 512, 512, 10, 0), (64, 11008, 128, 10, 1), (40, 256, 2, 10, 0)])
def test_weight_quantizer_bit_exact(P, N, K, group, alpha, mode):
    w = S.weights_gaussian(N, K, 21, outlier_col_frac=0.005)
    w[3, : min(K, 2 * group)] = 0            # zero groups
    if N > 8:
        w[7] = 0                             # a zero row
    ref = O.quantize_weights_int4_group(w, group, alpha, mode)
    got = P.is_quantize_weights_int4_group(dev(w), group, alpha, mode)
    assert np.array_equal(host(got.qweight), ref.qweight)
    assert np.array_equal(host(got.scale_f32), ref.scale_f32)
    assert np.array_equal(host(got.scale_i32), ref.scale_i32)
    assert np.array_equal(host(got.chan_scale), ref.chan_scale)
    assert int(host(got.alpha_log2_dev)[0]) == alpha


@pytest.mark.parametrize("mode", [0, 1])
def test_weight_quantizer_amplifier_search(P, mode):
    w = S.weights_gaussian(128, 2048, 22)
    ref = O.quantize_weights_int4_group(w, G, -1, mode)
    got = P.is_quantize_weights_int4_group(dev(w), G, P.IS_ALPHA_HEURISTIC, mode)
    assert int(host(got.alpha_log2_dev)[0]) == ref.alpha_log2
    assert np.array_equal(host(got.scale_i32), ref.scale_i32)
    assert np.array_equal(host(got.qweight), ref.qweight)


# ------------------------------------------------------------------------------------------------ GEMM, oracle-quantised inputs
SHAPES = [(1, 16, 128), (1, 4096, 4096), (1, 4096, 14336), (1, 100, 20480), (1, 4200, 12416), (8, 4096, 4096), (16, 272, 1024), (17, 40, 1024), (33, 100, 2048),
          (64, 4096, 1024), (64, 48, 11008), (100, 33, 1536), (7, 1, 256), (48, 2064, 3584),
          (65, 256, 128), (129, 300, 1024), (256, 512, 2048), (300, 700, 1152), (513, 257, 512),
          # several 16-row tiles per workgroup in every decode variant (more than 256 tiles)
          (1, 8208, 4096), (16, 5008, 11008), (32, 4360, 8192), (24, 4120, 1024), (64, 8208, 4096), (40, 4200, 1024)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_intscale_bit_exact_acc(P, kernel, M, N, K):
    rng = np.random.default_rng(1000 + M + N + K)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
    out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(qw), dev(IS), dev(c), G, 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")
    # without a channel scale and without the accumulator export
    ref1 = O.gemm_w4a8_intscale(xq, sa, qw, IS, None, G, 7)
    out1, acc1 = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(qw), dev(IS), None, G, 7)
    assert acc1 is None
    check_out(host(out1), ref1.out)


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_floatscale(P, kernel, M, N, K):
    rng = np.random.default_rng(2000 + M + N + K)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, G)
    out = P.is_gemm_w4a8_floatscale(dev(xq), dev(sa), dev(qw), dev(s), G)
    check_fs(host(out), fs, f"M{M} N{N} K{K}")


def test_gemm_extreme_codes_and_wide_scales(P, kernel):
    """All codes at -128 / -8 (the largest partial sums), negative and wider-than-24-bit integer scales, wrap-around."""
    M, N, K = 16, 32, 4096
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
        out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(IS), None, G, 10, want_acc=True)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out)


@pytest.mark.parametrize("M,N,K", [(200, 300, 1024), (129, 520, 2048)])
def test_tiled_kernel_wide_scales(P, M, N, K):
    """More than 64 token rows with integer scales beyond 24 bits (and extreme codes): the tiled kernel's 32-bit
    multiply instance, bit-exact modulo 2^32."""
    rng = np.random.default_rng(77 + M)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    xq[0], xq[1], q[0], q[1] = -128, 127, -8, 7
    sa = rng.random(M).astype(np.float32)
    for IS in (rng.integers(-2 ** 31, 2 ** 31, size=(N, K // G), dtype=np.int64).astype(np.int32),
               np.where(rng.random((N, K // G)) < 0.01, 2 ** 24, 5).astype(np.int32)):
        ref = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, None, G, 10)
        out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(IS), None, G, 10, want_acc=True)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out)


@pytest.mark.parametrize("group", [256, 512, 1024])
def test_gemm_wider_groups_and_coarse_grained(P, kernel, group):
    """group = K is the coarse-grained GEMM (Table 2, first column)."""
    M, N, K = 24, 80, 1024
    rng = np.random.default_rng(group)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    IS = rng.integers(0, 300, size=(N, K // group)).astype(np.int32)
    s = rng.random((N, K // group)).astype(np.float32) * 0.01
    sa = rng.random(M).astype(np.float32)
    ref = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, None, group, 8)
    out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(IS), None, group, 8, want_acc=True)
    assert np.array_equal(host(acc), ref.acc)
    check_out(host(out), ref.out)
    fs = O.gemm_w4a8_floatscale(xq, sa, O.pack_int4(q), s, group)
    check_fs(host(P.is_gemm_w4a8_floatscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(s), group)), fs)


@pytest.mark.parametrize("M,N,K", [(200, 300, 1024), (130, 80, 2048), (65, 264, 256), (513, 257, 1152)])
def test_coarse_grained_tiled_kernel(P, M, N, K):
    """group = K with more than 64 token rows: the tiled kernel's coarse-grained instance (partial products carried by
    the MFMA accumulators across all K steps, one scale per weight row in the epilogue), including extreme codes and
    scales that wrap the 32-bit result."""
    rng = np.random.default_rng(K + M)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    xq[0], xq[1], q[0], q[1] = -128, 127, -8, 7
    sa = rng.random(M).astype(np.float32)
    c = (rng.random(N) + 0.01).astype(np.float32)
    s = rng.random((N, 1)).astype(np.float32) * 0.01
    for IS in (rng.integers(0, 1025, size=(N, 1)).astype(np.int32),
               rng.integers(-2 ** 31, 2 ** 31, size=(N, 1), dtype=np.int64).astype(np.int32)):
        ref = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, c, K, 9)
        out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(IS), dev(c), K, 9, want_acc=True)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out)
        out2, _ = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(IS), dev(c), K, 9)
        check_out(host(out2), ref.out)
    fs = O.gemm_w4a8_floatscale(xq, sa, O.pack_int4(q), s, K)
    check_fs(host(P.is_gemm_w4a8_floatscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(s), K)), fs)


def test_group_sums_beyond_24_bits(P, kernel):
    """One group of 8192 int4 weights with the extreme codes: the partial sum is 2^23, one more than the signed 24-bit
    multiplier holds, so the scale step must take the 32-bit multiply whatever the scale."""
    M, N, K = 2, 16, 8192
    xq = np.full((M, K), -128, np.int8)
    q = np.full((N, K), -8, np.int8)
    IS = np.full((N, 1), 3, np.int32)
    sa = np.ones(M, np.float32)
    ref = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, None, K, 10)
    assert int(ref.acc64[0, 0]) == 3 * 2 ** 23
    out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(IS), None, K, 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc)
    check_out(host(out), ref.out)


def test_gemm_empty_batch(P):
    rng = np.random.default_rng(3)
    xq, qw, IS, s, sa, c = rand_quantised(rng, 1, 16, 128)
    e8 = torch.empty((0, 128), dtype=torch.int8, device="cuda:0")
    e32 = torch.empty((0,), dtype=torch.float32, device="cuda:0")
    out, _ = P.is_gemm_w4a8_intscale(e8, e32, dev(qw), dev(IS), None, G, 10)
    assert out.shape == (0, 16)


def test_gemm_repeatable(P):
    rng = np.random.default_rng(4)
    xq, qw, IS, s, sa, c = rand_quantised(rng, 32, 4096, 4096)
    args = (dev(xq), dev(sa), dev(qw), dev(IS), dev(c), G, 10)
    out0, acc0 = P.is_gemm_w4a8_intscale(*args, want_acc=True)
    fs0 = P.is_gemm_w4a8_floatscale(args[0], args[1], args[2], dev(s), G)
    for _ in range(3):
        out1, acc1 = P.is_gemm_w4a8_intscale(*args, want_acc=True)
        fs1 = P.is_gemm_w4a8_floatscale(args[0], args[1], args[2], dev(s), G)
        assert torch.equal(acc0, acc1) and torch.equal(out0, out1) and torch.equal(fs0, fs1)


# ------------------------------------------------------------------------------------------------ linear on fp16 activations
# one token through the decode kernel's three one-tile instances (K slices of 2, 4 and 6 steps, even and uneven
# splits of the groups over the waves, fewer tiles than workgroups, many tiles per workgroup), one token with K
# beyond the decode kernel, and several tokens (quantiser kernel + GEMM)
LINEAR_SHAPES = [(1, 4096, 4096), (1, 12288, 4096), (1, 4096, 8192), (1, 4096, 11008), (1, 272, 12288), (1, 40, 1024),
                 (1, 16, 128), (1, 8208, 2048), (1, 64, 28672), (8, 4096, 4096), (100, 300, 1024), (64, 48, 11008),
                 # one token, K slices of 7 to 10 steps per wave: the operands stay in LDS
                 (1, 4096, 14336), (1, 272, 20480), (1, 4360, 13312),
                 # more than 64 tokens: the tiled kernel's preparation quantises on the way (a wave per row; a workgroup
                 # per row with 4 and 8 chunks per lane; a ragged last row tile), and rows too long for that (quantiser
                 # kernel first)
                 (130, 512, 4096), (70, 272, 8192), (200, 256, 14336), (66, 128, 28672), (257, 40, 2048),
                 (70, 48, 40960)]


@pytest.mark.parametrize("M,N,K", LINEAR_SHAPES)
def test_linear_fp16_activations(P, kernel, M, N, K):
    rng = np.random.default_rng(7000 + M + N + K)
    _, qw, IS, s, _, c = rand_quantised(rng, 1, N, K)
    x = S.activations_outlier(M, K, 77 + K % 13)
    xq_ref, sa_ref = O.quantize_act_int8_token(x)
    ref = O.gemm_w4a8_intscale(xq_ref, sa_ref, qw, IS, c, G, 10)
    out, acc = P.is_linear_w4a8_intscale(dev(x), dev(qw), dev(IS), dev(c), G, 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K}")
    fs = O.gemm_w4a8_floatscale(xq_ref, sa_ref, qw, s, G)
    out_fs = P.is_linear_w4a8_floatscale(dev(x), dev(qw), dev(s), G)
    check_fs(host(out_fs), fs, f"M{M} N{N} K{K}")


@pytest.mark.parametrize("M", [1, 100])
@pytest.mark.parametrize("group", [256, 1024, 4096])
def test_linear_fp16_wider_groups(P, kernel, M, group):
    """Groups wider than a K step (several steps share a scale; group = K is the coarse-grained GEMM) and scales that
    need 32-bit multiplies, through both one-call routes that quantise inside the GEMM."""
    N, K = 272, 4096
    rng = np.random.default_rng(7300 + group + M)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    qw = O.pack_int4(q)
    c = (rng.random(N) * 0.05 + 1e-3).astype(np.float32)
    x = S.activations_student_t(M, K, 7300 + M)
    xq_ref, sa_ref = O.quantize_act_int8_token(x)
    for IS in (rng.integers(0, 1025, size=(N, K // group)).astype(np.int32),
               rng.integers(-2 ** 31, 2 ** 31, size=(N, K // group), dtype=np.int64).astype(np.int32)):
        ref = O.gemm_w4a8_intscale(xq_ref, sa_ref, qw, IS, c, group, 10)
        out, acc = P.is_linear_w4a8_intscale(dev(x), dev(qw), dev(IS), dev(c), group, 10, want_acc=True)
        assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
        check_out(host(out), ref.out, f"M{M} group {group}")


def test_linear_fp16_token_scale_and_zero_token(P):
    """The one-kernel route leaves the token's scale where the two-kernel route does, and an all-zero token gives
    scale 0 and an all-zero output."""
    N, K = 512, 4096
    rng = np.random.default_rng(7100)
    _, qw, IS, s, _, c = rand_quantised(rng, 1, N, K)
    x = S.activations_student_t(1, K, 5)
    _, sa_ref = O.quantize_act_int8_token(x)
    nbytes = P.is_linear_workspace_bytes(1, N, K, G)
    assert nbytes >= K + 256
    ws = torch.zeros((nbytes,), dtype=torch.uint8, device="cuda:0")
    P.is_linear_w4a8_intscale(dev(x), dev(qw), dev(IS), dev(c), G, 10, workspace=ws)
    sa = ws[K:K + 4].view(torch.float32)          # K = 4096 is already a multiple of 256
    assert np.array_equal(host(sa), sa_ref)
    out, acc = P.is_linear_w4a8_intscale(dev(np.zeros((1, K), np.float16)), dev(qw), dev(IS), dev(c), G, 10,
                                         want_acc=True, workspace=ws)
    assert not host(acc).any() and not host(out).any()
    assert host(ws[K:K + 4].view(torch.float32))[0] == 0.0


def test_linear_fp16_argument_checks(P):
    N, K = 64, 1024
    rng = np.random.default_rng(7200)
    _, qw, IS, s, _, c = rand_quantised(rng, 1, N, K)
    x = dev(S.activations_outlier(2, K, 3))
    small = torch.empty((16,), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(P.IntScaleError):
        P.is_linear_w4a8_intscale(x, dev(qw), dev(IS), dev(c), G, 10, workspace=small)
    out, _ = P.is_linear_w4a8_intscale(x[:0], dev(qw), dev(IS), dev(c), G, 10)
    assert out.shape == (0, N)


# ------------------------------------------------------------------------------------------------ seeded random shapes
def _random_shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        M = int(rng.choice([1, 1, 2, 7, 16, 17, 32, 33, 48, 64, 65, 100, 130]))
        N = int(rng.integers(1, 700))
        steps = int(rng.integers(1, 161 if M == 1 else 100))      # K up to 20480 for one token, 12672 otherwise
        spg = int(rng.choice([1, 1, 1, 2, 4]))                    # 128-wide steps per group
        K = 128 * spg * max(1, steps // spg)
        out.append((M, N, K, 128 * spg))
    return out


@pytest.mark.parametrize("M,N,K,group", _random_shapes(20240514, 48))
def test_random_shapes_both_entry_points(P, M, N, K, group):
    """Kernel choice, K split over the waves, ragged tiles: the GEMM on quantised activations and the linear call on
    the fp16 ones against the oracle, on shapes drawn from a fixed seed."""
    rng = np.random.default_rng(M * 1000003 + N * 1009 + K + group)
    q = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    qw = O.pack_int4(q)
    IS = rng.integers(0, 1025, size=(N, K // group)).astype(np.int32)
    s = (rng.random((N, K // group)) * 0.02 + 1e-4).astype(np.float32)
    c = (rng.random(N) * 0.05 + 1e-3).astype(np.float32)
    x = S.activations_outlier(M, K, int(rng.integers(1, 1 << 30)))
    xq, sa = O.quantize_act_int8_token(x)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, group, 10)
    out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(qw), dev(IS), dev(c), group, 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K} G{group}")
    out2, acc2 = P.is_linear_w4a8_intscale(dev(x), dev(qw), dev(IS), dev(c), group, 10, want_acc=True)
    assert np.array_equal(host(acc2), ref.acc), "int32 accumulators of the linear call differ"
    check_out(host(out2), ref.out, f"linear M{M} N{N} K{K} G{group}")
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, group)
    check_fs(host(P.is_linear_w4a8_floatscale(dev(x), dev(qw), dev(s), group)), fs, f"M{M} N{N} K{K} G{group}")


# ------------------------------------------------------------------------------------------------ fine-grained W8A8
@pytest.mark.parametrize("N,K,group,alpha,mode", [(16, 128, 128, 10, 0), (300, 1024, 128, 10, 1), (64, 2048, 256, -1, 1),
                                                  (33, 512, 512, -1, 0)])
def test_w8_weight_quantizer_bit_exact(P, N, K, group, alpha, mode):
    w = S.weights_gaussian(N, K, 31 + N)
    w[N // 2, :group] = 0
    ref = O.quantize_weights_int8_group(w, group, alpha, mode)
    got = P.is_quantize_weights_int8_group(dev(w), group, alpha, mode)
    assert np.array_equal(host(got.qweight), ref.qweight)
    assert np.array_equal(host(got.scale_f32), ref.scale_f32)
    assert np.array_equal(host(got.scale_i32), ref.scale_i32)
    assert np.array_equal(host(got.chan_scale), ref.chan_scale)
    assert int(host(got.alpha_log2_dev)[0]) == ref.alpha_log2


@pytest.mark.parametrize("M,N,K,group", [(1, 16, 128, 128), (8, 512, 1024, 128), (16, 272, 1024, 128), (64, 48, 2048, 128),
                                         (65, 256, 128, 128), (129, 300, 1024, 128), (300, 700, 1152, 128),
                                         (200, 264, 1024, 256), (130, 80, 512, 512), (513, 257, 512, 128),
                                         (1, 4096, 14336, 128), (24, 1040, 2048, 256), (33, 100, 1024, 1024),
                                         (48, 2064, 3584, 128)])
@pytest.mark.parametrize("route", ["auto", "tiled"])
def test_w8a8_gemm(P, route_setting, route, M, N, K, group):
    """Up to 64 token rows the library takes the general (bandwidth-bound) kernel, above that the tiled one; "tiled"
    sends every shape to the tiled kernel."""
    route_setting(route)
    rng = np.random.default_rng(4000 + M + N + K)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-128, 128, size=(N, K)).astype(np.int8)
    xq[0], q[0] = -128, -128  # the largest partial sums
    if M > 1:
        xq[1] = 127
    sa = (rng.random(M) + 0.01).astype(np.float32)
    c = (rng.random(N) + 0.01).astype(np.float32)
    s = (rng.random((N, K // group)) * 1e-4).astype(np.float32)  # keeps the extreme rows inside the fp16 range
    for IS, chan, a in ((rng.integers(0, 1025, size=(N, K // group)).astype(np.int32), c, 10),
                        (rng.integers(-2 ** 31, 2 ** 31, size=(N, K // group), dtype=np.int64).astype(np.int32), None, 7)):
        ref = O.gemm_w8a8_intscale(xq, sa, q, IS, chan, group, a)
        out, acc = P.is_gemm_w8a8_intscale(dev(xq), dev(sa), dev(q), dev(IS), None if chan is None else dev(chan), group, a,
                                           want_acc=True)
        assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
        check_out(host(out), ref.out, f"M{M} N{N} K{K}")
        out1, _ = P.is_gemm_w8a8_intscale(dev(xq), dev(sa), dev(q), dev(IS), None if chan is None else dev(chan), group, a)
        check_out(host(out1), ref.out)
    fs = O.gemm_w8a8_floatscale(xq, sa, q, s, group)
    check_fs(host(P.is_gemm_w8a8_floatscale(dev(xq), dev(sa), dev(q), dev(s), group)), fs, f"M{M} N{N} K{K}")


# ------------------------------------------------------------------------------------------------ overflow handling
@pytest.mark.parametrize("N,K,group", [(16, 128, 128), (300, 4096, 128), (4096, 11008, 128), (40, 1024, 512)])
def test_overflow_bound(P, N, K, group):
    rng = np.random.default_rng(N + K)
    for IS in (rng.integers(0, 1025, size=(N, K // group)).astype(np.int32),
               rng.integers(-2 ** 31, 2 ** 31, size=(N, K // group), dtype=np.int64).astype(np.int32),
               np.zeros((N, K // group), np.int32)):
        got = int(host(P.is_intscale_overflow_bound(dev(IS), group))[0])
        assert got == O.layer_overflow_bound(IS, group)


@pytest.mark.parametrize("M,N,K", [(1, 4096, 4096), (16, 272, 1024), (64, 48, 11008), (48, 2064, 3584), (129, 300, 1024),
                                   (300, 700, 1152)])
def test_gemm_intscale_safe(P, kernel, M, N, K):
    """The overflow-safe form against the oracle's exact sum: with ordinary scales, and with scales that wrap the
    32-bit accumulator of Eq. (2) (where the safe form must keep the true value)."""
    rng = np.random.default_rng(3000 + M + N + K)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K)
    big = rng.integers(-2 ** 20, 2 ** 20, size=IS.shape, dtype=np.int64).astype(np.int32)
    for scales, chan, a in ((IS, c, 10), (big, None, 12), (big, c, 0)):
        ref = O.gemm_w4a8_intscale_safe(xq, sa, qw, scales, chan, G, a)
        out = host(P.is_gemm_w4a8_intscale_safe(dev(xq), dev(sa), dev(qw), dev(scales), None if chan is None else dev(chan),
                                               G, a)).astype(np.float64)
        fin = np.abs(ref.out) < 60000.0
        err = np.abs(out[fin] - ref.out[fin])
        assert np.all(err <= 1e-2 * np.abs(ref.out[fin]) + 2e-5 * ref.abs_sum[fin] + 2.0 ** -24), f"M{M} N{N} K{K} a{a}"
        assert np.all(np.sign(out[~fin]) == np.sign(ref.out[~fin]))
    wrapped = O.gemm_w4a8_intscale(xq, sa, qw, big, None, G, 12)
    assert np.any(wrapped.acc.astype(np.int64) != wrapped.acc64), "the big scales are meant to wrap Eq. (2)'s accumulator"


# ------------------------------------------------------------------------------------------------ grouped (mixture of experts)
# (the first two go to the general kernel; from 65 rows per expert on average the tiled kernel takes over, with its table
# of existing row tiles: experts without rows, with several tiles, with exactly one full tile, ragged tile columns)
@pytest.mark.parametrize("counts,N", [([5, 0, 17, 64, 1, 0, 33, 8], 48), ([0, 0, 3], 48), ([130, 2], 48),
                                      ([0, 300, 0, 129, 70], 520), ([128, 128, 128], 256), ([0, 0, 0, 270], 48),
                                      ([257, 1, 1], 264)])
def test_grouped_gemm(P, counts, N):
    E, K = len(counts), 1024
    rng = np.random.default_rng(sum(counts))
    M = sum(counts)
    off = np.zeros(E + 1, np.int32)
    off[1:] = np.cumsum(counts)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    sa = (rng.random(M) + 0.01).astype(np.float32)
    q = np.stack([O.pack_int4(rng.integers(-8, 8, size=(N, K)).astype(np.int8)) for _ in range(E)])
    IS = rng.integers(0, 1025, size=(E, N, K // G)).astype(np.int32)
    s = (rng.random((E, N, K // G)) * 0.01).astype(np.float32)
    c = (rng.random((E, N)) + 0.01).astype(np.float32)
    acc_ref, out_ref = O.gemm_w4a8_intscale_grouped(xq, sa, q, IS, c, off, G, 10)
    out, acc = P.is_gemm_w4a8_intscale_grouped(dev(xq), dev(sa), dev(q), dev(IS), dev(c), dev(off), G, 10, want_acc=True)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(host(out), out_ref) or np.allclose(host(out).astype(np.float64), out_ref.astype(np.float64),
                                                             rtol=2e-3, atol=2.0 ** -24)
    fs_ref, fs_mag = O.gemm_w4a8_floatscale_grouped(xq, sa, q, s, off, G)
    fs = host(P.is_gemm_w4a8_floatscale_grouped(dev(xq), dev(sa), dev(q), dev(s), dev(off), G)).astype(np.float64)
    assert np.all(np.abs(fs - fs_ref) <= 1e-2 * np.abs(fs_ref) + 2e-5 * fs_mag + 2.0 ** -24)


# ------------------------------------------------------------------------------------------------ end to end, GPU-quantised
def test_config0_end_to_end(P, kernel):
    """M=8, K=N=4096, group 128, alpha 2^10: fp16 in, fp16 out, every stage compared."""
    sh = S.config_shapes(0)[0]
    x = S.make_activations(0, sh.M, sh.K, S.seed_for(0, 0, 0))
    w = S.make_weights(0, sh.N, sh.K, S.seed_for(0, 0, 1))
    for mode in (O.SCALE_RAW, O.SCALE_NORM):
        xq_r, sa_r = O.quantize_act_int8_token(x)
        qw_r = O.quantize_weights_int4_group(w, G, 10, mode)
        ref = O.gemm_w4a8_intscale(xq_r, sa_r, qw_r.qweight, qw_r.scale_i32, qw_r.chan_scale, G, 10)
        fs_r = O.gemm_w4a8_floatscale(xq_r, sa_r, qw_r.qweight, qw_r.scale_f32, G)
        xq, sa = P.is_quantize_act_int8_token(dev(x))
        qw = P.is_quantize_weights_int4_group(dev(w), G, 10, mode)
        out, acc = P.is_gemm_w4a8_intscale(xq, sa, qw.qweight, qw.scale_i32, qw.chan_scale, G, 10, want_acc=True)
        fs = P.is_gemm_w4a8_floatscale(xq, sa, qw.qweight, qw.scale_f32, G)
        assert np.array_equal(host(xq), xq_r) and np.array_equal(host(sa), sa_r)
        assert np.array_equal(host(qw.qweight), qw_r.qweight) and np.array_equal(host(qw.scale_i32), qw_r.scale_i32)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out)
        check_fs(host(fs), fs_r)
        assert ref.max_prefix.max() < 2 ** 31
