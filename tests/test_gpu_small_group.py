"""GPU parity of the fine-grained W4A8 GEMM for groups of 32 and 64 weights (group-wise quantisation, App. A.2, with
Eq. (2) / Eq. (1) per group) through the C ABI against the CPU oracle: int32 accumulators bit for bit, fp16 outputs
within the stated tolerance; plain, grouped, linear (fp16 activations in) and overflow-safe calls; K that is not a
multiple of 128, ragged N and M, several token-row blocks, wide and negative scales, end to end from fp16 weights.
"""
import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O
from test_gpu_parity import check_fs, check_out, dev, host

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_14597_amd as pkg
    pkg.load_library()
    return pkg


def rand_quantised(rng, M, N, K, G, is_lo=0, is_hi=1025):
    xq = rng.integers(-128, 128, size=(M, K), dtype=np.int64).astype(np.int8)
    q = rng.integers(-8, 8, size=(N, K), dtype=np.int64).astype(np.int8)
    IS = rng.integers(is_lo, is_hi, size=(N, K // G), dtype=np.int64).astype(np.int32)
    s = (rng.random((N, K // G)) * 0.02 + 1e-4).astype(np.float32)
    sa = (rng.random(M) * 0.1 + 1e-3).astype(np.float32)
    c = (rng.random(N) * 0.05 + 1e-3).astype(np.float32)
    return xq, O.pack_int4(q), IS, s, sa, c


# one token; fewer groups than waves; K not a multiple of 128; ragged N; 17 rows (the four-tile instance with one
# tile in use); several token-row blocks with a ragged last one; a LLaMA-sized K
SHAPES = [(1, 16, 64), (1, 4096, 4096), (7, 100, 192), (16, 272, 1024), (17, 40, 320), (33, 48, 192), (64, 264, 2048),
          (130, 96, 512), (300, 72, 1088)]


@pytest.mark.parametrize("G", [32, 64])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_intscale_bit_exact_acc(P, G, M, N, K):
    rng = np.random.default_rng(100 + M + N + K + G)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K, G)
    ref = O.gemm_w4a8_intscale(xq, sa, qw, IS, c, G, 10)
    out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(qw), dev(IS), dev(c), G, 10, want_acc=True)
    assert np.array_equal(host(acc), ref.acc), "int32 accumulators differ"
    check_out(host(out), ref.out, f"M{M} N{N} K{K} G{G}")
    ref1 = O.gemm_w4a8_intscale(xq, sa, qw, IS, None, G, 7)
    out1, acc1 = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(qw), dev(IS), None, G, 7)
    assert acc1 is None
    check_out(host(out1), ref1.out)


@pytest.mark.parametrize("G", [32, 64])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_floatscale(P, G, M, N, K):
    rng = np.random.default_rng(200 + M + N + K + G)
    xq, qw, IS, s, sa, c = rand_quantised(rng, M, N, K, G)
    fs = O.gemm_w4a8_floatscale(xq, sa, qw, s, G)
    out = P.is_gemm_w4a8_floatscale(dev(xq), dev(sa), dev(qw), dev(s), G)
    check_fs(host(out), fs, f"M{M} N{N} K{K} G{G}")


@pytest.mark.parametrize("G", [32, 64])
def test_extreme_codes_and_wide_scales(P, G):
    """All codes at -128 / -8 (the largest partial sums), negative and wider-than-24-bit integer scales, wrap-around."""
    M, N, K = 20, 32, 2048
    xq = np.full((M, K), -128, np.int8)
    q = np.full((N, K), -8, np.int8)
    xq[1::2] = 127
    q[::3] = 7
    rng = np.random.default_rng(5 + G)
    sa = np.ones(M, np.float32)
    for IS in (np.full((N, K // G), 511, np.int32), np.full((N, K // G), 40000, np.int32),
               rng.integers(-2 ** 31, 2 ** 31, size=(N, K // G), dtype=np.int64).astype(np.int32)):
        ref = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, None, G, 10)
        out, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(O.pack_int4(q)), dev(IS), None, G, 10, want_acc=True)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out)


@pytest.mark.parametrize("G", [32, 64])
def test_groups_are_scaled_one_by_one(P, G):
    """A scale that is non-zero for a single group picks out that group's partial sum: every group of the row, in turn,
    against the oracle's group_partials (a group mixed with its neighbour, or indices dealt to the wrong group, fails)."""
    M, N, K = 5, 16, 4 * 128
    rng = np.random.default_rng(17 + G)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    qw = O.pack_int4(rng.integers(-8, 8, size=(N, K)).astype(np.int8))
    partials = O.group_partials(xq, qw, G)                      # [M, N, NG]
    sa = np.ones(M, np.float32)
    for g in range(K // G):
        IS = np.zeros((N, K // G), np.int32)
        IS[:, g] = 3
        _, acc = P.is_gemm_w4a8_intscale(dev(xq), dev(sa), dev(qw), dev(IS), None, G, 0, want_acc=True)
        assert np.array_equal(host(acc), 3 * partials[:, :, g]), f"group {g}"


@pytest.mark.parametrize("G", [32, 64])
@pytest.mark.parametrize("counts,N", [([5, 0, 17, 64, 1, 0, 33, 8], 48), ([0, 0, 3], 40), ([130, 2], 48), ([0, 300, 70], 24)])
def test_grouped_gemm(P, G, counts, N):
    E, K = len(counts), 512
    rng = np.random.default_rng(sum(counts) + G)
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
    assert np.allclose(host(out).astype(np.float64), out_ref.astype(np.float64), rtol=2e-3, atol=2.0 ** -24)
    fs_ref, fs_mag = O.gemm_w4a8_floatscale_grouped(xq, sa, q, s, off, G)
    fs = host(P.is_gemm_w4a8_floatscale_grouped(dev(xq), dev(sa), dev(q), dev(s), dev(off), G)).astype(np.float64)
    assert np.all(np.abs(fs - fs_ref) <= 1e-2 * np.abs(fs_ref) + 2e-5 * fs_mag + 2.0 ** -24)


@pytest.mark.parametrize("G", [32, 64])
@pytest.mark.parametrize("M,N,K", [(1, 272, 1024), (40, 64, 4096), (200, 48, 512)])
def test_linear_and_safe_form_end_to_end(P, G, M, N, K):
    """From fp16 weights and activations: the library's quantisers (bit-exact against the oracle's), the linear call,
    and the overflow-safe form, all at this group size."""
    w = S.make_weights(0, N, K, 31 + G + N)
    x = S.activations_outlier(M, K, 77 + K % 13)
    for mode in (O.SCALE_RAW, O.SCALE_NORM):
        rw = O.quantize_weights_int4_group(w, G, 10, mode)
        qw = P.is_quantize_weights_int4_group(dev(w), G, 10, mode)
        assert np.array_equal(host(qw.qweight), rw.qweight) and np.array_equal(host(qw.scale_i32), rw.scale_i32)
        assert np.array_equal(host(qw.scale_f32), rw.scale_f32) and np.array_equal(host(qw.chan_scale), rw.chan_scale)
        xq_ref, sa_ref = O.quantize_act_int8_token(x)
        ref = O.gemm_w4a8_intscale(xq_ref, sa_ref, rw.qweight, rw.scale_i32, rw.chan_scale, G, 10)
        out, acc = P.is_linear_w4a8_intscale(dev(x), qw.qweight, qw.scale_i32, qw.chan_scale, G, 10, want_acc=True)
        assert np.array_equal(host(acc), ref.acc)
        check_out(host(out), ref.out, f"M{M} N{N} K{K} G{G}")
        fs = O.gemm_w4a8_floatscale(xq_ref, sa_ref, rw.qweight, rw.scale_f32, G)
        check_fs(host(P.is_linear_w4a8_floatscale(dev(x), qw.qweight, qw.scale_f32, G)), fs)
        safe = O.gemm_w4a8_intscale_safe(xq_ref, sa_ref, rw.qweight, rw.scale_i32, rw.chan_scale, G, 10)
        got = host(P.is_gemm_w4a8_intscale_safe(dev(xq_ref), dev(sa_ref), qw.qweight, qw.scale_i32, qw.chan_scale, G,
                                               10)).astype(np.float64)
        assert np.all(np.abs(got - safe.out) <= 1e-2 * np.abs(safe.out) + 2e-5 * safe.abs_sum + 2.0 ** -24)


def test_other_group_sizes_are_refused(P):
    lib = P.load_library()
    A = 4096
    for G in (16, 96, 160):
        K = 3 * G * 4
        assert lib.is_gemm_w4a8_intscale(A, A, A, A, None, 8, 16, K, G, 10, A, None, None, 0, None) == P.IS_ERR_UNSUPPORTED
    # the kernel layout and W8A8 stay with multiples of 128
    assert lib.is_prepack_w4_scale_bytes(16, 256, 64) == 0
    assert lib.is_gemm_w8a8_intscale(A, A, A, A, None, 8, 16, 256, 64, 10, A, None, None, 0, None) == P.IS_ERR_UNSUPPORTED
