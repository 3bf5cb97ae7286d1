"""Pins for the oracle's GEMMs (Eq. (1), Eq. (2), Table 2).

Independent formulations only: python-integer brute force, numpy de-quantise-then-multiply, the plain integer
matmul special case, algebraic invariants, the exact error bound between Eq. (1) and Eq. (2), and the 32-bit
overflow bound.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as O
import synth_inputs as S


def _rand_problem(rng, M, N, K, G, is_hi=300, full_range=True):
    lo_x, lo_q = (-128, -8) if full_range else (-127, -7)
    xq = rng.integers(lo_x, 128, size=(M, K), dtype=np.int64).astype(np.int8)
    q = rng.integers(lo_q, 8, size=(N, K), dtype=np.int64).astype(np.int8)
    IS = rng.integers(0, is_hi, size=(N, K // G), dtype=np.int64).astype(np.int32)
    s = (rng.random((N, K // G)) * 0.2).astype(np.float32)
    sa = (rng.random(M) * 0.1 + 0.01).astype(np.float32)
    c = (rng.random(N) * 0.5 + 0.01).astype(np.float32)
    return xq, q, IS, s, sa, c


@pytest.mark.parametrize("M,N,K,G", [(1, 1, 2, 2), (3, 5, 16, 4), (4, 6, 16, 8), (2, 3, 12, 2), (2, 2, 16, 16)])
def test_brute_force_python_integers(M, N, K, G):
    rng = np.random.default_rng(100 + K + G)
    xq, q, IS, s, sa, c = _rand_problem(rng, M, N, K, G)
    a = 7
    r = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, c, G, a)
    f = O.gemm_w4a8_floatscale(xq, sa, O.pack_int4(q), s, G)
    for m in range(M):
        for n in range(N):
            acc = 0
            fs = Fraction(0)
            for g in range(K // G):
                p = sum(int(xq[m, k]) * int(q[n, k]) for k in range(g * G, (g + 1) * G))
                acc += p * int(IS[n, g])
                fs += Fraction(p) * Fraction(float(s[n, g]))
            assert int(r.acc[m, n]) == acc and int(r.acc64[m, n]) == acc
            exact = Fraction(acc) * Fraction(float(sa[m])) * Fraction(float(c[n])) / (2 ** a)
            assert r.out[m, n] == pytest.approx(float(exact), rel=1e-14, abs=0)
            assert f.out[m, n] == pytest.approx(float(Fraction(float(sa[m])) * fs), rel=1e-13, abs=1e-300)


def test_dequantise_then_multiply_formulation():
    """Eq. (2) equals an ordinary matmul against weights de-quantised with the integer scales."""
    rng = np.random.default_rng(7)
    M, N, K, G, a = 9, 40, 512, 128, 10
    xq, q, IS, s, sa, c = _rand_problem(rng, M, N, K, G)
    r = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, c, G, a)
    w_int = q.astype(np.int64) * np.repeat(IS.astype(np.int64), G, axis=1)
    acc = xq.astype(np.int64) @ w_int.T
    assert np.array_equal(r.acc64, acc) and np.array_equal(r.acc.astype(np.int64), acc)
    ref = acc.astype(np.float64) * sa.astype(np.float64)[:, None] * c.astype(np.float64)[None, :] / 2 ** a
    assert np.allclose(r.out, ref, rtol=1e-14, atol=0)
    f = O.gemm_w4a8_floatscale(xq, sa, O.pack_int4(q), s, G)
    w_f = q.astype(np.float64) * np.repeat(s.astype(np.float64), G, axis=1)
    ref_f = (xq.astype(np.float64) @ w_f.T) * sa.astype(np.float64)[:, None]
    assert np.allclose(f.out, ref_f, rtol=1e-11, atol=1e-12)
    p = O.group_partials(xq, O.pack_int4(q), G)
    assert np.array_equal(p.astype(np.int64).sum(axis=2), xq.astype(np.int64) @ q.astype(np.int64).T)


def test_single_group_unit_scale_is_plain_integer_matmul():
    """Table 2, first column: with one group spanning K and scale 1 the recurrence is an ordinary integer GEMM."""
    rng = np.random.default_rng(8)
    M, N, K = 5, 33, 256
    xq, q, _, _, sa, _ = _rand_problem(rng, M, N, K, K)
    ones = np.ones((N, 1), dtype=np.int32)
    r = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), ones, None, K, 0)
    assert np.array_equal(r.acc.astype(np.int64), xq.astype(np.int64) @ q.astype(np.int64).T)
    # not symmetric in its operands: a transposed-operand mistake cannot pass
    assert not np.array_equal(r.acc[:, :M], r.acc[:, :M].T)


def test_algebraic_invariants():
    rng = np.random.default_rng(9)
    M, N, K, G, a = 4, 24, 1024, 128, 10
    xq, q, IS, s, sa, c = _rand_problem(rng, M, N, K, G)
    base = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, c, G, a)
    # doubling every integer scale doubles the accumulator; doubling alpha as well leaves the output alone
    dbl = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), 2 * IS, c, G, a + 1)
    assert np.array_equal(dbl.acc64, 2 * base.acc64)
    assert np.array_equal(dbl.out, base.out)
    # permuting whole groups (of x, w and the scales together) does not change the sum
    perm = rng.permutation(K // G)
    kperm = (perm[:, None] * G + np.arange(G)[None, :]).reshape(-1)
    pr = O.gemm_w4a8_intscale(xq[:, kperm], sa, O.pack_int4(q[:, kperm]), IS[:, perm], c, G, a)
    assert np.array_equal(pr.acc, base.acc)
    # negating the activations negates the accumulator; row/column scales act only in the epilogue
    neg = O.gemm_w4a8_intscale((-xq.astype(np.int16)).clip(-127, 127).astype(np.int8), sa, O.pack_int4(q), IS, c, G, a)
    mask = (xq != -128).all(axis=1)
    assert np.array_equal(neg.acc64[mask], -base.acc64[mask])
    sc = O.gemm_w4a8_intscale(xq, 2 * sa, O.pack_int4(q), IS, None, G, a)
    assert np.array_equal(sc.acc, base.acc)
    assert np.allclose(sc.out * c.astype(np.float64)[None, :], 2 * base.out, rtol=1e-15)
    # a zero integer scale removes its group from the sum
    IS0 = IS.copy()
    IS0[:, 3] = 0
    p = O.group_partials(xq, O.pack_int4(q), G).astype(np.int64)
    z = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS0, c, G, a)
    assert np.array_equal(z.acc64, base.acc64 - p[:, :, 3] * IS[:, 3].astype(np.int64)[None, :])


def _quantised_layer(M, N, K, seed, a, mode):
    x = S.activations_outlier(M, K, seed)
    w = S.weights_gaussian(N, K, seed + 1)
    xq, sa = O.quantize_act_int8_token(x)
    qw = O.quantize_weights_int4_group(w, 128, a, mode)
    return x, w, xq, sa, qw


@pytest.mark.parametrize("mode", [O.SCALE_RAW, O.SCALE_NORM])
def test_integer_scale_converges_to_float_scale(mode):
    """Eq. (2) -> Eq. (1) as alpha grows: exact bound |O_IS - O_FS| <= s_a c sum_g |P_g| / (2 alpha), error ~ 1/alpha."""
    M, N, K = 8, 64, 2048
    errs, fine = [], []
    for a in (6, 8, 10, 12, 14):
        _, _, xq, sa, qw = _quantised_layer(M, N, K, 31, a, mode)
        isr = O.gemm_w4a8_intscale(xq, sa, qw.qweight, qw.scale_i32, qw.chan_scale, 128, a)
        fsr = O.gemm_w4a8_floatscale(xq, sa, qw.qweight, qw.scale_f32, 128)
        assert np.all(isr.max_prefix < 2 ** 31)
        p = np.abs(O.group_partials(xq, qw.qweight, 128).astype(np.float64)).sum(axis=2)
        bound = sa.astype(np.float64)[:, None] * qw.chan_scale.astype(np.float64)[None, :] * p / (2 * 2.0 ** a)
        diff = np.abs(isr.out - fsr.out)
        assert np.all(diff <= bound * (1 + 1e-6) + 1e-12)
        errs.append(float(np.sqrt(np.mean(diff ** 2))))
        fine.append(int(qw.scale_i32[qw.scale_f32 > 0].min()) >= 4)
    # the error falls monotonically, and once the integer scales are a few units wide (rounding error uniform)
    # each factor 4 in alpha buys about a factor 4 in error
    for i, (e0, e1) in enumerate(zip(errs, errs[1:])):
        assert e1 < e0
        if fine[i]:
            assert 2.5 < e0 / e1 < 6.5
    assert sum(fine) >= 3
    # and the quantised layer approximates the fp16 layer it came from
    x, w, xq, sa, qw = _quantised_layer(M, N, K, 31, 10, mode)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    isr = O.gemm_w4a8_intscale(xq, sa, qw.qweight, qw.scale_i32, qw.chan_scale, 128, 10)
    rel = np.linalg.norm(isr.out - ref) / np.linalg.norm(ref)
    assert rel < 0.2


def test_dyadic_scales_make_both_equations_agree():
    """If every s * alpha is an integer, INT(.) changes nothing and Eq. (2) equals Eq. (1)."""
    rng = np.random.default_rng(12)
    N, K, G, M = 32, 1024, 128, 6
    w = rng.standard_normal((N, K)).astype(np.float32) * 0.01
    wg = w.reshape(N, K // G, G)
    # force each group's absmax to 7 * 2^-e so that s = 2^-e
    e = rng.integers(3, 9, size=(N, K // G))
    wg = wg / np.abs(wg).max(axis=2, keepdims=True) * (7.0 * 2.0 ** -e)[:, :, None]
    w16 = wg.reshape(N, K).astype(np.float16)
    x = S.activations_outlier(M, K, 77)
    xq, sa = O.quantize_act_int8_token(x)
    qw = O.quantize_weights_int4_group(w16, G, 10, O.SCALE_RAW)
    assert np.array_equal(qw.scale_i32.astype(np.float64), qw.scale_f32.astype(np.float64) * 1024)
    isr = O.gemm_w4a8_intscale(xq, sa, qw.qweight, qw.scale_i32, None, G, 10)
    fsr = O.gemm_w4a8_floatscale(xq, sa, qw.qweight, qw.scale_f32, G)
    assert np.allclose(isr.out, fsr.out, rtol=1e-12, atol=1e-14)
    assert np.array_equal(isr.out_fp16, fsr.out_fp16)


def test_overflow_bound_and_wraparound():
    """Appendix A.5: the 32-bit accumulator can overflow.  Worst-case inputs stay inside int32 up to the bound and
    wrap modulo 2^32 beyond it; the oracle reports both the wrapped value and the true sum."""
    K, G, N, M = 4096, 128, 4, 2
    bound = O.overflow_safe_scale_bound(K, G)
    assert bound == (2 ** 31 - 1) // (4096 * 1024) == 511
    xq = np.full((M, K), -128, dtype=np.int8)
    q = np.full((N, K), -8, dtype=np.int8)
    sa = np.ones(M, dtype=np.float32)
    ok = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), np.full((N, K // G), bound, np.int32), None, G, 10)
    assert np.all(ok.acc64 == 4096 * 1024 * bound) and np.all(ok.acc64 < 2 ** 31)
    assert np.array_equal(ok.acc.astype(np.int64), ok.acc64) and np.array_equal(ok.max_prefix, ok.acc64)
    over = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), np.full((N, K // G), bound + 1, np.int32), None, G, 10)
    true = 4096 * 1024 * (bound + 1)
    assert true >= 2 ** 31 and np.all(over.acc64 == true)
    assert np.all(over.acc.astype(np.int64) == true - 2 ** 32)
    assert np.all(over.out == (true - 2 ** 32) / 1024.0)
    # a prefix can leave int32 even when the final sum is back inside: signs alternate per group
    IS = np.full((N, K // G), 40000, np.int32)
    x2 = xq.copy()
    x2[:, K // 2:] = 127
    r = O.gemm_w4a8_intscale(x2, sa, O.pack_int4(q), IS, None, G, 10)
    half = 16 * 128 * 128 * 8 * 40000
    assert half >= 2 ** 31
    assert np.all(r.max_prefix == half)
    assert np.all(r.acc64 == half - 16 * 128 * 127 * 8 * 40000)
    assert np.array_equal(r.acc.astype(np.int64), r.acc64)      # wrap is harmless for the final value


def test_no_overflow_at_alpha_1024_on_benchmark_like_layers():
    """Sec. 6.1 / Appendix A.4: at amplifier 2^10 the accumulators stay within 2^31."""
    for K, N in ((4096, 64), (11008, 32)):
        x = S.activations_outlier(16, K, 5)
        w = S.weights_gaussian(N, K, 6, outlier_col_frac=0.005)
        xq, sa = O.quantize_act_int8_token(x)
        for mode in (O.SCALE_RAW, O.SCALE_NORM):
            qw = O.quantize_weights_int4_group(w, 128, 10, mode)
            r = O.gemm_w4a8_intscale(xq, sa, qw.qweight, qw.scale_i32, qw.chan_scale, 128, 10)
            assert r.max_prefix.max() < 2 ** 31
            assert np.array_equal(r.acc.astype(np.int64), r.acc64)


def test_grouped_form_matches_per_expert_calls():
    rng = np.random.default_rng(21)
    E, N, K, G, a = 3, 16, 256, 128, 10
    tok, exp, off = S.moe_routing(20, E, 2, seed=4)
    M = tok.size
    assert off[-1] == M and np.all(np.diff(exp) >= 0)
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    sa = rng.random(M).astype(np.float32)
    q = rng.integers(-8, 8, size=(E, N, K)).astype(np.int8)
    IS = rng.integers(0, 1025, size=(E, N, K // G)).astype(np.int32)
    c = rng.random((E, N)).astype(np.float32)
    qp = np.stack([O.pack_int4(q[e]) for e in range(E)])
    acc, out16 = O.gemm_w4a8_intscale_grouped(xq, sa, qp, IS, c, off, G, a)
    for m in range(M):
        e = int(exp[m])
        w_int = q[e].astype(np.int64) * np.repeat(IS[e].astype(np.int64), G, axis=1)
        assert np.array_equal(acc[m].astype(np.int64), xq[m].astype(np.int64) @ w_int.T)


def test_shape_mismatch_raises():
    xq = np.zeros((2, 8), np.int8)
    with pytest.raises(ValueError):
        O.gemm_w4a8_intscale(xq, np.ones(2, np.float32), np.zeros((3, 4), np.uint8), np.zeros((3, 1), np.int32), None, 4, 10)


# ------------------------------------------------------------------------------------------------ overflow-safe form
def test_layer_overflow_bound_is_reached_by_the_extreme_codes():
    """The bound is attained: all activation codes -128, all weight codes -8, non-negative scales."""
    rng = np.random.default_rng(11)
    N, K, G = 5, 256, 128
    IS = rng.integers(0, 5000, size=(N, K // G)).astype(np.int32)
    assert O.layer_overflow_bound(np.array([[3, -4]], np.int32), 128) == 7 * 128 * 128 * 8  # by hand
    bound = O.layer_overflow_bound(IS, G)
    assert bound == max(int(IS[n].astype(np.int64).sum()) for n in range(N)) * G * 1024
    xq = np.full((1, K), -128, np.int8)
    q = np.full((N, K), -8, np.int8)
    r = O.gemm_w4a8_intscale(xq, np.ones(1, np.float32), O.pack_int4(q), IS, None, G, 0)
    assert int(r.acc64.max()) == bound
    # scales within overflow_safe_scale_bound can never overflow
    cap = O.overflow_safe_scale_bound(K, G)
    assert O.layer_overflow_bound(np.full((3, K // G), cap, np.int32), G) < 2 ** 31
    assert O.layer_overflow_bound(np.full((3, K // G), cap + 1, np.int32), G) >= 2 ** 31


def test_safe_form_python_integers_and_overflow():
    """Brute force with python integers; where the 32-bit accumulator wraps, the safe form keeps the true value and
    differs from the wrapped one by a multiple of 2^32 (times the output factor)."""
    rng = np.random.default_rng(12)
    M, N, K, G, a = 3, 4, 32, 8, 10
    xq, q, _, _, sa, c = _rand_problem(rng, M, N, K, G)
    IS = rng.integers(-2 ** 27, 2 ** 27, size=(N, K // G)).astype(np.int32)  # large enough to wrap
    r = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, c, G, a)
    sres = O.gemm_w4a8_intscale_safe(xq, sa, O.pack_int4(q), IS, c, G, a)
    wrapped = 0
    for m in range(M):
        for n in range(N):
            acc, mag = 0, 0
            for g in range(K // G):
                p = sum(int(xq[m, k]) * int(q[n, k]) for k in range(g * G, (g + 1) * G))
                acc += p * int(IS[n, g])
                mag += abs(p * int(IS[n, g]))
            factor = Fraction(float(sa[m])) * Fraction(float(c[n])) / (2 ** a)
            assert sres.out[m, n] == pytest.approx(float(acc * factor), rel=1e-14, abs=0)
            assert sres.abs_sum[m, n] == pytest.approx(float(mag * factor), rel=1e-14, abs=0)
            assert (acc - int(r.acc[m, n])) % (2 ** 32) == 0
            wrapped += acc != int(r.acc[m, n])
    assert wrapped > 0, "the test is meant to include wrapped accumulators"


def test_safe_form_equals_eq2_without_overflow():
    rng = np.random.default_rng(13)
    M, N, K, G, a = 5, 24, 512, 128, 10
    xq, q, IS, _, sa, c = _rand_problem(rng, M, N, K, G)
    r = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q), IS, c, G, a)
    sres = O.gemm_w4a8_intscale_safe(xq, sa, O.pack_int4(q), IS, c, G, a)
    assert np.array_equal(r.acc.astype(np.int64), r.acc64)
    assert np.allclose(sres.out, r.out, rtol=1e-15, atol=0) and np.array_equal(sres.out_fp16, r.out_fp16)
    assert np.all(sres.abs_sum >= np.abs(sres.out) * (1 - 1e-12))


# ------------------------------------------------------------------------------------------------ W8A8
def test_w8a8_brute_force_and_plain_matmul():
    rng = np.random.default_rng(21)
    M, N, K, G, a = 3, 4, 24, 8, 9
    xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-128, 128, size=(N, K)).astype(np.int8)
    IS = rng.integers(-300, 300, size=(N, K // G)).astype(np.int32)
    s = (rng.random((N, K // G)) * 0.1).astype(np.float32)
    sa = (rng.random(M) + 0.01).astype(np.float32)
    c = (rng.random(N) + 0.01).astype(np.float32)
    r = O.gemm_w8a8_intscale(xq, sa, q, IS, c, G, a)
    f = O.gemm_w8a8_floatscale(xq, sa, q, s, G)
    for m in range(M):
        for n in range(N):
            acc, fs = 0, Fraction(0)
            for g in range(K // G):
                p = sum(int(xq[m, k]) * int(q[n, k]) for k in range(g * G, (g + 1) * G))
                acc += p * int(IS[n, g])
                fs += Fraction(p) * Fraction(float(s[n, g]))
            assert int(r.acc[m, n]) == acc == int(r.acc64[m, n])
            exact = Fraction(acc) * Fraction(float(sa[m])) * Fraction(float(c[n])) / 2 ** a
            assert r.out[m, n] == pytest.approx(float(exact), rel=1e-14, abs=0)
            assert f.out[m, n] == pytest.approx(float(Fraction(float(sa[m])) * fs), rel=1e-13, abs=1e-300)
    # one group with unit scale is the plain integer matmul; codes that fit 4 bits agree with the W4 oracle
    ones = np.ones((N, 1), np.int32)
    assert np.array_equal(O.gemm_w8a8_intscale(xq, sa, q, ones, None, K, 0).acc64, xq.astype(np.int64) @ q.astype(np.int64).T)
    q4 = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    r4 = O.gemm_w4a8_intscale(xq, sa, O.pack_int4(q4), IS, c, G, a)
    r8 = O.gemm_w8a8_intscale(xq, sa, q4, IS, c, G, a)
    assert np.array_equal(r4.acc, r8.acc) and np.array_equal(r4.out, r8.out) and np.array_equal(r4.max_prefix, r8.max_prefix)
    # wrap-around of the 32-bit accumulator
    big = np.full((N, K // G), 2 ** 30, np.int32)
    rw = O.gemm_w8a8_intscale(xq, sa, q, big, None, G, 0)
    assert np.all((rw.acc64 - rw.acc.astype(np.int64)) % 2 ** 32 == 0) and np.any(rw.acc64 != rw.acc)


def test_w8_weight_quantizer_hand_example_and_invariants():
    # s = 127 / 127 = 1 exactly: codes are the values rounded half to even
    w = np.array([[127.0, -126.5, 0.5, 1.5, 2.5, -0.5, -127.0, 64.0]], np.float16)
    r = O.quantize_weights_int8_group(w, 8, 3, O.SCALE_RAW)
    assert r.scale_f32[0, 0] == 1.0 and r.qweight.tolist() == [[127, -126, 0, 2, 2, 0, -127, 64]]
    assert r.scale_i32[0, 0] == 8 and r.chan_scale[0] == 1.0
    rng = np.random.default_rng(22)
    w = (rng.standard_normal((12, 512)) * 0.02).astype(np.float16)
    w[3, 128:256] = 0
    for mode in (O.SCALE_RAW, O.SCALE_NORM):
        r = O.quantize_weights_int8_group(w, 128, 10, mode)
        wg = w.astype(np.float64).reshape(12, 4, 128)
        qg = r.qweight.astype(np.float64).reshape(12, 4, 128)
        nz = r.scale_f32 > 0
        assert np.all(np.abs(qg).max(axis=2)[nz] == 127) and np.all(qg[~nz] == 0) and not nz[3, 1]
        assert np.all(np.abs(wg - qg * r.scale_f32.astype(np.float64)[:, :, None]) <= 0.5000001 * r.scale_f32[:, :, None])
        ratio = r.scale_f32 / r.chan_scale[:, None] if mode == O.SCALE_NORM else r.scale_f32
        assert np.all(np.abs(r.scale_i32 / 1024.0 - ratio) <= 0.5 / 1024 + 1e-7)
    assert O.quantize_weights_int8_group(w, 128, -1, O.SCALE_NORM).alpha_log2 == O.amplifier_log2(
        (r.scale_f32 / r.chan_scale[:, None]).astype(np.float32))
