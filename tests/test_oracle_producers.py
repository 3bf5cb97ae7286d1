"""Pins for the oracle's fused activation producers (RMSNorm / SiLU*up followed by the Appendix A.1 quantiser).

Independent formulations only: closed forms in double precision, hand-computed examples, exact invariants
(power-of-two scaling, constant rows, zero operands) and the half-ulp bound of one fp16 rounding.
"""
import numpy as np
import pytest

from oracle import oracle as O
import synth_inputs as S


def _ulp16(v):
    """Spacing of fp16 at |v| (subnormal spacing below the smallest normal)."""
    a = np.maximum(np.abs(np.asarray(v, dtype=np.float64)), 2.0 ** -14)
    return 2.0 ** (np.floor(np.log2(a)) - 10)


def test_exp_f32_against_double_exp():
    t = np.linspace(-87.0, 88.0, 350001).astype(np.float32)
    e = O.exp_f32(t).astype(np.float64)
    ref = np.exp(t.astype(np.float64))
    assert np.max(np.abs(e - ref) / ref) < 4e-7
    assert O.exp_f32(np.float32(0.0)) == np.float32(1.0)
    # the clamp: beyond the range the value of the nearest end
    assert O.exp_f32(np.float32(1000.0)) == O.exp_f32(np.float32(88.0))
    assert O.exp_f32(np.float32(-1000.0)) == O.exp_f32(np.float32(-87.0))
    # e^(a+b) = e^a e^b, loosely: catches a wrong ln2 split or a wrong polynomial coefficient
    a = np.float32(3.25)
    b = np.float32(-1.5)
    assert abs(float(O.exp_f32(a + b)) / (float(O.exp_f32(a)) * float(O.exp_f32(b))) - 1.0) < 1e-6


def test_silu_against_closed_form():
    g = np.concatenate([np.linspace(-30, 30, 200001), [0.0, 1e-3, -1e-3, 60.0, -60.0]]).astype(np.float32)
    s = O.silu_f32(g).astype(np.float64)
    g64 = g.astype(np.float64)
    ref = g64 / (1.0 + np.exp(-g64))
    assert np.max(np.abs(s - ref) / np.maximum(np.abs(ref), 1e-30)) < 1e-6
    assert O.silu_f32(np.float32(0.0)) == 0.0
    # SiLU(g) + SiLU(-g) = g tanh(g/2): a sign slip in the exponent fails this
    lhs = O.silu_f32(g).astype(np.float64) + O.silu_f32(-g).astype(np.float64)
    assert np.max(np.abs(lhs - g64 * np.tanh(g64 / 2))) < 1e-5
    # saturation: the identity for large g, zero for very negative g
    assert abs(float(O.silu_f32(np.float32(40.0))) - 40.0) < 1e-5
    assert abs(float(O.silu_f32(np.float32(-40.0)))) < 1e-15


def test_rmsnorm_hand_example():
    # mean(x^2) = (9 + 16) / 4 = 6.25, r = 0.4: y = (1.2, 0.8, 0, 0) with gamma (1, 0.5, 1, 1)
    x = np.array([[3.0, 4.0, 0.0, 0.0]], dtype=np.float16)
    gamma = np.array([1.0, 0.5, 1.0, 1.0], dtype=np.float16)
    y = O.rmsnorm_fp16(x, gamma, 0.0)
    assert y.dtype == np.float16
    assert np.array_equal(y, np.array([[1.2, 0.8, 0.0, 0.0]], dtype=np.float16))
    xq, sa = O.rmsnorm_quantize_act_int8_token(x, gamma, 0.0)
    # fp16(1.2) = 1.2001953125, fp16(0.8) = 0.7998046875: 0.7998046875 / 1.2001953125 * 127 = 84.63 -> 85
    assert sa[0] == np.float32(1.2001953125) / np.float32(127.0)
    assert xq.tolist() == [[127, 85, 0, 0]]


def test_rmsnorm_constant_rows_and_gamma_columns():
    K = 96
    x = np.full((3, K), 0.75, dtype=np.float16)
    x[1] *= -1
    x[2] *= 64
    gamma = np.ones(K, dtype=np.float16)
    gamma[5] = 0.0
    gamma[7] = -0.5
    y = O.rmsnorm_fp16(x, gamma, 0.0).astype(np.float64)
    want = np.sign(x.astype(np.float64)) * gamma.astype(np.float64)[None, :]
    assert np.array_equal(y, want)
    xq, sa = O.rmsnorm_quantize_act_int8_token(x, gamma, 0.0)
    assert np.all(sa == np.float32(1.0) / np.float32(127.0))
    assert np.all(xq[:, 5] == 0)
    assert xq[0, 7] == -64 and xq[1, 7] == 64          # 63.5 rounds to even
    assert np.all(xq[0, :5] == 127) and np.all(xq[1, :5] == -127)


def test_rmsnorm_power_of_two_invariance():
    # without eps the normalised row does not change when the input is scaled by a power of two
    x = S.activations_outlier(9, 512, seed=11).astype(np.float16)
    x = np.clip(x, -40, 40).astype(np.float16)
    gamma = (1.0 + 0.1 * np.random.default_rng(3).standard_normal(512)).astype(np.float16)
    base = O.rmsnorm_fp16(x, gamma, 0.0)
    for k in (-3, 2, 7):
        scaled = (x.astype(np.float32) * np.float32(2.0 ** k)).astype(np.float16)
        assert np.array_equal(O.rmsnorm_fp16(scaled, gamma, 0.0), base)
    q0 = O.rmsnorm_quantize_act_int8_token(x, gamma, 0.0)
    q1 = O.rmsnorm_quantize_act_int8_token((x.astype(np.float32) * 4).astype(np.float16), gamma, 0.0)
    assert np.array_equal(q0[0], q1[0]) and np.array_equal(q0[1], q1[1])


@pytest.mark.parametrize("eps", [1e-5, 1e-2, 10.0])
def test_rmsnorm_against_double_formula(eps):
    M, K = 17, 1000
    x = S.activations_outlier(M, K, seed=21).astype(np.float16)
    gamma = (1.0 + 0.2 * np.random.default_rng(5).standard_normal(K)).astype(np.float16)
    y = O.rmsnorm_fp16(x, gamma, eps).astype(np.float64)
    x64 = x.astype(np.float64)
    ref = x64 / np.sqrt(np.mean(x64 * x64, axis=1, keepdims=True) + eps) * gamma.astype(np.float64)[None, :]
    # one fp16 rounding of a value computed to ~3 single-precision ulps
    assert np.all(np.abs(y - ref) <= 0.5 * _ulp16(ref) * (1 + 1e-3) + 1e-12)
    # de-quantised codes reproduce the normalised row to half a step
    xq, sa = O.rmsnorm_quantize_act_int8_token(x, gamma, eps)
    step = sa.astype(np.float64)[:, None]
    assert np.all(np.abs(xq.astype(np.float64) * step - y) <= 0.5 * step * (1 + 1e-6))
    assert np.array_equal(sa, (np.abs(y).max(axis=1) / 127.0).astype(np.float32)) or \
        np.allclose(sa, np.abs(y).max(axis=1) / 127.0, rtol=2e-7)


def test_rmsnorm_eps_dominates_small_rows():
    x = np.full((1, 64), 2.0 ** -10, dtype=np.float16)
    gamma = np.ones(64, dtype=np.float16)
    y = O.rmsnorm_fp16(x, gamma, 1.0).astype(np.float64)
    # mean(x^2) = 2^-20 against eps = 1: y = x / sqrt(1 + 2^-20) -> x to fp16 precision
    assert np.array_equal(y, x.astype(np.float64))


def test_silu_mul_layout_and_values():
    # gate | up: SiLU(10) * 0.5 and SiLU(0.5) * 10 differ, so swapped halves fail
    gate_up = np.array([[10.0, 0.5, 0.5, 10.0]], dtype=np.float16)
    h = O.silu_mul_fp16(gate_up).astype(np.float64)
    want = np.array([[10.0 / (1 + np.exp(-10.0)) * 0.5, 0.5 / (1 + np.exp(-0.5)) * 10.0]])
    assert h.shape == (1, 2)
    assert np.all(np.abs(h - want) <= 0.5 * _ulp16(want) * (1 + 1e-3))
    assert abs(want[0, 0] - want[0, 1]) > 1.0


def test_silu_mul_zero_operands():
    rng = np.random.default_rng(8)
    inter = 40
    gate = rng.standard_normal((4, inter)).astype(np.float16)
    up = rng.standard_normal((4, inter)).astype(np.float16)
    z = np.zeros_like(gate)
    for gu in (np.concatenate([gate, z], axis=1), np.concatenate([z, up], axis=1)):
        xq, sa = O.silu_mul_quantize_act_int8_token(gu)
        assert not xq.any() and not sa.any()


def test_silu_mul_against_double_formula():
    M, inter = 13, 1536
    rng = np.random.default_rng(31)
    gate = (3.0 * rng.standard_normal((M, inter))).astype(np.float16)
    up = S.activations_outlier(M, inter, seed=32).astype(np.float16)
    gu = np.concatenate([gate, up], axis=1)
    h = O.silu_mul_fp16(gu).astype(np.float64)
    g64, u64 = gate.astype(np.float64), up.astype(np.float64)
    ref = g64 / (1.0 + np.exp(-g64)) * u64
    assert np.all(np.abs(h - ref) <= 0.5 * _ulp16(ref) * (1 + 2e-3) + 1e-12)
    xq, sa = O.silu_mul_quantize_act_int8_token(gu)
    assert xq.shape == (M, inter) and xq.dtype == np.int8 and sa.shape == (M,)
    step = sa.astype(np.float64)[:, None]
    assert np.all(np.abs(xq.astype(np.float64) * step - h) <= 0.5 * step * (1 + 1e-6))
    assert np.all(np.abs(xq).max(axis=1) == 127)


def test_silu_mul_rejects_odd_width():
    with pytest.raises(ValueError):
        O.silu_mul_fp16(np.zeros((2, 7), dtype=np.float16))
