"""GPU parity of the activation quantiser folded into its producer (RMSNorm, SiLU * up) against the CPU oracle:
codes and token scales bit-exact, since both sides take every floating-point decision in the same precision and
order.
"""
import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_14597_amd as pkg
    pkg.load_library()
    return pkg


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def _gamma(K, seed):
    return (1.0 + 0.25 * np.random.default_rng(seed).standard_normal(K)).astype(np.float16)


# few rows (1024 lanes per row, 1 / 2 / 4 chunks per lane), many rows (256 lanes, 2 / 8 / 16 chunks), the three-pass
# kernel (K = 40000), one chunk, ragged last chunk slots
@pytest.mark.parametrize("M,K,eps", [(1, 4096, 1e-5), (7, 4096, 1e-6), (33, 5120, 1e-5), (5, 8192, 1e-5),
                                     (3, 14336, 1e-5), (2, 28672, 1e-6), (2, 40000, 1e-5), (64, 128, 1e-5),
                                     (3, 8, 1e-5), (130, 11008, 1e-2), (260, 11008, 1e-5), (257, 28672, 1e-5), (300, 2048, 1e-5)])
def test_rmsnorm_quantize_bit_exact(P, M, K, eps):
    x = S.activations_outlier(M, K, 100 + K % 97).astype(np.float16)
    if M > 2:
        x[1] = 0                       # an all-zero token row: r = 1 / sqrt(eps), codes 0
        x[2, K // 2] = 30000           # a large outlier
    gamma = _gamma(K, 7)
    gamma[0] = 0
    xq_ref, sa_ref = O.rmsnorm_quantize_act_int8_token(x, gamma, eps)
    xq, sa = P.is_rmsnorm_quantize_act_int8_token(dev(x), dev(gamma), eps)
    assert np.array_equal(host(sa), sa_ref)
    assert np.array_equal(host(xq), xq_ref)


def test_rmsnorm_quantize_prefill_size(P):
    M, K = 4096, 4096
    x = S.activations_outlier(M, K, 5).astype(np.float16)
    gamma = _gamma(K, 9)
    xq_ref, sa_ref = O.rmsnorm_quantize_act_int8_token(x, gamma, 1e-5)
    xq, sa = P.is_rmsnorm_quantize_act_int8_token(dev(x), dev(gamma), 1e-5)
    assert np.array_equal(host(sa), sa_ref)
    assert np.array_equal(host(xq), xq_ref)


def test_rmsnorm_quantize_matches_unfused_chain(P):
    """The fused call against the library's own quantiser fed with the oracle's fp16 norm output."""
    M, K = 19, 4096
    x = S.activations_student_t(M, K, 15).astype(np.float16)
    gamma = _gamma(K, 3)
    y = O.rmsnorm_fp16(x, gamma, 1e-5)
    xq_u, sa_u = P.is_quantize_act_int8_token(dev(y))
    xq, sa = P.is_rmsnorm_quantize_act_int8_token(dev(x), dev(gamma), 1e-5)
    assert torch.equal(xq, xq_u) and torch.equal(sa, sa_u)


def test_rmsnorm_quantize_empty_and_bad_arguments(P):
    x = torch.empty((0, 4096), dtype=torch.float16, device="cuda:0")
    g = torch.ones((4096,), dtype=torch.float16, device="cuda:0")
    xq, sa = P.is_rmsnorm_quantize_act_int8_token(x, g, 1e-5)
    assert xq.shape == (0, 4096) and sa.shape == (0,)
    x1 = torch.ones((2, 4096), dtype=torch.float16, device="cuda:0")
    for eps in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(P.IntScaleError):
            P.is_rmsnorm_quantize_act_int8_token(x1, g, eps)


# few rows (1024 lanes per row), many rows (256 lanes, 2 / 8 / 16 chunks per lane), the two-pass kernel
# (inter = 40960), one chunk, a ragged tail
@pytest.mark.parametrize("M,inter", [(1, 11008), (8, 11008), (33, 14336), (3, 28672), (2, 40960), (64, 136),
                                     (5, 8), (130, 4096), (260, 11008), (257, 28672), (300, 2048)])
def test_silu_mul_quantize_bit_exact(P, M, inter):
    rng = np.random.default_rng(200 + inter % 89)
    gate = (3.0 * rng.standard_normal((M, inter))).astype(np.float16)
    up = S.activations_outlier(M, inter, 300 + M).astype(np.float16)
    up = np.clip(up, -200, 200).astype(np.float16)
    if M > 2:
        up[1] = 0                      # an all-zero product row
        gate[2, :8] = [-100, 100, -20, 20, -88, 88, 0, -0.0]     # both clamps of the exponent, zeros
    gu = np.concatenate([gate, up], axis=1)
    xq_ref, sa_ref = O.silu_mul_quantize_act_int8_token(gu)
    xq, sa = P.is_silu_mul_quantize_act_int8_token(dev(gu))
    assert np.array_equal(host(sa), sa_ref)
    assert np.array_equal(host(xq), xq_ref)


def test_silu_mul_quantize_prefill_size(P):
    M, inter = 2048, 14336
    rng = np.random.default_rng(41)
    gate = (2.0 * rng.standard_normal((M, inter))).astype(np.float16)
    up = rng.standard_normal((M, inter)).astype(np.float16)
    gu = np.concatenate([gate, up], axis=1)
    xq_ref, sa_ref = O.silu_mul_quantize_act_int8_token(gu)
    xq, sa = P.is_silu_mul_quantize_act_int8_token(dev(gu))
    assert np.array_equal(host(sa), sa_ref)
    assert np.array_equal(host(xq), xq_ref)


def _fp16_tie_pairs(count, seed):
    """(gate, up) fp16 pairs whose single-precision product SiLU(gate) * up lies exactly half way between two fp16
    values while the exact product does not: rounding it once, straight to fp16, gives the other neighbour."""
    rng = np.random.default_rng(seed)
    gs, us = [], []
    while len(gs) < count:
        g = (rng.uniform(3.0, 8.0, 1 << 20)).astype(np.float16)
        u = (rng.uniform(4.0, 8.0, 1 << 20) * rng.choice([-1.0, 1.0], 1 << 20)).astype(np.float16)
        s32 = O.silu_f32(g.astype(np.float32))
        p32 = s32 * u.astype(np.float32)
        tie = (p32.view(np.uint32) & 0x1FFF) == 0x1000          # 13 bits below fp16's last place: exactly one half
        exact = s32.astype(np.float64) * u.astype(np.float64)
        once = exact.astype(np.float16)                            # the exact product rounded once
        twice = p32.astype(np.float16)
        pick = np.flatnonzero(tie & (once != twice))
        gs += g[pick].tolist()
        us += u[pick].tolist()
    return np.array(gs[:count], np.float16), np.array(us[:count], np.float16)


def test_silu_mul_rounds_to_fp32_before_fp16(P):
    """The product is rounded to single precision and then to fp16 (the stated definition), also where a conversion
    merged into the multiply would round differently: rows whose largest product sits on such a tie (its fp16 value
    is the token scale) and rows made of such products only."""
    g, u = _fp16_tie_pairs(96, 77)
    assert np.abs(O.silu_f32(g.astype(np.float32)) * u.astype(np.float32)).min() > 8.0
    rng = np.random.default_rng(78)
    M, inter = 64, 2048
    gate = rng.standard_normal((M, inter)).astype(np.float16)
    up = rng.standard_normal((M, inter)).astype(np.float16)
    gate[:, 5], up[:, 5] = g[:M], u[:M]                            # the row's absmax
    gate[:32, 100:132], up[:32, 100:132] = g[64:96], u[64:96]
    gu = np.concatenate([gate, up], axis=1)
    for rows in (gu, gu[:3], np.repeat(gu, 5, axis=0)):            # 1024 lanes per row, and 256
        xq_ref, sa_ref = O.silu_mul_quantize_act_int8_token(rows)
        xq, sa = P.is_silu_mul_quantize_act_int8_token(dev(rows))
        assert np.array_equal(host(sa), sa_ref)
        assert np.array_equal(host(xq), xq_ref)


def test_silu_mul_quantize_empty(P):
    gu = torch.empty((0, 256), dtype=torch.float16, device="cuda:0")
    xq, sa = P.is_silu_mul_quantize_act_int8_token(gu)
    assert xq.shape == (0, 128) and sa.shape == (0,)


# ---- the same two calls against the plain definitions in double precision (nothing of the oracle, no polynomial):
# y = x / sqrt(mean(x^2) + eps) * gamma and h = g / (1 + exp(-g)) * u, rounded to fp16, then Appendix A.1 per row.
def _check_against_plain_definition(h64, xq, sa):
    """h64: the producer's output in double precision.  The kernel rounds its own single-precision value to fp16, which
    can differ from fp16(h64) by one fp16 step (relative 2^-10) where h64 sits next to a rounding boundary; that bounds
    what may differ downstream:
      token scale: s_a * 127 within one fp16 step of the row's absmax;
      codes: equal to rint(h64 / s_a) except where that quotient lies within |q| * 2^-10 (+ 1e-4) of a half-integer,
             and there by one at most."""
    M, K = h64.shape
    assert xq.shape == (M, K) and sa.shape == (M,)
    amax = np.abs(h64).max(axis=1)
    step16 = np.spacing(amax.astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(sa.astype(np.float64) * 127.0 - amax) <= step16 * 1.001 + 1e-30)
    live = sa > 0
    assert np.all(xq[~live] == 0)
    q = h64[live] / sa[live].astype(np.float64)[:, None]
    want = np.clip(np.rint(q), -128, 127)
    diff = xq[live].astype(np.int64) - want.astype(np.int64)
    eps = np.abs(q) * 2.0 ** -10 + 1e-4
    near_half = np.abs(np.abs(q - np.floor(q)) - 0.5) <= eps
    assert np.all((diff == 0) | (near_half & (np.abs(diff) <= 1)))
    assert np.count_nonzero(diff) <= 0.02 * diff.size + 4      # and such places are rare


@pytest.mark.parametrize("M,K,eps", [(1, 4096, 1e-5), (33, 5120, 1e-5), (5, 8192, 1e-6), (2, 28672, 1e-5),
                                     (300, 2048, 1e-5), (130, 11008, 1e-2)])
def test_rmsnorm_quantize_against_plain_double_precision_definition(P, M, K, eps):
    x = S.activations_outlier(M, K, 300 + K % 89).astype(np.float16)
    if M > 2:
        x[1] = 0
    gamma = _gamma(K, 11)
    x64, g64 = x.astype(np.float64), gamma.astype(np.float64)
    y64 = x64 / np.sqrt(np.mean(x64 * x64, axis=1, keepdims=True) + eps) * g64[None, :]
    xq, sa = P.is_rmsnorm_quantize_act_int8_token(dev(x), dev(gamma), eps)
    _check_against_plain_definition(y64, host(xq), host(sa))


@pytest.mark.parametrize("M,I", [(1, 11008), (16, 11008), (64, 14336), (3, 28672), (300, 2048), (2, 8)])
def test_silu_mul_quantize_against_plain_double_precision_definition(P, M, I):
    gu = S.activations_outlier(M, 2 * I, 400 + I % 83).astype(np.float16)
    if M > 2:
        gu[1] = 0
    g64, u64 = gu[:, :I].astype(np.float64), gu[:, I:].astype(np.float64)
    h64 = g64 / (1.0 + np.exp(-g64)) * u64
    xq, sa = P.is_silu_mul_quantize_act_int8_token(dev(gu))
    _check_against_plain_definition(h64, host(xq), host(sa))
