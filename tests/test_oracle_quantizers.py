"""Pins for the oracle's quantisers (Appendix A.1, A.2; Eq. (2)'s INT(s*alpha); Sec. 4.1 amplifier search).

None of these re-type the oracle's formula: they are hand-worked examples with exactly representable values,
invariants that follow from the definition, and the facts the paper states.
"""
import json
import os

import numpy as np
import pytest

from oracle import oracle as O
import synth_inputs as S


def test_weight_quantizer_hand_example_ties_to_even():
    # One row, one group of 8. absmax = 7/8 so s = 1/8 exactly and every w/s below is exact in fp32.
    # Multiples of s: 7, -3.5, 2.5, 1.5, -0.5, 0, -7, 4  -> round-half-even: 7, -4, 2, 2, -0, 0, -7, 4.
    w = np.array([[0.875, -0.4375, 0.3125, 0.1875, -0.0625, 0.0, -0.875, 0.5]], dtype=np.float16)
    r = O.quantize_weights_int4_group(w, group=8, alpha_log2=10, scale_mode=O.SCALE_RAW)
    assert r.scale_f32.tolist() == [[0.125]]
    assert O.unpack_int4(r.qweight).tolist() == [[7, -4, 2, 2, 0, 0, -7, 4]]
    # canonical packing: even k in the low nibble, two's-complement nibbles
    assert r.qweight.tolist() == [[0xC7, 0x22, 0x00, 0x49]]
    assert r.scale_i32.tolist() == [[128]]          # 0.125 * 2^10
    assert r.chan_scale.tolist() == [1.0]
    assert r.alpha_log2 == 10


def test_weight_quantizer_two_groups_raw_and_norm():
    # group 0: absmax 7/8 (s = 1/8); group 1: absmax 7/16 (s = 1/16)
    g0 = [0.875, 0.125, -0.25, 0.0]
    g1 = [0.0625, -0.4375, 0.1875, 0.03125]     # /s: 1, -7, 3, 0.5 -> 1, -7, 3, 0
    w = np.array([g0 + g1], dtype=np.float16)
    raw = O.quantize_weights_int4_group(w, group=4, alpha_log2=6, scale_mode=O.SCALE_RAW)
    assert raw.scale_f32.tolist() == [[0.125, 0.0625]]
    assert O.unpack_int4(raw.qweight).tolist() == [[7, 1, -2, 0, 1, -7, 3, 0]]
    assert raw.scale_i32.tolist() == [[8, 4]]
    assert raw.chan_scale.tolist() == [1.0]
    norm = O.quantize_weights_int4_group(w, group=4, alpha_log2=6, scale_mode=O.SCALE_NORM)
    assert norm.chan_scale.tolist() == [0.125]
    assert norm.scale_i32.tolist() == [[64, 32]]      # (s/c) * 2^6 = 1*64, 0.5*64
    assert np.array_equal(norm.qweight, raw.qweight)
    assert np.array_equal(norm.scale_f32, raw.scale_f32)


def test_weight_quantizer_zero_group_and_zero_row():
    w = np.zeros((2, 8), dtype=np.float16)
    w[0, 4:] = [0.5, -0.25, 0.125, 0.0]
    for mode in (O.SCALE_RAW, O.SCALE_NORM):
        r = O.quantize_weights_int4_group(w, group=4, alpha_log2=8, scale_mode=mode)
        q = O.unpack_int4(r.qweight)
        assert q[1].tolist() == [0] * 8 and q[0, :4].tolist() == [0] * 4
        assert r.scale_f32[1].tolist() == [0.0, 0.0] and r.scale_f32[0, 0] == 0.0
        assert r.scale_i32[1].tolist() == [0, 0] and r.scale_i32[0, 0] == 0
        assert np.all(np.isfinite(r.chan_scale))


def test_scale_count_matches_paper(golden_dir):
    facts = json.load(open(os.path.join(golden_dir, "paper_facts.json")))
    w = S.weights_gaussian(4096, 4096, seed=1)
    r = O.quantize_weights_int4_group(w, group=facts["group_size"]["value"], alpha_log2=10)
    assert r.scale_f32.size == facts["dense_4096x4096_group128_scale_count"]["value"]
    assert r.scale_i32.size == r.scale_f32.size
    assert r.qweight.shape == (4096, 2048)


@pytest.mark.parametrize("group", [32, 128])
def test_weight_quantizer_invariants(group):
    N, K = 96, 1024
    w = S.weights_gaussian(N, K, seed=11, outlier_col_frac=0.01)
    r = O.quantize_weights_int4_group(w, group=group, alpha_log2=10)
    q = O.unpack_int4(r.qweight).astype(np.int32)
    qg = q.reshape(N, K // group, group)
    wg = w.astype(np.float64).reshape(N, K // group, group)
    s = r.scale_f32.astype(np.float64)
    # the element of largest magnitude maps to +-7, nothing reaches -8 with this scale definition
    assert np.all(np.abs(qg).max(axis=2) == 7)
    assert q.min() >= -7 and q.max() <= 7
    # scale is absmax / 7 (to fp32 rounding)
    assert np.allclose(s * 7.0, np.abs(wg).max(axis=2), rtol=2e-7, atol=0)
    # rounding to nearest: reconstruction error at most half a step (plus fp32 slack)
    err = np.abs(wg - qg * s[:, :, None])
    assert np.all(err <= 0.5 * s[:, :, None] * (1 + 1e-5))
    # sign is preserved wherever the code is non-zero
    nz = qg != 0
    assert np.all(np.sign(qg[nz]) == np.sign(wg[nz]))


def test_integer_scale_is_nearest_integer():
    N, K, G = 64, 2048, 128
    w = S.weights_gaussian(N, K, seed=5)
    for a in (6, 8, 10, 12):
        raw = O.quantize_weights_int4_group(w, G, a, O.SCALE_RAW)
        alpha = 2.0 ** a
        d = raw.scale_i32.astype(np.float64) / alpha - raw.scale_f32.astype(np.float64)
        assert np.all(np.abs(d) <= 0.5 / alpha)
        norm = O.quantize_weights_int4_group(w, G, a, O.SCALE_NORM)
        ratio = norm.scale_f32.astype(np.float64) / norm.chan_scale.astype(np.float64)[:, None]
        d = norm.scale_i32.astype(np.float64) / alpha - ratio
        assert np.all(np.abs(d) <= 0.5 / alpha + 1e-7)
        assert norm.scale_i32.max() == 2 ** a and norm.scale_i32.min() >= 0
        assert np.array_equal(norm.chan_scale, norm.scale_f32.max(axis=1))


def test_weight_mse_at_alpha_1024_is_in_the_papers_range(golden_dir):
    """Sec. 4.1: weight MSE between integer-scale and float-scale de-quantised weights at 2^10 lies in (1e-7, 1e-6).

    With round-to-nearest the scale error is uniform in +-1/(2 alpha): MSE = E[q^2] / (12 alpha^2), about 5e-7 for
    Gaussian groups.  Truncating INT(.) instead would give E[q^2] / (3 alpha^2), about 2e-6, outside the range.
    """
    facts = json.load(open(os.path.join(golden_dir, "paper_facts.json")))
    lo, hi = facts["weight_mse_alpha_2p10_open_range"]["value"]
    w = S.weights_gaussian(256, 4096, seed=3)
    r = O.quantize_weights_int4_group(w, 128, 10, O.SCALE_RAW)
    q = O.unpack_int4(r.qweight).astype(np.float64).reshape(256, 32, 128)
    w_fs = q * r.scale_f32.astype(np.float64)[:, :, None]
    w_is = q * (r.scale_i32.astype(np.float64) / 1024.0)[:, :, None]
    mse = float(np.mean((w_is - w_fs) ** 2))
    assert lo < mse < hi
    closed_form = float(np.mean(q ** 2)) / (12 * 1024.0 ** 2)
    assert abs(mse - closed_form) < 0.15 * closed_form
    # the truncating reading is outside the stated range
    trunc = q * (np.floor(r.scale_f32.astype(np.float64) * 1024.0) / 1024.0)[:, :, None]
    assert float(np.mean((trunc - w_fs) ** 2)) > hi


@pytest.mark.parametrize("smin,expected", [(0.9, 1), (0.5, 1), (2.0 ** -9, 9), (0.0015, 10), (1.01 * 2.0 ** -10, 10),
                                           (1.0, 0), (3.0, 0), (2.0 ** -10, 10), (0.99 * 2.0 ** -10, 11)])
def test_amplifier_search(smin, expected):
    # Sec. 4.1: the first power of two 2^i with smin * 2^i >= 1.
    scales = np.array([0.7, smin, 5.0, 0.0], dtype=np.float32)   # zeros are ignored
    if smin > 0.7:
        scales[0] = smin + 1
    a = O.amplifier_log2(scales)
    assert a == expected
    assert smin * 2.0 ** a >= 1.0 and (a == 0 or smin * 2.0 ** (a - 1) < 1.0)


def test_amplifier_search_cap_and_empty():
    assert O.amplifier_log2(np.array([1e-9], dtype=np.float32)) == 16
    assert O.amplifier_log2(np.zeros(4, dtype=np.float32)) == 0


@pytest.mark.parametrize("sigma", [0.02, 0.012, 0.008, 0.006, 0.004])
def test_heuristic_amplifier_is_the_first_power_of_two_that_lifts_every_scale_to_one(sigma):
    """Sec. 4.1 (the heuristic search of Listing 1), written out here as the plain doubling loop: the amplifier is the
    first power of two whose product with the smallest group scale reaches 1."""
    w = S.weights_gaussian(512, 4096, seed=9, sigma=sigma)
    r = O.quantize_weights_int4_group(w, 128, -1, O.SCALE_RAW)
    smin = float(r.scale_f32.min())
    shifts, amp = 0, 1.0
    while smin * amp < 1.0:
        amp *= 2.0
        shifts += 1
    assert r.alpha_log2 == shifts
    assert r.scale_i32.min() >= 1


def test_heuristic_amplifier_on_llm_like_weights(golden_dir):
    """Sec. 4.1 / Fig. 3(b): the layers of LLaMA-2-7B need 9 or 10 shifts, that is, their smallest group scale lies in
    [2^-10, 2^-8).  Gaussian weights put it there for a standard deviation of 0.004 to 0.012 (the bulk of an LLM's
    linear layers); the benchmark recipe's 0.02 has its smallest scale at 2^-7.6 and needs 8, which is why that value
    is not part of this pin."""
    facts = json.load(open(os.path.join(golden_dir, "paper_facts.json")))
    for sigma in (0.012, 0.008, 0.006, 0.004):
        w = S.weights_gaussian(512, 4096, seed=9, sigma=sigma)
        r = O.quantize_weights_int4_group(w, 128, -1, O.SCALE_RAW)
        assert r.alpha_log2 in facts["typical_bit_shifts"]["value"], sigma
        assert 2.0 ** -10 <= float(r.scale_f32.min()) < 2.0 ** -8
        assert r.scale_i32.min() >= 1


def test_act_quantizer_hand_example():
    # absmax = 127/64 -> s_a = 1/64 exactly; entries are (k + 1/2)/64 ties and plain multiples.
    x = np.array([[127 / 64, -2.5 / 64, 1.5 / 64, 0.5 / 64, -0.5 / 64, 100 / 64, -127 / 64, 0.0],
                  [0.0] * 8], dtype=np.float16)
    xq, sa = O.quantize_act_int8_token(x)
    assert sa.tolist() == [1 / 64, 0.0]
    assert xq[0].tolist() == [127, -2, 2, 0, 0, 100, -127, 0]
    assert xq[1].tolist() == [0] * 8


def test_act_quantizer_invariants():
    x = S.activations_outlier(33, 4096, seed=2)
    xq, sa = O.quantize_act_int8_token(x)
    x64 = x.astype(np.float64)
    assert np.all(np.abs(xq.astype(np.int32)).max(axis=1) == 127)
    assert xq.min() >= -127
    assert np.allclose(sa.astype(np.float64) * 127.0, np.abs(x64).max(axis=1), rtol=2e-7, atol=0)
    err = np.abs(x64 - xq.astype(np.float64) * sa.astype(np.float64)[:, None])
    assert np.all(err <= 0.5 * sa.astype(np.float64)[:, None] * (1 + 1e-5))
    # per-token: scaling one row changes only that row's scale, never its codes
    x2 = x.copy()
    x2[5] = (x2[5].astype(np.float32) * 0.5).astype(np.float16)
    xq2, sa2 = O.quantize_act_int8_token(x2)
    assert np.array_equal(np.delete(xq2, 5, 0), np.delete(xq, 5, 0)) and np.array_equal(np.delete(sa2, 5), np.delete(sa, 5))
    assert sa2[5] == sa[5] * 0.5


def test_pack_unpack_roundtrip_and_nibble_order():
    q = np.arange(-8, 8, dtype=np.int8).reshape(1, 16)
    p = O.pack_int4(q)
    assert p.tolist() == [[0x98, 0xBA, 0xDC, 0xFE, 0x10, 0x32, 0x54, 0x76]]
    assert np.array_equal(O.unpack_int4(p), q)


def test_bad_arguments_raise():
    w = np.zeros((2, 6), dtype=np.float16)
    with pytest.raises(ValueError):
        O.quantize_weights_int4_group(w, group=4, alpha_log2=10)
    with pytest.raises(ValueError):
        O.quantize_weights_int4_group(np.zeros((2, 8), np.float16), group=4, alpha_log2=17)
