"""Pins for the layer on the TLQ levels themselves ("Hardware Implementation": a code's value is
+-round(2^r 2^I) 2^(f-I)), the fidelity reference of the int8-table path.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth

GRID = synth.DEFAULT_GRID


def _case(bits, N=24, K=128, M=7, seed=0):
    rng = np.random.default_rng(seed)
    W = (rng.standard_t(4, (N, K)) * 0.02).astype(np.float32)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    codes = oracle.tlq_encode(W, p)
    q = rng.integers(-127, 128, (M, K)).astype(np.int8)
    scale = (rng.random(M) + 0.5).astype(np.float32)
    return W, p, codes, q, scale


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("I", [0, 3, 6, 7])
def test_levels_with_up_to_seven_mantissa_bits_are_bf16_values(bits, I):
    # round(2^r 2^I) lies in [2^I, 2^(I+1)]: at most 8 significant bits for I <= 7, which is what bf16 holds
    _, p, _, _, _ = _case(bits, seed=I)
    v = oracle.tlq_level_values(p, I)
    back = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(v))
    assert np.array_equal(back, v)
    mant = np.abs(v) / np.exp2(np.floor(np.log2(np.abs(v))))            # in [1, 2)
    assert np.array_equal(mant * 128, np.rint(mant * 128))


def test_eight_mantissa_bits_do_not_fit():
    _, p, _, _, _ = _case(4, seed=5)
    v = oracle.tlq_level_values(p, 8)
    back = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(v))
    assert not np.array_equal(back, v)


@pytest.mark.parametrize("bits", [3, 4])
def test_against_exact_rational_arithmetic(bits):
    # every level is a dyadic rational, every q an integer: the sum is a rational number that Fractions hold exactly
    _, p, codes, q, scale = _case(bits, N=5, K=64, M=3, seed=11)
    v = oracle.tlq_level_values(p, 7)
    bias = np.linspace(-1, 1, 5).astype(np.float32)
    y = oracle.qlinear_levels_from_parts(q, scale, codes, v, bits, bias)
    mask = 2 ** bits - 1
    for t in range(3):
        for n in range(5):
            acc = sum(int(q[t, k]) * Fraction(float(v[n, int(codes[n, k]) & mask])) for k in range(64))
            ref = float(acc * Fraction(float(scale[t])) + Fraction(float(bias[n])))
            assert y[t, n] == pytest.approx(ref, rel=1e-13, abs=1e-300)


@pytest.mark.parametrize("bits", [3, 4])
def test_distance_to_the_int8_table_path_is_the_table_rounding(bits):
    # lut = rint(v / wscale): each weight moves by at most wscale / 2, so the two layers differ by at most
    # scale_t * (wscale_n / 2) * sum_k |q[t, k]|; and they do differ (the table does round)
    _, p, codes, q, scale = _case(bits, seed=3)
    v = oracle.tlq_level_values(p, 7)
    lut, wscale = oracle.tlq_lut(p, 7)
    y_lv = oracle.qlinear_levels_from_parts(q, scale, codes, v, bits)
    y_i8 = oracle.qlinear_from_parts(q, scale, codes, lut, wscale, bits)
    bound = (scale.astype(np.float64)[:, None] * np.abs(q.astype(np.float64)).sum(axis=1)[:, None]
             * (wscale.astype(np.float64)[None, :] / 2)) * (1 + 1e-6)     # wscale itself is rounded to fp32
    assert np.all(np.abs(y_lv - y_i8) <= bound)
    assert np.any(y_lv != y_i8)


def test_reduces_to_the_fake_quant_product_with_dequantized_weights():
    # with I < 0 the levels are Eq. dequant's 2^e exactly: the layer is (q * scale) . W_f^T
    _, p, codes, q, scale = _case(4, seed=9)
    v = oracle.tlq_level_values(p, -1)
    y = oracle.qlinear_levels_from_parts(q, scale, codes, v, 4)
    ref = (q.astype(np.float64) * scale.astype(np.float64)[:, None]) @ oracle.tlq_dequant(codes, p).T
    assert np.allclose(y, ref, rtol=1e-12, atol=0)


def test_linearity_in_the_activation_scale_and_per_channel_locality():
    _, p, codes, q, scale = _case(3, seed=2)
    v = oracle.tlq_level_values(p, 7)
    y = oracle.qlinear_levels_from_parts(q, scale, codes, v, 3)
    assert np.allclose(oracle.qlinear_levels_from_parts(q, 2 * scale, codes, v, 3), 2 * y, rtol=1e-15)
    v2 = v.copy()
    v2[4] *= 3.0                                    # touching channel 4's table moves column 4 only
    y2 = oracle.qlinear_levels_from_parts(q, scale, codes, v2, 3)
    assert np.allclose(y2[:, 4], 3 * y[:, 4], rtol=1e-15)
    assert np.array_equal(np.delete(y2, 4, axis=1), np.delete(y, 4, axis=1))
