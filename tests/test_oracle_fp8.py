"""Pins of the oracle's FP8 E4M3 value map ("Hardware Implementation", integerisation with I = 3) - CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth

GRID = synth.DEFAULT_GRID


def _all_finite():
    bits = np.array([b for b in range(256) if (b & 0x7f) != 0x7f], dtype=np.uint8)
    return bits, oracle.e4m3_bits_to_f64(bits)


def test_e4m3_values_from_the_format_definition():
    # sign, 4 exponent bits (bias 7), 3 mantissa bits; subnormals m/8 * 2^-6; no infinities; 0x7f / 0xff are NaN
    v = oracle.e4m3_bits_to_f64(np.array([0x00, 0x01, 0x07, 0x08, 0x38, 0x3c, 0x40, 0x7e, 0x80, 0xb8, 0xfe], dtype=np.uint8))
    assert v.tolist() == [0.0, 2.0 ** -9, 7 * 2.0 ** -9, 2.0 ** -6, 1.0, 1.5, 2.0, 448.0, -0.0, -1.0, -448.0]
    assert np.isnan(oracle.e4m3_bits_to_f64(np.array([0x7f, 0xff], dtype=np.uint8))).all()
    bits, vals = _all_finite()
    for b, x in zip(bits.tolist(), vals.tolist()):          # scalar re-evaluation in exact rationals
        e, m = (b >> 3) & 15, b & 7
        mag = Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
        assert Fraction(x) == (-mag if b & 0x80 else mag)


def test_conversion_is_the_nearest_value_ties_to_even_and_saturates():
    bits, vals = _all_finite()
    assert np.array_equal(oracle.f64_to_e4m3_bits(vals), bits)                  # round trip of every value
    pos = np.sort(vals[bits < 0x80])
    rng = np.random.default_rng(3)
    x = np.abs(rng.standard_normal(4000)) * np.exp2(rng.integers(-13, 10, 4000))
    got = np.abs(oracle.e4m3_bits_to_f64(oracle.f64_to_e4m3_bits(x)))
    for xi, gi in zip(x, got):
        d = np.abs(pos - min(xi, 448.0))
        assert abs(gi - min(xi, 448.0)) == d.min()
    mids = (pos[:-1] + pos[1:]) / 2                                                # exact ties: the even neighbour wins
    tb = oracle.f64_to_e4m3_bits(mids)
    assert np.all(tb % 2 == 0)
    assert np.all((oracle.e4m3_bits_to_f64(tb) == pos[:-1]) | (oracle.e4m3_bits_to_f64(tb) == pos[1:]))
    assert oracle.f64_to_e4m3_bits(np.array([1e9, -1e9, 464.0, 2.0 ** -10, -3 * 2.0 ** -10, -3 * 2.0 ** -11])).tolist() == [0x7e, 0xfe, 0x7e, 0x00, 0x82, 0x81]


@pytest.mark.parametrize("bits", [3, 4])
def test_fp8_level_table(bits):
    W = synth.make_weights(24, 256, (960, bits, 0))
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    lut, wscale = oracle.tlq_lut_fp8(p)
    v = oracle.tlq_level_values(p, 3)
    val = oracle.e4m3_bits_to_f64(lut)
    assert lut.dtype == np.uint8 and lut.shape == v.shape and wscale.dtype == np.float32
    assert np.all(np.log2(wscale.astype(np.float64)) % 1 == 0)                  # a power of two: dividing by it is exact
    top = np.abs(val).max(axis=1)
    assert np.all((top >= 128) & (top < 256))
    scaled = v / wscale.astype(np.float64)[:, None]
    big = np.abs(scaled) >= 2.0 ** -6                                            # E4M3's normal range: four bits fit exactly
    assert big.any() and np.array_equal(val[big], scaled[big])
    assert np.all(np.abs(val - scaled) <= 2.0 ** -10)                             # subnormal spacing 2^-9 below it
    assert np.array_equal(np.sign(val[val != 0]), np.sign(scaled[val != 0]))
    half = 2 ** (bits - 1)
    order = [c & (2 ** bits - 1) for c in range(-half, half)]
    assert np.all(np.diff(val[:, order], axis=1) >= 0)                           # monotone in the signed code


def test_fp8_layer_equals_the_levels_layer_when_nothing_underflows():
    # weights spread over two binades only: every scaled level is an E4M3 normal, so the FP8 layer is the I = 3 levels layer
    rng = np.random.default_rng(11)
    W = (rng.uniform(0.05, 0.2, size=(16, 128)) * rng.choice([-1.0, 1.0], size=(16, 128))).astype(np.float32)
    p = oracle.tlq_calibrate(W, 4, np.array([1.0], np.float32), np.array([1.0], np.float32))
    codes = oracle.tlq_encode(W, p)
    lut, wscale = oracle.tlq_lut_fp8(p)
    q = rng.integers(-7, 8, size=(9, 128)).astype(np.int8)
    scale = rng.random(9).astype(np.float32)
    bias = rng.standard_normal(16).astype(np.float32)
    a = oracle.qlinear_fp8_from_parts(q, scale, codes, lut, wscale, 4, bias)
    b = oracle.qlinear_levels_from_parts(q, scale, codes, oracle.tlq_level_values(p, 3), 4, bias)
    assert np.allclose(a, b, rtol=1e-14, atol=0)
    # the activation codes themselves are E4M3 values
    assert np.array_equal(oracle.e4m3_bits_to_f64(oracle.act_codes_to_e4m3(q)), q.astype(np.float64))
    with pytest.raises(AssertionError):
        oracle.act_codes_to_e4m3(np.array([[9]], dtype=np.int8))
