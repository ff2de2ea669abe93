"""Pins for the oracle's zero-point activation quantizer (Preliminaries, Eq. 1 as printed)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth


def test_worked_example_by_hand():
    # b = 4: L = 15.  x in [-1, 2]: range 3, s = 0.2, inv = 5, z = round(-1 / 0.2) = -5
    # x_q = clamp(round(5 x) + 5, 0, 15): -1 -> 0, 2 -> 15, 0 -> 5, 0.5 -> round(2.5) = 2 (tie to even) + 5 = 7, 1.3 -> 6.5 -> 6 + 5 = 11
    u = np.array([[-1.0, 2.0, 0.0, 0.5, 1.3]])
    q, s, zero = oracle.quantize_per_token_asym(u, 4, 1.0)
    xq = q.astype(int) + 8
    z = zero.astype(int) - 8
    assert xq.tolist() == [[0, 15, 5, 7, 11]] and z.tolist() == [-5]
    assert s[0] == np.float32(0.2)
    # dequantisation x_f = s (x_q + z)
    assert np.allclose(0.2 * (xq + z), [[-1.0, 2.0, 0.0, 0.4, 1.2]])


@pytest.mark.parametrize("a_bits", [4, 6, 8])
def test_brute_force_eq1_in_exact_rationals(a_bits):
    rng = np.random.default_rng(40 + a_bits)
    u = rng.standard_normal((5, 33)) * 3.0 + rng.standard_normal((5, 1)) * 4.0      # rows with non-zero mean
    q, s, zero = oracle.quantize_per_token_asym(u, a_bits, 1.0)
    L, half = 2 ** a_bits - 1, 2 ** (a_bits - 1)
    for t in range(u.shape[0]):
        xs = [Fraction(float(v)) for v in u[t]]
        rng_t = max(xs) - min(xs)
        zq = min(xs) * L / rng_t                                       # x_min / s with s = range / L, exactly
        z = int(zero[t]) - half
        assert abs(zq - z) <= Fraction(1, 2) + Fraction(1, 10 ** 9)
        for k, x in enumerate(xs):
            target = x * L / rng_t
            near = min(range(int(target) - 2, int(target) + 3), key=lambda c: abs(target - c))
            want = min(max(near - z, 0), L)
            if abs(abs(target - near) - Fraction(1, 2)) > Fraction(1, 10 ** 9):   # away from ties the fp64 decision is the exact one
                assert int(q[t, k]) + half == want


@pytest.mark.parametrize("a_bits", [4, 6, 8])
def test_properties(a_bits):
    rng = np.random.default_rng(50 + a_bits)
    u = rng.standard_normal((12, 200)) * np.exp(rng.standard_normal((12, 1))) + rng.standard_normal((12, 1)) * 5
    q, s, zero = oracle.quantize_per_token_asym(u, a_bits, 1.0)
    L, half = 2 ** a_bits - 1, 2 ** (a_bits - 1)
    xq = q.astype(np.int64) + half
    assert q.dtype == np.int8 and zero.dtype == np.int32 and s.dtype == np.float32
    assert xq.min() >= 0 and xq.max() <= L
    # the extremes take the end codes (up to the rounding of the zero-point), the range is fully used
    assert np.all(xq[np.arange(12), u.argmin(axis=1)] <= 1) and np.all(xq[np.arange(12), u.argmax(axis=1)] >= L - 1)
    # reconstruction within half a step (a full step at the clamped ends)
    rec = s.astype(np.float64)[:, None] * (q.astype(np.float64) + zero[:, None])
    step = (u.max(axis=1) - u.min(axis=1)) / L
    assert np.all(np.abs(rec - u) <= step[:, None] * (1.0 + 1e-6))
    assert np.mean(np.abs(rec - u) <= step[:, None] * 0.5 * (1 + 1e-6)) > 0.97
    # codes are invariant to a power-of-two rescale; the scale follows it
    q2, s2, zero2 = oracle.quantize_per_token_asym(u * 4.0, a_bits, 1.0)
    assert np.array_equal(q, q2) and np.array_equal(zero, zero2) and np.array_equal(s2, s * np.float32(4))
    # the Hadamard normalisation only enters the scale
    q3, s3, zero3 = oracle.quantize_per_token_asym(u, a_bits, np.sqrt(128.0))
    assert np.array_equal(q, q3) and np.array_equal(zero, zero3)
    # a one-sided row wastes no codes on the empty side, unlike the symmetric form
    v = np.abs(u)
    qa, sa, _ = oracle.quantize_per_token_asym(v, a_bits, 1.0)
    qs, ss = oracle.quantize_per_token(v, a_bits, 1.0)
    assert np.all(sa < ss)


def test_constant_rows():
    u = np.array([[3.5] * 8, [0.0] * 8, [-2.0] * 8])
    q, s, zero = oracle.quantize_per_token_asym(u, 8, 1.0)
    rec = s.astype(np.float64)[:, None] * (q.astype(np.float64) + zero[:, None])
    assert np.array_equal(rec, u)
    assert np.all(q == -128)


def test_linear_layer_with_zero_point_equals_fake_quant_product():
    spec = synth.LayerSpec("t", 92, 0, 0, 20, 256, 24, 4, 8, "hadamard", 128, 0.05, 2, 40.0)
    X, W, _, bias = synth.layer_tensors(spec, with_bias=True)
    X = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(X) + np.float32(1.5))          # shifted activations: zero-points matter
    q, s, zero = oracle.ars_rotate_quant_asym(X, 8, "hadamard", 128)
    p = oracle.tlq_calibrate(W, 4, synth.DEFAULT_GRID, synth.DEFAULT_GRID)
    codes = oracle.tlq_encode(W, p)
    lut, wscale = oracle.tlq_lut(p, 7)
    y = oracle.qlinear_from_parts_asym(q, s, zero, codes, lut, wscale, 4, bias)
    xf = s.astype(np.float64)[:, None] * (q.astype(np.float64) + zero[:, None])
    wq = np.take_along_axis(lut.astype(np.float64), codes.astype(np.int64) & 15, axis=1) * wscale.astype(np.float64)[:, None]
    assert np.allclose(y, xf @ wq.T + bias[None, :], rtol=1e-12, atol=1e-12)
    # and the dequantised activations are close to the normalised rotation of x
    u = oracle.rotate_hadamard(oracle.bf16_bits_to_f64(X), 128) / np.sqrt(128.0)
    assert np.linalg.norm(xf - u) / np.linalg.norm(u) < 0.02
    # zero == 2^(b-1) - ... reduces to the symmetric product when the row is symmetric: q + zero carries the same information
    assert zero.shape == (20,)
