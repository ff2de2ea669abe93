"""Pins for the oracle's per-token activation quantizer (Preliminaries, Eq. 1, symmetric form)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def test_worked_example_by_hand():
    # qmax = 127, amax = 2 -> inv = 63.5;  1.0 -> 63.5 -> 64 (tie to even), -0.5 -> -31.75 -> -32,
    # 0.26 -> 16.51 -> 17, 2.0 -> 127
    u = np.array([[1.0, -0.5, 0.26, 2.0]])
    q, s = oracle.quantize_per_token(u, 8, 1.0)
    assert q.tolist() == [[64, -32, 17, 127]]
    assert s[0] == np.float32(2.0 / 127.0)
    # amax = 127 -> inv = 1 exactly: every half-integer is a tie and goes to the even neighbour
    u = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, 63.5, -126.5]])
    q, s = oracle.quantize_per_token(u, 8, 1.0)
    assert q.tolist() == [[127, 0, 2, 2, 0, -2, 64, -126]] and s[0] == np.float32(1.0)
    q4, s4 = oracle.quantize_per_token(np.array([[7.0, -3.5, 2.5, 0.4]]), 4, 1.0)
    assert q4.tolist() == [[7, -4, 2, 0]] and s4[0] == np.float32(1.0)


@pytest.mark.parametrize("a_bits", [4, 6, 8])
def test_brute_force_nearest_grid_point(a_bits):
    rng = np.random.default_rng(a_bits)
    u = rng.standard_normal((6, 40)) * 3.0
    q, s = oracle.quantize_per_token(u, a_bits, 1.0)
    qmax = 2 ** (a_bits - 1) - 1
    for t in range(u.shape[0]):
        amax = max(abs(Fraction(float(v))) for v in u[t])
        for k in range(u.shape[1]):
            target = Fraction(float(u[t, k])) * qmax / amax            # exact rational u * qmax / amax
            best = min(range(-qmax, qmax + 1), key=lambda c: abs(target - c))
            # the fp64 decision may differ from the exact one only at a tie within 1e-12
            if abs(abs(target - best) - Fraction(1, 2)) > Fraction(1, 10 ** 12):
                assert q[t, k] == best


@pytest.mark.parametrize("a_bits", [4, 6, 8])
def test_properties(a_bits):
    rng = np.random.default_rng(20 + a_bits)
    u = rng.standard_normal((16, 257)) * np.exp(rng.standard_normal((16, 1)) * 3)
    qmax = 2 ** (a_bits - 1) - 1
    q, s = oracle.quantize_per_token(u, a_bits, 1.0)
    amax = np.abs(u).max(axis=1)
    assert q.dtype == np.int8 and s.dtype == np.float32
    assert q.min() >= -qmax and q.max() <= qmax
    # reconstruction error bounded by half a step
    assert np.all(np.abs(u - q * (amax / qmax)[:, None]) <= (amax / (2 * qmax))[:, None] * (1 + 1e-12))
    # the absmax element takes +-qmax
    arg = np.abs(u).argmax(axis=1)
    assert np.all(np.abs(q[np.arange(16), arg]) == qmax)
    assert np.all(s > 0) and np.allclose(s, amax / qmax, rtol=1e-7)
    # codes are invariant to a power-of-two rescale, scale follows it; sign symmetry
    q2, s2 = oracle.quantize_per_token(u * 8.0, a_bits, 1.0)
    assert np.array_equal(q, q2) and np.array_equal(s2, s * np.float32(8))
    qn, _ = oracle.quantize_per_token(-u, a_bits, 1.0)
    assert np.array_equal(qn, -q)


def test_hadamard_norm_goes_into_scale_only():
    rng = np.random.default_rng(3)
    u = rng.standard_normal((4, 128))
    q1, s1 = oracle.quantize_per_token(u, 8, 1.0)
    q2, s2 = oracle.quantize_per_token(u, 8, np.sqrt(128.0))
    assert np.array_equal(q1, q2)
    assert np.allclose(s2.astype(np.float64) * np.sqrt(128.0), s1, rtol=1e-6)


def test_zero_row():
    u = np.zeros((2, 16))
    u[1, 3] = -4.0
    q, s = oracle.quantize_per_token(u, 8, 1.0)
    assert np.all(q[0] == 0) and s[0] == 0
    assert q[1, 3] == -127 and np.count_nonzero(q[1]) == 1


def test_rotate_then_quantize_one_hot_closed_form():
    # a single salient outlier alpha e_c: after the Hadamard every |u| = alpha, so every code is +-qmax
    # with the sign pattern of row c, and the scale is alpha / (qmax sqrt(h))  (Lemma, salient outlier case)
    import synth
    h, c = 128, 5
    x = np.zeros((1, h), np.float32)
    x[0, c] = 244.0
    q, s = oracle.ars_rotate_quant(synth.f32_to_bf16_bits(x), 8, "hadamard", h)
    assert np.array_equal(q[0], (127 * oracle.hadamard_matrix(h)[c]).astype(np.int8))
    assert s[0] == np.float32(244.0 / (127.0 * np.sqrt(128.0)))


def test_packed_4bit_codes_hand_example_and_round_trip():
    # codes -7 .. 0 -> nibbles 1 .. 8; byte j = nibble[j] | nibble[4 + j] << 4
    q = np.array([[-7, -6, -5, -4, -3, -2, -1, 0, 7, 0, 1, -1, 2, 3, 4, 5]], dtype=np.int8)
    want = np.array([[0x51, 0x62, 0x73, 0x84, 0xAF, 0xB8, 0xC9, 0xD7]], dtype=np.uint8)
    got = oracle.pack_act_codes4(q)
    assert got.dtype == np.uint8 and np.array_equal(got, want)
    assert np.array_equal(oracle.unpack_act_codes4(want), q)
    rng = np.random.default_rng(5)
    q = rng.integers(-7, 8, size=(9, 64)).astype(np.int8)
    p = oracle.pack_act_codes4(q)
    assert p.shape == (9, 32) and np.array_equal(oracle.unpack_act_codes4(p), q)
    assert ((p & 15) >= 1).all() and ((p >> 4) >= 1).all()           # nibble 0 (code -8) never occurs
    with pytest.raises(AssertionError):
        oracle.pack_act_codes4(np.full((1, 8), -8, dtype=np.int8))     # outside the symmetric 4-bit range
