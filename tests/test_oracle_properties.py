"""Property tests of the oracle on generated inputs (hypothesis, CPU): invariants that hold for any input, not only for
the seeded workloads."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
import synth

GRID = synth.DEFAULT_GRID
SET = settings(max_examples=25, deadline=None)


def _rng(seed):
    return np.random.default_rng(seed)


@SET
@given(seed=st.integers(0, 2 ** 31), bits=st.sampled_from([3, 4]), n=st.integers(1, 9), groups=st.integers(1, 12))
def test_pack_unpack_round_trip(seed, bits, n, groups):
    K = 8 * groups
    half = 2 ** (bits - 1)
    codes = _rng(seed).integers(-half, half, (n, K)).astype(np.int8)
    packed = oracle.pack_codes(codes, bits)
    assert packed.shape == (n, K * bits // 8) and packed.dtype == np.uint8
    assert np.array_equal(oracle.unpack_codes(packed, bits, K), codes)


@SET
@given(seed=st.integers(0, 2 ** 31), log2h=st.integers(0, 7), blocks=st.integers(1, 3), m=st.integers(1, 4))
def test_hadamard_applied_twice_is_h_times_the_identity(seed, log2h, blocks, m):
    h = 2 ** log2h
    x = _rng(seed).integers(-1000, 1000, (m, blocks * h)).astype(np.float64)
    twice = oracle.rotate_hadamard(oracle.rotate_hadamard(x, h), h)
    assert np.array_equal(twice, h * x)                       # integers: every butterfly is exact
    # and the transform preserves each block's energy up to the factor h
    u = oracle.rotate_hadamard(x, h)
    assert np.array_equal((u ** 2).reshape(m, blocks, h).sum(-1), h * (x ** 2).reshape(m, blocks, h).sum(-1))


@SET
@given(seed=st.integers(0, 2 ** 31), a_bits=st.sampled_from([4, 6, 8]), k=st.integers(-20, 20), m=st.integers(1, 5),
       K=st.integers(1, 40))
def test_quantizer_codes_do_not_depend_on_a_power_of_two_factor(seed, a_bits, k, m, K):
    u = _rng(seed).standard_normal((m, K)) * 3.0
    q, s = oracle.quantize_per_token(u, a_bits)
    q2, s2 = oracle.quantize_per_token(np.ldexp(u, k), a_bits)
    qmax = 2 ** (a_bits - 1) - 1
    assert np.array_equal(q, q2)
    assert np.array_equal(s2.astype(np.float64), np.ldexp(s.astype(np.float64), k)) or np.any(s == 0)
    assert np.abs(q).max() <= qmax
    top = np.argmax(np.abs(u), axis=1)
    assert np.all(np.abs(q[np.arange(m), top]) == qmax)
    # reconstruction error at most half a step
    amax = np.abs(u).max(axis=1, keepdims=True)
    assert np.all(np.abs(q * (amax / qmax) - u) <= amax / (2 * qmax) * (1 + 1e-12))


@SET
@given(seed=st.integers(0, 2 ** 31), bits=st.sampled_from([3, 4]), n=st.integers(1, 6))
def test_tlq_codes_keep_the_sign_of_the_weight(seed, bits, n):
    g = _rng(seed)
    W = (g.standard_t(4, (n, 64)) * 0.02).astype(np.float32)
    W[g.random((n, 64)) < 0.1] = 0.0
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    codes = oracle.tlq_encode(W, p)
    half = 2 ** (bits - 1)
    assert np.all(codes[W > 0] >= 0) and np.all(codes[W < 0] < 0) and np.all(codes[W == 0] == 0)
    assert codes.min() >= -half and codes.max() <= half - 1
    # decoding gives back the weight's sign, and a second encode of the decoded weights changes nothing
    Wf = oracle.tlq_dequant(codes, p)
    assert np.all(np.sign(Wf[W != 0]) == np.sign(W[W != 0]))
    assert np.array_equal(oracle.tlq_encode(Wf.astype(np.float64), p)[W != 0], codes[W != 0])


@SET
@given(seed=st.integers(0, 2 ** 31), split=st.integers(1, 7))
def test_layer_output_is_additive_over_a_split_of_k(seed, split):
    g = _rng(seed)
    N, K, M, bits = 5, 64, 3, 4
    K1 = 8 * split
    W = (g.standard_t(4, (N, K)) * 0.02).astype(np.float32)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    codes = oracle.tlq_encode(W, p)
    lut, wscale = oracle.tlq_lut(p, 7)
    v = oracle.tlq_level_values(p, 7)
    q = g.integers(-127, 128, (M, K)).astype(np.int8)
    s = (g.random(M) + 0.5).astype(np.float32)
    full = oracle.qlinear_from_parts(q, s, codes, lut, wscale, bits)
    parts = (oracle.qlinear_from_parts(q[:, :K1], s, codes[:, :K1], lut, wscale, bits)
             + oracle.qlinear_from_parts(q[:, K1:], s, codes[:, K1:], lut, wscale, bits))
    assert np.allclose(full, parts, rtol=1e-13, atol=1e-300)
    full_lv = oracle.qlinear_levels_from_parts(q, s, codes, v, bits)
    parts_lv = (oracle.qlinear_levels_from_parts(q[:, :K1], s, codes[:, :K1], v, bits)
                + oracle.qlinear_levels_from_parts(q[:, K1:], s, codes[:, K1:], v, bits))
    assert np.allclose(full_lv, parts_lv, rtol=1e-12, atol=1e-300)
