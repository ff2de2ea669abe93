"""Pins for the oracle's rotations: Hadamard definition, butterfly vs matrix form, the Lemma's
closed forms, computational invariance (Preliminaries, "Rotation Transformation")."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.linalg

import oracle
import synth


@pytest.mark.parametrize("h", [1, 2, 4, 8, 64, 128, 1024])
def test_hadamard_matches_library_and_is_orthogonal(h):
    H = oracle.hadamard_matrix(h)
    assert np.array_equal(H, scipy.linalg.hadamard(h).astype(np.float64))   # Sylvester construction
    assert np.array_equal(H @ H.T, h * np.eye(h))                           # H H^T = n I
    assert np.array_equal(H, H.T)
    assert set(np.unique(H)) <= {-1.0, 1.0}


def test_hadamard_normalised_h2_is_the_papers():
    H2 = oracle.hadamard_matrix(2) / np.sqrt(2.0)
    assert np.allclose(H2, np.array([[1, 1], [1, -1]]) / np.sqrt(2.0))
    assert np.allclose(H2 @ H2.T, np.eye(2))


@pytest.mark.parametrize("h,K", [(2, 8), (8, 24), (128, 1152), (512, 4608), (4096, 4096)])
def test_butterfly_equals_matrix_form_exactly(h, K):
    rng = np.random.default_rng(h + K)
    x = rng.integers(-255, 256, size=(3, K)).astype(np.float64)          # integer data: every sum exact
    u = oracle.fwht_blocks(x, h)
    H = oracle.hadamard_matrix(h)
    ref = (x.reshape(3, K // h, h) @ H).reshape(3, K)
    assert np.array_equal(u, ref)


def test_butterfly_sign_pattern_by_brute_force_rationals():
    # u[j] = sum_i x[i] (-1)^popcount(i & j), exact rational arithmetic on bf16-valued inputs
    h = 16
    bits = synth.make_activations(2, h, (99, 0, 0), 0.05, 2, 40.0)
    x = oracle.bf16_bits_to_f64(bits)
    u = oracle.fwht_blocks(x, h)
    for t in range(2):
        xs = [Fraction(float(v)) for v in x[t]]
        for j in range(h):
            s = sum(xs[i] * (-1) ** bin(i & j).count("1") for i in range(h))
            assert Fraction(float(u[t, j])) == s


def test_one_hot_outlier_is_spread_evenly():
    # Lemma: a vector dominated by one salient outlier alpha e_c has ||x H/sqrt(C)||_inf = alpha/sqrt(C)
    h, c, alpha = 128, 37, 245.0
    x = np.zeros((1, h))
    x[0, c] = alpha
    u = oracle.fwht_blocks(x, h)
    assert np.array_equal(u[0], alpha * oracle.hadamard_matrix(h)[c])
    assert np.max(np.abs(u / np.sqrt(h))) == pytest.approx(alpha / np.sqrt(h), rel=1e-15)


def test_norm_is_preserved():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((4, 1152))
    for u in (oracle.fwht_blocks(x, 128) / np.sqrt(128.0),):
        assert np.allclose(np.linalg.norm(u, axis=1), np.linalg.norm(x, axis=1), rtol=1e-13)


def test_blocks_are_independent():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 384))
    u = oracle.fwht_blocks(x, 128)
    x2 = x.copy()
    x2[:, 128:256] = 0.0
    u2 = oracle.fwht_blocks(x2, 128)
    assert np.array_equal(u[:, :128], u2[:, :128]) and np.array_equal(u[:, 256:], u2[:, 256:])
    assert np.all(u2[:, 128:256] == 0)


def test_computational_invariance_hadamard():
    # Y = X W^T = (X H)(W H)^T for orthogonal H
    rng = np.random.default_rng(7)
    X, W = rng.standard_normal((5, 256)), rng.standard_normal((9, 256))
    Xh = oracle.rotate_hadamard(X, 128) / np.sqrt(128.0)
    Wh = oracle.rotate_hadamard(W, 128) / np.sqrt(128.0)
    assert np.allclose(Xh @ Wh.T, X @ W.T, rtol=1e-12, atol=1e-12)


def test_dense_rotation_matches_library_matmul_and_invariance():
    rng = np.random.default_rng(8)
    K = 96
    Q, _ = np.linalg.qr(rng.standard_normal((K, K)))
    X, W = rng.standard_normal((7, K)), rng.standard_normal((4, K))
    U = oracle.rotate_dense(X, Q)
    assert np.allclose(U, X @ Q, rtol=1e-13, atol=1e-13)
    assert np.allclose(U @ oracle.rotate_dense(W, Q).T, X @ W.T, rtol=1e-12, atol=1e-12)
    assert np.allclose(np.linalg.norm(U, axis=1), np.linalg.norm(X, axis=1), rtol=1e-13)


def test_dense_rotation_exact_on_integers_and_not_transposed():
    rng = np.random.default_rng(9)
    X = rng.integers(-9, 10, (3, 8)).astype(np.float64)
    R = rng.integers(-9, 10, (8, 8)).astype(np.float64)
    U = oracle.rotate_dense(X, R)
    ref = np.array([[sum(int(X[t, k]) * int(R[k, j]) for k in range(8)) for j in range(8)] for t in range(3)])
    assert np.array_equal(U, ref.astype(np.float64))


def test_bf16_round_trip_against_torch():
    import torch
    rng = np.random.default_rng(10)
    y = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 0.0, 255.5, 256.5 * 2])])
    mine = oracle.f64_to_bf16_bits(y)
    # torch rounds fp32 -> bf16 (RNE); make the fp64 -> fp32 step exact by pre-truncating the inputs to fp32
    y32 = y.astype(np.float32)
    mine32 = oracle.f64_to_bf16_bits(y32.astype(np.float64))
    ref = torch.from_numpy(y32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine32, ref)
    assert np.array_equal(oracle.bf16_bits_to_f64(ref), torch.from_numpy(ref.view(np.int16)).view(torch.bfloat16).double().numpy())
    # ties go to even in a single rounding from fp64
    assert oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(np.array([1.0 + 2.0 ** -8])))[0] == 1.0
    assert oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8])))[0] == 1.0 + 2.0 ** -6
    assert mine.shape == y.shape
    assert np.array_equal(synth.f32_to_bf16_bits(y32), ref)               # the generator's storage cast too
