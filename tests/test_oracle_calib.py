"""Pins for the oracle's fluctuation metric J (Method, Eq. J) and the threshold rule - CPU only."""
import numpy as np

import oracle
import synth


def _bits(a):
    return synth.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_J_of_a_constant_tensor_is_its_magnitude():
    assert oracle.fluctuation_J(_bits(np.full((7, 24), -3.0))) == 3.0


def test_J_of_a_single_spike():
    x = np.zeros((4, 16))
    x[2, 5] = 8.0
    assert oracle.fluctuation_J(_bits(x)) == 8.0 / np.sqrt(64.0)        # = 1.0 exactly


def test_J_is_the_root_mean_square():
    rng = np.random.default_rng(0)
    b = _bits(rng.standard_normal((33, 40)))
    x = oracle.bf16_bits_to_f64(b)
    assert np.isclose(oracle.fluctuation_J(b), np.linalg.norm(x) / np.sqrt(x.size), rtol=1e-14)
    assert np.isclose(oracle.fluctuation_J(b), np.sqrt(np.mean(x ** 2)), rtol=1e-14)


def test_J_scales_linearly_and_ignores_the_token_split():
    rng = np.random.default_rng(1)
    b = _bits(rng.standard_normal((16, 32)))
    x4 = _bits(4.0 * oracle.bf16_bits_to_f64(b))                          # power of two: exact in bf16
    assert np.isclose(oracle.fluctuation_J(x4), 4.0 * oracle.fluctuation_J(b), rtol=1e-15)
    assert np.isclose(oracle.fluctuation_J(b.reshape(2, 8, 32).reshape(16, 32)), oracle.fluctuation_J(b.reshape(64, 8)), rtol=1e-15)


def test_threshold_rule():
    # J below the threshold: Hadamard; at or above: the outlier-aware dual transformation; default threshold 1
    assert oracle.select_rotation(0.999) == "hadamard"
    assert oracle.select_rotation(1.0) == "outlier-aware"
    assert oracle.select_rotation(3.0, threshold=5.0) == "hadamard"


def test_salient_outlier_layers_score_higher():
    mild = synth.make_activations(256, 256, (1, 2, 3), 0.05, 0, 1.0)
    salient = synth.make_activations(256, 256, (1, 2, 3), 0.05, 8, 60.0)
    assert oracle.fluctuation_J(salient) > 2.0 * oracle.fluctuation_J(mild)


# ------------------------------------------------------------------ smoothing factor (migration strength)
def _xw(seed=0, T=64, N=48, K=32):
    X = synth.make_activations(T, K, (7, seed, 0), 0.05, 3, 30.0)
    W = synth.make_weights(N, K, (7, seed, 1))
    return X, W


def test_half_migration_equalises_activation_and_weight_ranges():
    # with alpha = 0.5 both smoothed ranges become sqrt(max|x| max|w|) per channel
    X, W = _xw()
    s, inv = oracle.smoothing_factor(X, W, 0.5)
    a = np.abs(oracle.bf16_bits_to_f64(X)).max(axis=0)
    w = np.abs(W.astype(np.float64)).max(axis=0)
    assert np.allclose(a * inv, np.sqrt(a * w), rtol=1e-6)
    assert np.allclose(w * s, np.sqrt(a * w), rtol=1e-6)
    assert np.allclose(s.astype(np.float64) * inv, 1.0, rtol=3e-7)


def test_migration_extremes():
    X, W = _xw(1)
    a = np.abs(oracle.bf16_bits_to_f64(X)).max(axis=0)
    w = np.abs(W.astype(np.float64)).max(axis=0)
    s1, _ = oracle.smoothing_factor(X, W, 1.0)           # all difficulty to the weights: activations end at range 1
    assert np.allclose(s1, a, rtol=1e-6)
    s0, _ = oracle.smoothing_factor(X, W, 0.0)           # none migrated ... weights end at range 1
    assert np.allclose(s0, 1.0 / w, rtol=1e-6)
    s3, _ = oracle.smoothing_factor(X, W, 0.3)
    assert np.allclose(s3, a ** 0.3 / w ** 0.7, rtol=1e-6)


def test_smoothing_leaves_the_product_unchanged():
    X, W = _xw(2)
    s, inv = oracle.smoothing_factor(X, W, 0.5)
    x = oracle.bf16_bits_to_f64(X)
    y = x @ W.astype(np.float64).T
    y2 = (x * inv.astype(np.float64)) @ oracle.smooth_weights(W, s).astype(np.float64).T
    assert np.allclose(y, y2, rtol=0, atol=1e-5 * np.abs(y).max())


def test_dead_channels_take_factor_one():
    X, W = _xw(3)
    Xz = X.copy()
    Xz[:, 4] = 0
    Wz = W.copy()
    Wz[:, 9] = 0.0
    s, inv = oracle.smoothing_factor(Xz, Wz, 0.5)
    assert s[4] == 1.0 and inv[4] == 1.0 and s[9] == 1.0 and inv[9] == 1.0
    assert np.all(np.isfinite(s)) and np.all(np.isfinite(inv))


def test_prescale_enters_before_the_rotation():
    X, W = _xw(4, K=64)
    _, inv = oracle.smoothing_factor(X, W, 0.5)
    q, sc = oracle.ars_rotate_quant(X, 8, "hadamard", 64, prescale=inv)
    x = oracle.bf16_bits_to_f64(X) * inv.astype(np.float64)
    u = x @ oracle.hadamard_matrix(64)
    back = q.astype(np.float64) * sc.astype(np.float64)[:, None] * 8.0            # sqrt(64)
    assert np.abs(back - u).max() <= 0.51 * (np.abs(u).max(axis=1) / 127.0).max() * 1.0001
    q0, _ = oracle.ars_rotate_quant(X, 8, "hadamard", 64)
    assert not np.array_equal(q, q0)
