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
