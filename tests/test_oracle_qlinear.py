"""Pins for the oracle's quantized linear layer and for how throughput is counted."""
import os

import numpy as np
import pytest

import oracle
import synth

GRID = synth.DEFAULT_GRID


def test_ops_are_counted_as_2mnk_like_the_papers_table():
    path = os.path.join(os.path.dirname(__file__), "golden", "gemm_latency_table.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 6
    for M, N, K, _prec, ms, tflops in rows:
        got = 2 * int(M) * int(N) * int(K) / (float(ms) * 1e-3) / 1e12
        assert got == pytest.approx(float(tflops), rel=5e-3)     # times are printed to 3 digits
    spec = synth.config_layers(1)[0]
    assert spec.ops == 2 * 256 * 1152 * 1152


def test_integer_gemm_against_int64_library_matmul():
    rng = np.random.default_rng(0)
    M, N, K, bits = 9, 13, 64, 4
    q = rng.integers(-127, 128, (M, K)).astype(np.int8)
    codes = rng.integers(-8, 8, (N, K)).astype(np.int8)
    lut = rng.integers(-127, 128, (N, 16)).astype(np.int8)
    scale = rng.random(M).astype(np.float32) + 0.5
    wscale = rng.random(N).astype(np.float32) + 0.5
    y = oracle.qlinear_from_parts(q, scale, codes, lut, wscale, bits)
    wv = np.array([[int(lut[n, int(codes[n, k]) & 15]) for k in range(K)] for n in range(N)], dtype=np.int64)
    acc = q.astype(np.int64) @ wv.T
    ref = acc.astype(np.float64) * scale.astype(np.float64)[:, None] * wscale.astype(np.float64)[None, :]
    assert np.allclose(y, ref, rtol=1e-15, atol=0)
    # bias is added per output channel
    b = rng.standard_normal(N).astype(np.float32)
    assert np.allclose(oracle.qlinear_from_parts(q, scale, codes, lut, wscale, bits, b), ref + b[None, :], rtol=1e-14)


def test_identity_table_reduces_to_textbook_int8_gemm():
    rng = np.random.default_rng(1)
    M, N, K = 5, 6, 32
    q = rng.integers(-7, 8, (M, K)).astype(np.int8)
    codes = rng.integers(-8, 8, (N, K)).astype(np.int8)
    lut = np.tile(np.array([(c if c < 8 else c - 16) for c in range(16)], dtype=np.int8), (N, 1))   # lut[c & 15] = c
    one_m, one_n = np.ones(M, np.float32), np.ones(N, np.float32)
    y = oracle.qlinear_from_parts(q, one_m, codes, lut, one_n, 4)
    assert np.array_equal(y, (q.astype(np.int64) @ codes.astype(np.int64).T).astype(np.float64))
    # linear in both scales
    y2 = oracle.qlinear_from_parts(q, one_m * 2, codes, lut, one_n * 0.5, 4)
    assert np.array_equal(y2, y)
    y3 = oracle.qlinear_from_parts(q, one_m * 4, codes, lut, one_n, 4)
    assert np.array_equal(y3, 4 * y)


@pytest.mark.parametrize("w_bits,a_bits", [(4, 8), (3, 4)])
def test_end_to_end_equals_fake_quant_product(w_bits, a_bits):
    # Y must equal (dequantised activations) . (dequantised int8-table weights)^T
    spec = synth.LayerSpec("t", 90, 0, 0, 24, 256, 40, w_bits, a_bits, "hadamard", 128, 0.05, 2, 40.0)
    X, W, _, _ = synth.layer_tensors(spec)
    r = oracle.qlinear(X, W, w_bits, a_bits, "hadamard", 128, alpha_grid=GRID, beta_grid=GRID)
    xq = r["q"].astype(np.float64) * r["scale"].astype(np.float64)[:, None]
    idx = r["codes"].astype(np.int64) & (2 ** w_bits - 1)
    wq = np.take_along_axis(r["lut"].astype(np.float64), idx, axis=1) * r["wscale"].astype(np.float64)[:, None]
    assert np.allclose(r["y"], xq @ wq.T, rtol=1e-12, atol=1e-12)
    # and it approximates the unquantized product in the rotated basis (loose: low-bit log grid)
    ref = oracle.reference_linear(X, W, "hadamard", 128)
    rel = np.linalg.norm(r["y"] - ref) / np.linalg.norm(ref)
    assert rel < (0.35 if w_bits == 4 else 0.6)
    # activation dequantisation alone is tight at 8 bits
    if a_bits == 8:
        u = oracle.rotate_hadamard(oracle.bf16_bits_to_f64(X), 128) / np.sqrt(128.0)
        assert np.linalg.norm(xq - u) / np.linalg.norm(u) < 0.02


def test_dense_rotation_path():
    spec = synth.LayerSpec("t", 91, 0, 0, 8, 64, 16, 4, 8, "dense", 64, 0.05, 2, 40.0)
    X, W, R, _ = synth.layer_tensors(spec)
    q, s = oracle.ars_rotate_quant(X, 8, "dense", R_bits=R)
    u = oracle.bf16_bits_to_f64(X) @ oracle.bf16_bits_to_f64(R)
    assert np.linalg.norm(q * s.astype(np.float64)[:, None] - u) / np.linalg.norm(u) < 0.02
    qn, sn = oracle.ars_rotate_quant(X, 8, "none")
    assert np.abs(qn).max() == 127 and sn.shape == (8,)


def test_synth_generators_are_seeded_and_row_sliceable():
    spec = synth.config_layers(2)[0]
    a = synth.make_activations(spec.M, spec.K, spec.key, spec.p_mild, spec.n_salient, spec.gain, rows=(500, 530))
    b = synth.make_activations(spec.M, spec.K, spec.key, spec.p_mild, spec.n_salient, spec.gain, rows=(250, 600))
    assert np.array_equal(a, b[250:280])
    x = oracle.bf16_bits_to_f64(b)
    ch = synth.salient_channels(spec.K, spec.n_salient, spec.key)
    rms = np.sqrt((x ** 2).mean(axis=0))
    assert rms[ch].min() > 20 and np.median(rms) < 2.5           # salient channels: all tokens, fixed channels
    mask = np.ones(spec.K, bool); mask[ch] = False
    assert 0.01 < (np.abs(x[:, mask]) > 4).mean() < 0.03         # mild outliers are rare
    W = synth.make_weights(64, 1152, spec.key)
    assert W.dtype == np.float32 and np.abs(W).max() < 1.0 and abs(W.mean()) < 1e-3
    kurt = ((W - W.mean()) ** 4).mean() / W.var() ** 2
    assert kurt > 4.0                                            # long tails on both sides
    R = oracle.bf16_bits_to_f64(synth.make_rotation(64, (1, 2, 3)))
    assert np.allclose(R.T @ R, np.eye(64), atol=0.02)


def test_config_tables():
    c = {i: synth.config_layers(i) for i in range(1, 6)}
    assert [(l.M, l.K, l.N) for l in c[2]] == [(8192, 1152, 3456), (8192, 1152, 1152), (8192, 1152, 4608), (8192, 4608, 1152)]
    assert [l.had_block for l in c[2]] == [128, 128, 128, 512]
    assert [l.had_block for l in c[3]] == [1024, 1024, 1024, 4096] and all(l.a_bits == 4 for l in c[3])
    assert sum(l.rotation == "dense" for l in c[4]) == 2 and c[4][3].rotation == "hadamard"
    assert all(l.M == 35100 for l in c[4])
    assert len(c[5]) == 28 * 5 and all(l.w_bits == 3 and l.a_bits == 4 for l in c[5])
    frac = sum(l.rotation == "dense" for l in c[5]) / len(c[5])
    assert 0.02 <= frac <= 0.12
    assert sum(l.ops for l in c[2]) == pytest.approx(261e9, rel=0.01)
