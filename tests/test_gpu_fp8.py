"""GPU parity of the FP8 E4M3 value map (levels with I = 3 mantissa bits and 4-bit activation codes as E4M3 operands of
v_mfma_f32_32x32x64_f8f6f4): tables and activation bytes bit-exact, outputs to the fp32 accumulation of K exact products
(relative Frobenius error <= 1e-3 is the stated bar; 1e-5 is what it gives)."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import bf16_bits_from_dev, bf16_to_dev, rel_fro, to_dev

pytestmark = pytest.mark.gpu
GRID = synth.DEFAULT_GRID


@pytest.fixture(scope="module")
def lrq():
    import torch
    assert torch.cuda.is_available()
    import paper_2508_03485_amd as m
    m.lib()
    return m


def _acts(M, K, seed):
    return synth.make_activations(M, K, (970, seed, 0), 0.05, 4, 40.0)


@pytest.mark.parametrize("M,K,kind,h", [(256, 1152, "hadamard", 128), (70, 1536, "hadamard", 512), (40, 3072, "hadamard", 1024),
                                        (19, 12288, "hadamard", 4096), (9, 64, "hadamard", 4), (11, 256, "none", 0),
                                        (130, 256, "dense", 0), (300, 1152, "dense", 0)])
def test_rotate_quant_fp8_bit_exact(lrq, M, K, kind, h):
    print(f"case fp8 acts M={M} K={K} {kind} h={h}", flush=True)
    X = _acts(M, K, M + K + h)
    kw, okw = {}, {}
    if kind == "dense":
        R = synth.make_rotation(K, (970, K, 1))
        kw, okw = dict(R=bf16_to_dev(R)), dict(R_bits=R)
    rot = lrq.Rotation(kind, had_block=h if kind == "hadamard" else 0, **kw)
    q_ref, s_ref = oracle.ars_rotate_quant(X, 4, kind, h, **okw)
    q8, s = lrq.ars_rotate_quant_fp8(bf16_to_dev(X), rot)
    assert np.array_equal(q8.cpu().numpy(), oracle.act_codes_to_e4m3(q_ref))
    assert np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("M,N,K,w_bits", [(256, 1152, 1152, 4), (300, 352, 1152, 3), (513, 200, 256, 3), (2, 6912, 1152, 3),
                                          (130, 260, 64, 4), (700, 512, 3072, 4)])
def test_qgemm_fp8_against_oracle(lrq, M, N, K, w_bits):
    import torch
    print(f"case qgemm fp8 M={M} N={N} K={K} W{w_bits}", flush=True)
    W = synth.make_weights(N, K, (971, N, K))
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), w_bits, 7, gd, gd)
    p = oracle.tlq_calibrate(W, w_bits, GRID, GRID)
    codes = oracle.tlq_encode(W, p)
    lut8, ws8 = oracle.tlq_lut_fp8(p)
    assert np.array_equal(w.lut_fp8.cpu().numpy()[:, :2 ** w_bits], lut8)                  # the table itself, bit for bit
    assert np.all(w.lut_fp8.cpu().numpy()[:, 2 ** w_bits:] == 0)
    assert np.array_equal(w.wscale_fp8.cpu().numpy(), ws8)
    X = _acts(M, K, 13 + M)
    q, s = oracle.ars_rotate_quant(X, 4, "hadamard", synth.default_had_block(K))
    bias = synth.make_bias(N, (971, N, K))
    q8d, sd = to_dev(oracle.act_codes_to_e4m3(q)), to_dev(s)
    y_ref = oracle.qlinear_fp8_from_parts(q, s, codes, lut8, ws8, w_bits, bias)
    y32 = lrq.qgemm_fp8(q8d, sd, w, bias=to_dev(bias), out_dtype=torch.float32).cpu().numpy()
    assert rel_fro(y32, y_ref) <= 1e-5
    y_ref_nb = oracle.qlinear_fp8_from_parts(q, s, codes, lut8, ws8, w_bits)
    y16 = bf16_bits_from_dev(lrq.qgemm_fp8(q8d, sd, w, out_dtype=torch.bfloat16))
    ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(y_ref_nb))
    assert rel_fro(oracle.bf16_bits_to_f64(y16), ref16) <= 1e-3
    # the fused call: same rotation + quantizer in front
    Y = lrq.qlinear_fp8(bf16_to_dev(X), lrq.Rotation("hadamard", synth.default_had_block(K)), w, bias=to_dev(bias),
                        out_dtype=torch.float32).cpu().numpy()
    assert rel_fro(Y, y_ref) <= 1e-5
    # and it is the I = 3 levels layer wherever no scaled level falls below E4M3's normal range
    v3 = oracle.tlq_level_values(p, 3)
    y_lev = oracle.qlinear_levels_from_parts(q, s, codes, v3, w_bits, bias)
    lost = np.abs(v3 - oracle.e4m3_bits_to_f64(lut8) * ws8.astype(np.float64)[:, None]).max(axis=1)     # per channel
    bound = s.astype(np.float64)[:, None] * np.abs(q.astype(np.float64)).sum(axis=1)[:, None] * lost[None, :]
    assert np.all(np.abs(y_ref - y_lev) <= bound * (1 + 1e-9) + 1e-12)


@pytest.mark.parametrize("cfg,layer", [(3, 1), (3, 3), (5, 2)])
def test_qlinear_fp8_at_full_size(lrq, cfg, layer):
    import torch
    spec = synth.config_layers(cfg)[layer]
    print(f"fp8 layer {spec.name} cfg{cfg} M={spec.M} K={spec.K} N={spec.N} W{spec.w_bits}A{spec.a_bits} h={spec.had_block}", flush=True)
    assert spec.a_bits == 4 and spec.rotation == "hadamard"
    X, W, _, _ = synth.layer_tensors(spec)
    g = synth.rng_for(972, cfg, layer)
    rows = np.array(sorted(set(g.choice(spec.M, size=40, replace=False).tolist()) | {0, spec.M - 1}))
    chans = np.array(sorted(set(g.choice(spec.N, size=160, replace=False).tolist()) | {0, spec.N - 1}))
    rot = lrq.Rotation("hadamard", spec.had_block)
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), spec.w_bits, 7, gd, gd)
    Y = lrq.qlinear_fp8(bf16_to_dev(X), rot, w, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ridx, cidx = torch.from_numpy(rows).to(Y.device), torch.from_numpy(chans).to(Y.device)
    y_s = Y[ridx][:, cidx].cpu().numpy()
    q_ref, s_ref = oracle.ars_rotate_quant(X[rows], 4, "hadamard", spec.had_block)
    p = oracle.tlq_calibrate(W[chans], spec.w_bits, GRID, GRID)
    codes = oracle.tlq_encode(W[chans], p)
    lut8, ws8 = oracle.tlq_lut_fp8(p)
    assert np.array_equal(w.lut_fp8[cidx].cpu().numpy()[:, :2 ** spec.w_bits], lut8)
    y_ref = oracle.qlinear_fp8_from_parts(q_ref, s_ref, codes, lut8, ws8, spec.w_bits)
    assert rel_fro(y_s, y_ref) <= 1e-5
