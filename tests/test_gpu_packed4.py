"""GPU parity of the packed 4-bit activation path (two codes per byte between rotate+quantize and the GEMM): packed
codes bit-exact against the oracle's codes in the oracle's packing, GEMM outputs identical to the unpacked path's."""
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
    return synth.make_activations(M, K, (950, seed, 0), 0.05, 4, 40.0)


@pytest.mark.parametrize("M,K,kind,h", [
    (256, 1152, "hadamard", 128), (37, 1152, "hadamard", 64), (70, 1536, "hadamard", 512), (40, 3072, "hadamard", 1024),
    (19, 12288, "hadamard", 4096), (33, 2048, "hadamard", 2048),         # packed inside the rotate kernels
    (9, 64, "hadamard", 4), (3, 16384, "hadamard", 16384), (11, 256, "none", 0), (5, 48, "none", 0),   # int8 codes, then the packing pass
    (130, 256, "dense", 0), (300, 1152, "dense", 0), (140, 384, "blockperm", 128),
])
def test_rotate_quant_packed4_bit_exact(lrq, M, K, kind, h):
    print(f"case packed4 M={M} K={K} {kind} h={h}", flush=True)
    X = _acts(M, K, M + K + h)
    kw, okw = {}, {}
    if kind == "dense":
        R = synth.make_rotation(K, (950, K, 1))
        kw, okw = dict(R=bf16_to_dev(R)), dict(R_bits=R)
    if kind == "blockperm":
        R1, R2 = synth.make_block_rotations(K, h, (950, K, 2), 0), synth.make_block_rotations(K, h, (950, K, 2), 1)
        perm = synth.make_channel_permutation(K, (950, K, 2))
        kw = dict(block=h, R1=bf16_to_dev(R1), perm=to_dev(perm), R2=bf16_to_dev(R2))
        okw = dict(blockperm=(R1, perm, R2))
    rot = lrq.Rotation(kind, had_block=h if kind == "hadamard" else 0, **kw)
    q_ref, s_ref = oracle.ars_rotate_quant(X, 4, kind, h, **okw)
    q4, s = lrq.ars_rotate_quant_packed4(bf16_to_dev(X), rot)
    assert np.array_equal(q4.cpu().numpy(), oracle.pack_act_codes4(q_ref))
    assert np.array_equal(s.cpu().numpy(), s_ref)


def test_prescaled_rotate_quant_packed4(lrq):
    M, K, h = 90, 1152, 128
    X = _acts(M, K, 7)
    ps = (0.25 + synth.rng_for(951, M, K).random(K) * 3.0).astype(np.float32)
    q_ref, s_ref = oracle.ars_rotate_quant(X, 4, "hadamard", h, prescale=ps)
    q4, s = lrq.ars_rotate_quant_packed4(bf16_to_dev(X), lrq.Rotation("hadamard", h, prescale=to_dev(ps)))
    assert np.array_equal(q4.cpu().numpy(), oracle.pack_act_codes4(q_ref)) and np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("M,N,K,w_bits", [(256, 1152, 1152, 4), (300, 352, 1152, 3), (513, 200, 256, 3), (2, 6912, 1152, 3),
                                          (64, 200, 256, 4), (33, 1152, 4608, 4), (700, 512, 3072, 4)])
def test_qgemm_packed4_equals_the_unpacked_gemm(lrq, M, N, K, w_bits):
    import torch
    print(f"case qgemm packed4 M={M} N={N} K={K} W{w_bits}", flush=True)
    W = synth.make_weights(N, K, (952, N, K))
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), w_bits, 7, gd, gd)
    X = _acts(M, K, 11 + M)
    q, s = oracle.ars_rotate_quant(X, 4, "hadamard", synth.default_had_block(K))
    bias = synth.make_bias(N, (952, N, K))
    qd, q4d, sd = to_dev(q), to_dev(oracle.pack_act_codes4(q)), to_dev(s)
    for dt in (torch.float32, torch.bfloat16):
        y = lrq.qgemm(qd, sd, w, bias=to_dev(bias), out_dtype=dt)
        y4 = lrq.qgemm_packed4(q4d, sd, w, bias=to_dev(bias), out_dtype=dt)
        assert torch.equal(y, y4)
    p = oracle.tlq_calibrate(W, w_bits, GRID, GRID)
    lut, wscale = oracle.tlq_lut(p, 7)
    y_ref = oracle.qlinear_from_parts(q, s, oracle.tlq_encode(W, p), lut, wscale, w_bits, bias)
    y32 = lrq.qgemm_packed4(q4d, sd, w, bias=to_dev(bias), out_dtype=torch.float32).cpu().numpy()
    assert rel_fro(y32, y_ref) <= 1e-3
    assert np.allclose(y32, y_ref, rtol=3e-6, atol=2e-6 * np.abs(y_ref).max())


@pytest.mark.parametrize("cfg,layer", [(3, 1), (3, 3), (5, 0), (5, 4)])
def test_qlinear_packed4_at_full_size(lrq, cfg, layer):
    """The W4A4 / W3A4 workloads through lrq_qlinear_packed4: identical to lrq_qlinear, sampled rows against the oracle."""
    import torch
    spec = synth.config_layers(cfg)[layer]
    print(f"packed4 layer {spec.name} cfg{cfg} M={spec.M} K={spec.K} N={spec.N} W{spec.w_bits}A{spec.a_bits} h={spec.had_block}", flush=True)
    assert spec.a_bits == 4 and spec.rotation == "hadamard"
    X, W, _, _ = synth.layer_tensors(spec)
    rot = lrq.Rotation("hadamard", spec.had_block)
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), spec.w_bits, 7, gd, gd)
    Xd = bf16_to_dev(X)
    Y = lrq.qlinear(Xd, rot, 4, w, out_dtype=torch.bfloat16)
    Y4 = lrq.qlinear_packed4(Xd, rot, w, out_dtype=torch.bfloat16)
    assert torch.equal(Y, Y4)
    q4, sc = lrq.ars_rotate_quant_packed4(Xd, rot)
    g = synth.rng_for(953, cfg, layer)
    rows = np.array(sorted(set(g.choice(spec.M, size=min(24, spec.M), replace=False).tolist()) | {0, spec.M - 1}))
    ridx = torch.from_numpy(rows).to(Xd.device)
    q_ref, s_ref = oracle.ars_rotate_quant(X[rows], 4, "hadamard", spec.had_block)
    assert np.array_equal(q4[ridx].cpu().numpy(), oracle.pack_act_codes4(q_ref))
    assert np.array_equal(sc[ridx].cpu().numpy(), s_ref)
