"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.

The whole layer runs on the GPU (TLQ pack of the full weight matrix, rotate + quantize of every token,
fused lrq_qlinear with bf16 output).  The oracle then recomputes, one by one, a seeded sample of token
rows and output channels - rows are independent under per-token quantization and channels under
per-channel weight quantization, so parity on the sample is exact for those rows / channels:
  * activation codes and scales of the sampled rows: bit-exact;
  * packed weight codes, level tables of the sampled channels: bit-exact;
  * Y on the sampled rows x channels: relative Frobenius error <= 1e-3 against the oracle rounded to bf16.
"""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import bf16_bits_from_dev, bf16_to_dev, rel_fro, to_dev

pytestmark = pytest.mark.gpu
GRID = synth.DEFAULT_GRID
N_ROWS, N_CH = 40, 160


@pytest.fixture(scope="module")
def lrq():
    import torch
    assert torch.cuda.is_available()
    import paper_2508_03485_amd as m
    m.lib()
    return m


def _sample(n, k, key):
    g = synth.rng_for(777, *key, n)
    idx = set(g.choice(n, size=min(k, n), replace=False).tolist()) | {0, n - 1}
    return np.array(sorted(idx))


def _check_layer(lrq, spec):
    import torch
    print(f"layer {spec.name} cfg{spec.config} M={spec.M} K={spec.K} N={spec.N} W{spec.w_bits}A{spec.a_bits} "
          f"{spec.rotation} h={spec.had_block}", flush=True)
    X, W, R, _ = synth.layer_tensors(spec)
    rows, chans = _sample(spec.M, N_ROWS, spec.key), _sample(spec.N, N_CH, spec.key)
    Xd = bf16_to_dev(X)
    rot = lrq.Rotation(spec.rotation, spec.had_block, None if R is None else bf16_to_dev(R))
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), spec.w_bits, 7, gd, gd)
    q, sc = lrq.ars_rotate_quant(Xd, rot, spec.a_bits)
    Y = lrq.qlinear(Xd, rot, spec.a_bits, w, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ridx, cidx = torch.from_numpy(rows).to(Xd.device), torch.from_numpy(chans).to(Xd.device)
    q_s, sc_s = q[ridx].cpu().numpy(), sc[ridx].cpu().numpy()
    y_s = bf16_bits_from_dev(Y[ridx][:, cidx].contiguous())
    codes_s, lut_s = w.codes[cidx].cpu().numpy(), w.lut[cidx].cpu().numpy()
    wscale_s = w.wscale[cidx].cpu().numpy()
    del Xd, q, Y

    q_ref, s_ref = oracle.ars_rotate_quant(X[rows], spec.a_bits, spec.rotation, spec.had_block, R)
    assert np.array_equal(q_s, q_ref), "activation codes differ"
    assert np.array_equal(sc_s, s_ref), "activation scales differ"
    p = oracle.tlq_calibrate(W[chans], spec.w_bits, GRID, GRID)
    codes = oracle.tlq_encode(W[chans], p)
    lut, wscale = oracle.tlq_lut(p, 7)
    assert np.array_equal(codes_s, oracle.pack_codes(codes, spec.w_bits)), "packed weight codes differ"
    assert np.array_equal(lut_s[:, :2 ** spec.w_bits], lut), "level tables differ"
    assert np.all(np.abs(wscale_s.view(np.int32) - wscale.view(np.int32)) <= 1)        # at most one fp32 ulp
    y_ref = oracle.qlinear_from_parts(q_ref, s_ref, codes, lut, wscale, spec.w_bits)
    ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(y_ref))
    err = rel_fro(oracle.bf16_bits_to_f64(y_s), ref16)
    assert err <= 1e-3, f"relative output error {err}"


@pytest.mark.parametrize("cfg,layer", [(2, 0), (2, 1), (2, 2), (2, 3), (3, 0), (3, 1), (3, 2), (3, 3)])
def test_configs_2_and_3(lrq, cfg, layer):
    _check_layer(lrq, synth.config_layers(cfg)[layer])


@pytest.mark.parametrize("layer", [0, 1, 2, 3])
def test_config_4(lrq, layer):
    _check_layer(lrq, synth.config_layers(4)[layer])


def test_config_5_block_and_a_dense_layer(lrq):
    specs = synth.config_layers(5)
    for s in specs[:5]:                       # block 0: qkv, proj, fc1, fc2, adaLN (two tokens)
        _check_layer(lrq, s)
    dense = [s for s in specs if s.rotation == "dense"]
    assert dense, "config 5 has layers above the fluctuation threshold"
    _check_layer(lrq, dense[0])


def test_config_4_weight_codes_in_full(lrq):
    # every channel of the largest weight matrix shape, packed codes compared in full
    spec = synth.config_layers(4)[0]          # 3072 -> 9216
    W = synth.make_weights(spec.N, spec.K, spec.key)
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), spec.w_bits, 7, gd, gd)
    got = w.codes.cpu().numpy()
    p = oracle.tlq_calibrate(W, spec.w_bits, GRID, GRID)
    assert np.array_equal(got, oracle.pack_codes(oracle.tlq_encode(W, p), spec.w_bits))


@pytest.mark.parametrize("cfg,layer", [(2, 3), (4, 1), (3, 3), (4, 0)])
def test_zero_point_form_at_full_size(lrq, cfg, layer):
    """The paper's Eq. 1 quantizer (zero-point per token) through lrq_qlinear_asym at full size, sampled; config 4's first
    layer takes the dense rotation."""
    import torch
    spec = synth.config_layers(cfg)[layer]
    print(f"asym layer {spec.name} cfg{cfg} M={spec.M} K={spec.K} N={spec.N} {spec.rotation} h={spec.had_block}", flush=True)
    X, W, R, _ = synth.layer_tensors(spec)
    rows, chans = _sample(spec.M, N_ROWS, spec.key), _sample(spec.N, N_CH, spec.key)
    Xd = bf16_to_dev(X)
    rot = lrq.Rotation(spec.rotation, spec.had_block, None if R is None else bf16_to_dev(R))
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), spec.w_bits, 7, gd, gd)
    q, sc, zr = lrq.ars_rotate_quant(Xd, rot, spec.a_bits, asym=True)
    Y = lrq.qlinear(Xd, rot, spec.a_bits, w, out_dtype=torch.bfloat16, asym=True)
    torch.cuda.synchronize()
    ridx, cidx = torch.from_numpy(rows).to(Xd.device), torch.from_numpy(chans).to(Xd.device)
    q_ref, s_ref, z_ref = oracle.ars_rotate_quant_asym(X[rows], spec.a_bits, spec.rotation, spec.had_block, R)
    assert np.array_equal(q[ridx].cpu().numpy(), q_ref)
    assert np.array_equal(zr[ridx].cpu().numpy(), z_ref)
    assert np.array_equal(sc[ridx].cpu().numpy(), s_ref)
    p = oracle.tlq_calibrate(W[chans], spec.w_bits, GRID, GRID)
    codes = oracle.tlq_encode(W[chans], p)
    lut, wscale = oracle.tlq_lut(p, 7)
    y_ref = oracle.qlinear_from_parts_asym(q_ref, s_ref, z_ref, codes, lut, wscale, spec.w_bits)
    ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(y_ref))
    y_s = bf16_bits_from_dev(Y[ridx][:, cidx].contiguous())
    assert rel_fro(oracle.bf16_bits_to_f64(y_s), ref16) <= 1e-3


def test_structured_rotation_at_config_4_size(lrq):
    """X.R1.P.R2 with 128-channel blocks on a config-4 layer that takes the outlier-aware branch, sampled rows."""
    import torch
    spec = [s for s in synth.config_layers(4) if s.rotation == "dense"][0]
    B = 128
    print(f"structured layer {spec.name} M={spec.M} K={spec.K} N={spec.N} B={B}", flush=True)
    X = synth.make_activations(spec.M, spec.K, spec.key, spec.p_mild, spec.n_salient, spec.gain)
    R1 = synth.make_block_rotations(spec.K, B, spec.key, 0)
    R2 = synth.make_block_rotations(spec.K, B, spec.key, 1)
    perm = synth.make_channel_permutation(spec.K, spec.key)
    rot = lrq.Rotation("blockperm", block=B, R1=bf16_to_dev(R1), perm=to_dev(perm), R2=bf16_to_dev(R2))
    q, sc = lrq.ars_rotate_quant(bf16_to_dev(X), rot, spec.a_bits)
    torch.cuda.synchronize()
    rows = _sample(spec.M, N_ROWS, spec.key)
    ridx = torch.from_numpy(rows).to(q.device)
    q_ref, s_ref = oracle.ars_rotate_quant(X[rows], spec.a_bits, "blockperm", blockperm=(R1, perm, R2))
    assert np.array_equal(q[ridx].cpu().numpy(), q_ref)
    assert np.array_equal(sc[ridx].cpu().numpy(), s_ref)


@pytest.mark.parametrize("cfg,layer", [(2, 2), (4, 3), (5, 1)])
def test_levels_path_at_full_size(lrq, cfg, layer):
    """lrq_qlinear_levels (the GEMM on the levels themselves, bf16 matrix cores) at full size, sampled rows x channels."""
    import torch
    spec = synth.config_layers(cfg)[layer]
    print(f"levels layer {spec.name} cfg{cfg} M={spec.M} K={spec.K} N={spec.N} W{spec.w_bits}", flush=True)
    X, W, _, _ = synth.layer_tensors(spec)
    rows, chans = _sample(spec.M, N_ROWS, spec.key), _sample(spec.N, N_CH, spec.key)
    rot = lrq.Rotation("hadamard", spec.had_block)
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), spec.w_bits, 7, gd, gd)
    Y = lrq.qlinear(bf16_to_dev(X), rot, spec.a_bits, w, out_dtype=torch.float32, levels=True)
    torch.cuda.synchronize()
    ridx, cidx = torch.from_numpy(rows).to(Y.device), torch.from_numpy(chans).to(Y.device)
    y_s = Y[ridx][:, cidx].cpu().numpy()
    q_ref, s_ref = oracle.ars_rotate_quant(X[rows], spec.a_bits, "hadamard", spec.had_block)
    p = oracle.tlq_calibrate(W[chans], spec.w_bits, GRID, GRID)
    codes = oracle.tlq_encode(W[chans], p)
    v = oracle.tlq_level_values(p, 7)
    lv = w.levels[cidx].view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(lv[:, :2 ** spec.w_bits], oracle.f64_to_bf16_bits(v))
    y_ref = oracle.qlinear_levels_from_parts(q_ref, s_ref, codes, v, spec.w_bits)
    assert rel_fro(y_s, y_ref) <= 1e-5


def test_dense_rotation_whose_last_round_of_tiles_is_sparse(lrq):
    """2100 x 4096: 32 x 17 = 544 tiles of 128 x 128, 32 more than the 512 resident at a time, so the fp64 evaluation
    cuts the last rows (2048 ...) into 64-row tiles; sampled rows from both regions, and the ragged last rows, bit for
    bit - codes, scales and the fp64 rotated activations; the default (matrix-core) evaluation gives the same codes."""
    import torch
    M, K = 2100, 4096
    X = synth.make_activations(M, K, (931, M, K), 0.05, 8, 40.0)
    R = synth.make_rotation(K, (931, K, 0))
    rows = np.array(sorted(set(_sample(M, 24, (931,)).tolist()) | {2047, 2048, 2049, 2099, 2111 % M, 1, 127, 128}))
    q_ref, s_ref = oracle.ars_rotate_quant(X[rows], 8, "dense", R_bits=R)
    Rd, Xd = bf16_to_dev(R), bf16_to_dev(X)
    for kind in ("dense_f64", "dense"):
        rot = lrq.Rotation(kind, 0, Rd)
        ws = torch.zeros(lrq.ars_workspace_bytes(M, K, rot, 8), dtype=torch.uint8, device="cuda")
        q, sc = lrq.ars_rotate_quant(Xd, rot, 8, workspace=ws)
        torch.cuda.synchronize()
        ridx = torch.from_numpy(rows).to(q.device)
        assert np.array_equal(q[ridx].cpu().numpy(), q_ref), kind
        assert np.array_equal(sc[ridx].cpu().numpy(), s_ref), kind
        if kind == "dense_f64":
            u = ws[:M * K * 8].view(torch.float64).view(M, K)[ridx].cpu().numpy()
            assert np.array_equal(u, oracle.rotate_dense(oracle.bf16_bits_to_f64(X[rows]), oracle.bf16_bits_to_f64(R)))


def _config_5_blocks():
    specs = synth.config_layers(5)
    blocks = {}
    for s in specs:
        blocks.setdefault(s.name.split(".")[0], []).append(s)
    return specs, blocks


def test_config_5_dense_layers_and_two_more_blocks(lrq):
    """Every config-5 layer above the fluctuation threshold (among them two-token adaLN calls, which take the fp64
    evaluation, and 8192-token ones, which take the matrix-core one), plus all five layers of a middle and of the
    last block: sampled rows and channels, the bar of _check_layer."""
    specs, blocks = _config_5_blocks()
    dense = [s for s in specs if s.rotation == "dense"]
    assert {s.M for s in dense} >= {2, specs[0].M}, "want both token counts among the dense layers"
    assert len({(s.K, s.N) for s in dense}) >= 4, "want the dense layers to span the shapes of a block"
    names = sorted(blocks, key=lambda b: int(b[1:]))
    picked = dense + blocks[names[len(names) // 2]] + blocks[names[-1]]
    seen = set()
    for s in picked:
        if s.name not in seen:
            seen.add(s.name)
            _check_layer(lrq, s)


@pytest.mark.parametrize("part", [0, 1, 2, 3])
def test_config_5_weight_tables_of_every_layer(lrq, part):
    """All 140 weight matrices of config 5 go through the pack kernel; the packed codes, level tables and channel
    scales of a seeded sample of channels of each are compared (the channels are independent under per-channel TLQ)."""
    import torch
    specs, _ = _config_5_blocks()
    gd = to_dev(GRID)
    mine = specs[part::4]
    print(f"config 5 weight tables, part {part}: {len(mine)} layers", flush=True)
    for s in mine:
        W = synth.make_weights(s.N, s.K, s.key)
        chans = _sample(s.N, 24, s.key)
        w = lrq.tlq_quantize_pack(to_dev(W), s.w_bits, 7, gd, gd)
        cidx = torch.from_numpy(chans).to(w.codes.device)
        codes_s, lut_s, ws_s = w.codes[cidx].cpu().numpy(), w.lut[cidx].cpu().numpy(), w.wscale[cidx].cpu().numpy()
        p = oracle.tlq_calibrate(W[chans], s.w_bits, GRID, GRID)
        assert np.array_equal(codes_s, oracle.pack_codes(oracle.tlq_encode(W[chans], p), s.w_bits)), s.name
        lut, wscale = oracle.tlq_lut(p, 7)
        assert np.array_equal(lut_s[:, :2 ** s.w_bits], lut), s.name
        assert np.all(np.abs(ws_s.view(np.int32) - wscale.view(np.int32)) <= 1), s.name


@pytest.mark.parametrize("which", ["qkv", "fc2", "adaLN"])
def test_config_5_weight_codes_in_full(lrq, which):
    """One W3 matrix of each of three shapes (K -> 3K, 4K -> K, K -> 6K), every channel, packed codes and tables."""
    specs, blocks = _config_5_blocks()
    names = sorted(blocks, key=lambda b: int(b[1:]))
    s = [x for x in blocks[names[len(names) // 3]] if x.name.endswith("." + which)][0]
    print(f"config 5 full weight check {s.name} N={s.N} K={s.K} W{s.w_bits}", flush=True)
    W = synth.make_weights(s.N, s.K, s.key)
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), s.w_bits, 7, gd, gd)
    p = oracle.tlq_calibrate(W, s.w_bits, GRID, GRID)
    assert np.array_equal(w.codes.cpu().numpy(), oracle.pack_codes(oracle.tlq_encode(W, p), s.w_bits))
    lut, wscale = oracle.tlq_lut(p, 7)
    assert np.array_equal(w.lut.cpu().numpy()[:, :2 ** s.w_bits], lut)
    assert np.all(np.abs(w.wscale.cpu().numpy().view(np.int32) - wscale.view(np.int32)) <= 1)
