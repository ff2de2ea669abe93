"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
Bar: bit-exact packed weight codes and activation codes; relative Frobenius error <= 1e-3 on
outputs (bf16 outputs are compared with the oracle output rounded to bf16, since rounding to 8
significant bits alone costs about 1.5e-3)."""
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


def _acts(M, K, seed, n_salient=4, gain=40.0):
    return synth.make_activations(M, K, (900, seed, 0), 0.05, n_salient, gain)


# ------------------------------------------------------------------ rotate + quantize
@pytest.mark.parametrize("M,K,h,a_bits", [
    (256, 1152, 128, 8),      # config 1
    (37, 1152, 128, 4),       # ragged token count, 4-bit
    (5, 64, 1, 8), (5, 64, 2, 8), (9, 64, 4, 4), (3, 192, 8, 8), (33, 192, 64, 8),
    (70, 1536, 512, 8), (65, 4608, 512, 8), (40, 3072, 1024, 4), (19, 12288, 4096, 8), (3, 16384, 16384, 8),
    (1, 1152, 128, 8),
    (131, 1152, 128, 6), (77, 3072, 1024, 6),     # 6-bit activations (the paper's W4A6 settings)
])
def test_hadamard_rotate_quant_bit_exact(lrq, M, K, h, a_bits):
    print(f"case M={M} K={K} h={h} a={a_bits}", flush=True)
    X = _acts(M, K, K + h + M)
    q_ref, s_ref = oracle.ars_rotate_quant(X, a_bits, "hadamard", h)
    q, s = lrq.ars_rotate_quant(bf16_to_dev(X), lrq.Rotation("hadamard", h), a_bits)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("M,K,a_bits,asym", [
    (600, 12288, 8, False),       # one row per workgroup, 256 workgroups: two or three row groups each, single-round exchange
    (1100, 4096, 4, False),       # two rows per workgroup, two workgroups per CU
    (300, 16384, 8, False),       # LDS has no room for the single round: the two-round persistent form
    (560, 12288, 6, True),        # zero-point form
])
def test_hadamard_4096_persistent_workgroups(lrq, M, K, a_bits, asym):
    """h = 4096 with more row groups than resident workgroups: the kernel walks over row groups, loads the next group's
    data early and (LDS permitting) exchanges the block in a single round with three barriers per group.  Every code and
    scale against the oracle."""
    print(f"case persistent hadamard M={M} K={K} a={a_bits} asym={asym}", flush=True)
    X = _acts(M, K, K + M)
    rot = lrq.Rotation("hadamard", 4096)
    if asym:
        q_ref, s_ref, z_ref = oracle.ars_rotate_quant_asym(X, a_bits, "hadamard", 4096)
        q, s, z = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits, asym=True)
        assert np.array_equal(z.cpu().numpy(), z_ref)
    else:
        q_ref, s_ref = oracle.ars_rotate_quant(X, a_bits, "hadamard", 4096)
        q, s = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    # a second call on the same buffers (stale LDS state must not leak between launches or groups)
    if not asym:
        q2, s2 = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits)
        assert np.array_equal(q2.cpu().numpy(), q_ref) and np.array_equal(s2.cpu().numpy(), s_ref)


def test_rotate_quant_edge_rows(lrq):
    K, h = 1152, 128
    X = oracle.bf16_bits_to_f64(_acts(6, K, 1)).astype(np.float32)
    X[0] = 0.0                                   # all-zero token
    X[1] = 0.0; X[1, 700] = -244.0               # one-hot salient outlier
    X[2, :] = X[2, :] * 2.0 ** -60               # tiny magnitudes
    X[3, ::7] *= 2.0 ** 20                       # wide dynamic range inside a block
    X[4] = 1.0                                   # constant row: all energy in one coefficient per block
    Xb = synth.f32_to_bf16_bits(X)
    for a_bits in (8, 4):
        q_ref, s_ref = oracle.ars_rotate_quant(Xb, a_bits, "hadamard", h)
        q, s = lrq.ars_rotate_quant(bf16_to_dev(Xb), lrq.Rotation("hadamard", h), a_bits)
        assert np.array_equal(q.cpu().numpy(), q_ref)
        assert np.array_equal(s.cpu().numpy(), s_ref)
        assert np.all(q_ref[0] == 0) and s_ref[0] == 0


def test_no_rotation_quant(lrq):
    X = _acts(11, 256, 2)
    q_ref, s_ref = oracle.ars_rotate_quant(X, 8, "none")
    q, s = lrq.ars_rotate_quant(bf16_to_dev(X), lrq.Rotation("none"), 8)
    assert np.array_equal(q.cpu().numpy(), q_ref) and np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("M,K,a_bits", [(70, 128, 8), (130, 256, 4), (64, 1152, 8), (200, 192, 8),
                                        (2, 1152, 4), (8, 192, 8), (1, 3072, 8), (64, 384, 8), (65, 384, 8),      # up to 64 rows: the column-per-thread kernel
                                        (300, 1152, 8), (129, 3072, 6), (257, 2048, 4),
                                        (140, 4224, 8),             # K > 4096: the row of x no longer stays in registers
                                        (16420, 256, 8), (11013, 384, 4)])      # more tiles than workgroups: chained tiles, a cut last row tile
def test_dense_rotate_quant_bit_exact(lrq, M, K, a_bits):
    print(f"case dense M={M} K={K} a={a_bits}", flush=True)
    X = _acts(M, K, 3 + K)
    R = synth.make_rotation(K, (901, K, 0))
    import torch
    q_ref, s_ref = oracle.ars_rotate_quant(X, a_bits, "dense", R_bits=R)
    u_ref = oracle.rotate_dense(oracle.bf16_bits_to_f64(X), oracle.bf16_bits_to_f64(R))
    Rd = bf16_to_dev(R)
    # the evaluation in fp64: codes, scales and the rotated activations themselves (fp64 scratch at the head of the
    # workspace) - same bits as the definition's ascending-k accumulation, i.e. the kernel's summation order is the oracle's
    rot = lrq.Rotation("dense_f64", 0, Rd)
    ws = torch.zeros(lrq.ars_workspace_bytes(M, K, rot, a_bits), dtype=torch.uint8, device="cuda")
    q, s = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits, workspace=ws)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    u = ws[:M * K * 8].view(torch.float64).view(M, K).cpu().numpy()
    assert np.array_equal(u, u_ref)
    # the default evaluation (bf16 matrix cores + error bound + exact recomputation where the bound does not decide;
    # shapes it does not serve fall back to the one above): the same codes and scales
    rot = lrq.Rotation("dense", 0, Rd)
    ws = torch.zeros(lrq.ars_workspace_bytes(M, K, rot, a_bits), dtype=torch.uint8, device="cuda")
    q, s = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits, workspace=ws)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    if M > 64 and K % 128 == 0:
        ut, eps, cnt, whole = (a.cpu().numpy() for a in lrq.ars_dense_diagnostics(ws, M, K))
        err = np.abs(ut.astype(np.float64) - u_ref).max(axis=1)
        assert np.all(err <= eps), f"error bound violated: worst ratio {np.max(err / eps)}"
        print(f"  max |u~ - u| / eps = {np.max(err / np.maximum(eps, 1e-300)):.3f}, undecided fraction "
              f"{cnt.sum() / (M * K):.2e}, whole rows {int(whole.sum())}", flush=True)
        assert whole.sum() == 0 and cnt.sum() < 0.05 * M * K        # the bound decides almost everything on this data


def test_dense_rotation_with_a_prepared_matrix(lrq):
    """lrq_ars_dense_prepare: R's transpose and statistics computed once; calls that carry them give the oracle's codes and
    scales, also through lrq_qlinear, and a K the matrix-core evaluation does not serve is refused."""
    import torch
    M, K, N = 200, 1152, 256
    X = _acts(M, K, 77)
    R = synth.make_rotation(K, (902, K, 0))
    q_ref, s_ref = oracle.ars_rotate_quant(X, 8, "dense", R_bits=R)
    Rd, Xd = bf16_to_dev(R), bf16_to_dev(X)
    prep = lrq.ars_dense_prepare(Rd)
    assert prep.numel() == lrq.lib().lrq_ars_dense_prepared_bytes(K)
    rot = lrq.Rotation("dense", 0, Rd, prepared=prep)
    for _ in range(2):                                  # the prepared buffer is only read: a second call gives the same
        q, s = lrq.ars_rotate_quant(Xd, rot, 8)
        assert np.array_equal(q.cpu().numpy(), q_ref)
        assert np.array_equal(s.cpu().numpy(), s_ref)
    W = synth.make_weights(N, K, (902, 1))
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), 4, 7, gd, gd)
    Y1 = lrq.qlinear(Xd, rot, 8, w, out_dtype=torch.float32)
    Y0 = lrq.qlinear(Xd, lrq.Rotation("dense", 0, Rd), 8, w, out_dtype=torch.float32)
    assert torch.equal(Y0, Y1)
    assert lrq.lib().lrq_ars_dense_prepared_bytes(192) == 0
    with pytest.raises(lrq.LrqError):
        lrq.ars_dense_prepare(bf16_to_dev(synth.make_rotation(192, (902, 192, 0))))


def test_dense_rotation_rows_the_bound_cannot_decide(lrq):
    """Rows built so that the matrix-core evaluation cannot settle them: exact ties on a rounding boundary, rows whose
    rotated values are tiny against their inputs (heavy cancellation), an all-zero row, a single spike, and equal
    maxima - every one must still give the oracle's codes (through the exact recomputation)."""
    import torch
    M, K = 130, 256
    X = oracle.bf16_bits_to_f64(_acts(M, K, 4242)).astype(np.float32)
    R = np.zeros((K, K), np.float32)
    R[np.arange(K), (np.arange(K) * 7 + 3) % K] = 1.0          # a permutation matrix: u holds x's values exactly
    R[5, :] = 0.0; R[5, (5 * 7 + 3) % K] = 0.5
    X[0] = 0.0
    X[1] = 0.0; X[1, 9] = -3.0
    X[2, :] = 1.0                                              # every element is the maximum
    X[3, :] = 0.5; X[3, 0] = 127.0                             # u * inv = 0.5 exactly: ties, rounded to even
    X[4, :] = 2.5; X[4, 1] = 127.0                             # 2.5 -> 2
    X[5, :] = 1.5; X[5, 2] = -127.0
    Xb = synth.f32_to_bf16_bits(X)
    Rb = synth.f32_to_bf16_bits(R)
    for a_bits in (8, 4):
        q_ref, s_ref = oracle.ars_rotate_quant(Xb, a_bits, "dense", R_bits=Rb)
        rot = lrq.Rotation("dense", 0, bf16_to_dev(Rb))
        ws = torch.zeros(lrq.ars_workspace_bytes(M, K, rot, a_bits), dtype=torch.uint8, device="cuda")
        q, s = lrq.ars_rotate_quant(bf16_to_dev(Xb), rot, a_bits, workspace=ws)
        assert np.array_equal(q.cpu().numpy(), q_ref)
        assert np.array_equal(s.cpu().numpy(), s_ref)
        _, _, cnt, whole = (a.cpu().numpy() for a in lrq.ars_dense_diagnostics(ws, M, K))
        assert whole[2] == 1                                   # 256 equal maxima: recomputed as a whole
        if a_bits == 8:
            assert cnt[3] >= K - 1 or whole[3] == 1            # the ties were not decided by the approximation
    # heavy cancellation: R's lower half is its upper half negated and the second half of x repeats the first up to one
    # element that differs in its last bit, so u is 2^-7 of a single product while sum |x| |R| is large: the bound
    # decides nothing and every row is recomputed as a whole
    g = synth.rng_for(913, 1)
    A = oracle.bf16_bits_to_f64(synth.f32_to_bf16_bits(g.standard_normal((K // 2, K)).astype(np.float32)))
    Rb = synth.f32_to_bf16_bits(np.concatenate([A, -A], axis=0).astype(np.float32))
    half = synth.f32_to_bf16_bits(g.standard_normal((M, K // 2)).astype(np.float32))
    other = half.copy()
    other[np.arange(M), np.arange(M) % (K // 2)] ^= 1
    Xb = np.concatenate([half, other], axis=1)
    q_ref, s_ref = oracle.ars_rotate_quant(Xb, 8, "dense", R_bits=Rb)
    rot = lrq.Rotation("dense", 0, bf16_to_dev(Rb))
    ws = torch.zeros(lrq.ars_workspace_bytes(M, K, rot, 8), dtype=torch.uint8, device="cuda")
    q, s = lrq.ars_rotate_quant(bf16_to_dev(Xb), rot, 8, workspace=ws)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    assert np.abs(q_ref).max() == 127 and (q_ref != 0).mean() > 0.5
    _, _, _, whole = (a.cpu().numpy() for a in lrq.ars_dense_diagnostics(ws, M, K))
    assert whole.sum() == M


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_dense_rotation_error_bound_on_mixed_exponents(lrq, seed):
    """Inputs chosen against the rounding model of the matrix instruction rather than for realism: x and a (non-orthogonal) R
    whose entries are +-m 2^e with exponents spread over 2^-12 ... 2^12 inside every 16-k group, so that most addends of an
    instruction are truncated against the largest one and the running sums cancel.  The certified bound must still hold
    for every element, and the codes must still be the oracle's."""
    import torch
    M, K = 160, 512
    g = synth.rng_for(917, seed)
    def mixed(shape):
        m = g.integers(128, 256, size=shape).astype(np.float64)          # 8 significant bits: a bf16 value
        e = g.integers(-12, 13, size=shape).astype(np.float64)
        sgn = g.choice([-1.0, 1.0], size=shape)
        return synth.f32_to_bf16_bits((sgn * m * np.exp2(e - 7)).astype(np.float32))
    Xb, Rb = mixed((M, K)), mixed((K, K))
    if seed == 2:                                       # one operand at a single magnitude: the other's spread alone
        Rb = synth.f32_to_bf16_bits(g.choice([-1.0, 1.0], size=(K, K)).astype(np.float32))
    if seed == 3:
        # per 16-k group one product of magnitude about 1 and fifteen full-mantissa products about 2^-11 of it, same sign:
        # their low bits fall below the alignment cut of the instruction, fifteen times per instruction
        x = np.full((M, K), 255.0 / 128 * 2.0 ** -6)
        r = np.full((K, K), 253.0 / 128 * 2.0 ** -6)
        x[:, ::16] = 1.0
        r[::16, :] = 251.0 / 128
        x[1::2] *= -1.0
        Xb, Rb = synth.f32_to_bf16_bits(x.astype(np.float32)), synth.f32_to_bf16_bits(r.astype(np.float32))
    q_ref, s_ref = oracle.ars_rotate_quant(Xb, 8, "dense", R_bits=Rb)
    u_ref = oracle.rotate_dense(oracle.bf16_bits_to_f64(Xb), oracle.bf16_bits_to_f64(Rb))
    rot = lrq.Rotation("dense", 0, bf16_to_dev(Rb))
    ws = torch.zeros(lrq.ars_workspace_bytes(M, K, rot, 8), dtype=torch.uint8, device="cuda")
    q, s = lrq.ars_rotate_quant(bf16_to_dev(Xb), rot, 8, workspace=ws)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    ut, eps, cnt, whole = (a.cpu().numpy() for a in lrq.ars_dense_diagnostics(ws, M, K))
    err = np.abs(ut.astype(np.float64) - u_ref).max(axis=1)
    print(f"  seed {seed}: max |u~ - u| / eps = {np.max(err / eps):.3f}, whole rows {int(whole.sum())}", flush=True)
    assert np.all(err <= eps), f"error bound violated: worst ratio {np.max(err / eps)}"


@pytest.mark.parametrize("seed", range(10))
def test_dense_rotation_random_shapes(lrq, seed):
    """Seeded random token counts, widths (every multiple of 128 up to 1536: one to twelve pairs of K stages, with and without
    the two-stage tail) and bit-widths through the matrix-core evaluation, with and without a prepared R."""
    g = synth.rng_for(919, seed)
    M, K, a_bits = int(g.integers(65, 520)), 128 * int(g.integers(1, 13)), int(g.choice([4, 6, 8]))
    prepared, asym = bool(g.integers(0, 2)), bool(g.integers(0, 2))
    print(f"case dense random seed={seed} M={M} K={K} a={a_bits} prepared={prepared} asym={asym}", flush=True)
    X = _acts(M, K, 800 + seed)
    if asym:                                            # a non-zero mean, so that the zero-points matter
        X = synth.f32_to_bf16_bits(oracle.bf16_bits_to_f64(X).astype(np.float32) + np.float32(0.5))
    R = synth.make_rotation(K, (919, seed, 1))
    Rd = bf16_to_dev(R)
    rot = lrq.Rotation("dense", 0, Rd, prepared=lrq.ars_dense_prepare(Rd) if prepared else None)
    got = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits, asym=asym)
    ref = oracle.ars_rotate_quant_asym(X, a_bits, "dense", 0, R) if asym else oracle.ars_rotate_quant(X, a_bits, "dense", R_bits=R)
    for a, b in zip(got, ref):
        assert np.array_equal(a.cpu().numpy(), b)


def _blockperm_inputs(lrq, K, B, seed):
    R1 = synth.make_block_rotations(K, B, (903, K, seed), 0)
    R2 = synth.make_block_rotations(K, B, (903, K, seed), 1)
    perm = synth.make_channel_permutation(K, (903, K, seed))
    rot = lrq.Rotation("blockperm", block=B, R1=bf16_to_dev(R1), perm=to_dev(perm), R2=bf16_to_dev(R2))
    return (R1, perm, R2), rot


@pytest.mark.parametrize("M,K,B,a_bits,asym", [(70, 128, 128, 8, False), (130, 256, 128, 4, False),
                                               (200, 1152, 128, 8, False), (129, 768, 256, 8, True),
                                               (1, 384, 128, 4, True), (300, 3072, 128, 8, False)])
def test_blockperm_rotate_quant_bit_exact(lrq, M, K, B, a_bits, asym):
    """Structured outlier-aware rotation X.R1.P.R2 (Method, ARS case equation, second branch)."""
    import torch
    print(f"case blockperm M={M} K={K} B={B} a={a_bits} asym={asym}", flush=True)
    X = _acts(M, K, 5 + K)
    bp, rot = _blockperm_inputs(lrq, K, B, M)
    ws = torch.zeros(lrq.ars_workspace_bytes(M, K, rot, a_bits), dtype=torch.uint8, device="cuda")
    if asym:
        q_ref, s_ref, z_ref = oracle.ars_rotate_quant_asym(X, a_bits, "blockperm", blockperm=bp)
        q, s, z = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits, workspace=ws, asym=True)
        assert np.array_equal(z.cpu().numpy(), z_ref)
    else:
        q_ref, s_ref = oracle.ars_rotate_quant(X, a_bits, "blockperm", blockperm=bp)
        q, s = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits, workspace=ws)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    # the rotated activations themselves (fp64 scratch at the head of the workspace), bit for bit
    u = ws[:M * K * 8].view(torch.float64).view(M, K).cpu().numpy()
    u_ref = oracle.rotate_blockperm(oracle.bf16_bits_to_f64(X), oracle.bf16_bits_to_f64(bp[0]), bp[1],
                                    oracle.bf16_bits_to_f64(bp[2]))
    assert np.array_equal(u, u_ref)


def test_blockperm_qlinear_against_oracle(lrq):
    import torch
    M, K, N, B = 150, 1152, 320, 128
    X = _acts(M, K, 77)
    W = synth.make_weights(N, K, (904, N, K))
    bp, rot = _blockperm_inputs(lrq, K, B, 1)
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), 4, 7, gd, gd)
    Y = lrq.qlinear(bf16_to_dev(X), rot, 8, w, out_dtype=torch.float32)
    p = oracle.tlq_calibrate(W, 4, GRID, GRID)
    lut, wscale = oracle.tlq_lut(p, 7)
    q_ref, s_ref = oracle.ars_rotate_quant(X, 8, "blockperm", blockperm=bp)
    y_ref = oracle.qlinear_from_parts(q_ref, s_ref, oracle.tlq_encode(W, p), lut, wscale, 4)
    assert rel_fro(Y.cpu().numpy(), y_ref) <= 1e-3


@pytest.mark.parametrize("T,K,B,n", [(96, 256, 128, 2), (333, 384, 128, 4), (64, 512, 256, 3)])
def test_greedy_rotation_builder_bit_exact(lrq, T, K, B, n):
    """Greedy block rotations, staggered permutation, second rotation (Method, equation R^i = E R~ Q E):
    every output bit for bit, because both sides sum term by term in the same order."""
    print(f"case builder T={T} K={K} B={B} n={n}", flush=True)
    nb = K // B
    key = (905, T, K)
    X = synth.make_activations(T, K, key, 0.05, 6, 50.0)
    Rt = synth.make_spreading_matrix(B)
    Q1, Q2 = synth.make_step_rotations(nb, n, B, key, 0), synth.make_step_rotations(nb, n, B, key, 1)
    R1_ref, perm_ref, R2_ref = oracle.build_outlier_rotation(oracle.bf16_bits_to_f64(X), B, Rt, Q1, Q2)
    rot = lrq.ars_build_rotation(bf16_to_dev(X), B, to_dev(Rt), to_dev(Q1), to_dev(Q2))
    assert np.array_equal(rot.perm.cpu().numpy(), perm_ref)
    assert np.array_equal(bf16_bits_from_dev(rot.R1), oracle.f64_to_bf16_bits(R1_ref))
    assert np.array_equal(bf16_bits_from_dev(rot.R2), oracle.f64_to_bf16_bits(R2_ref))
    # and the built rotation drives the runtime path
    q_ref, s_ref = oracle.ars_rotate_quant(X, 8, "blockperm", blockperm=(oracle.f64_to_bf16_bits(R1_ref), perm_ref,
                                                                        oracle.f64_to_bf16_bits(R2_ref)))
    q, s = lrq.ars_rotate_quant(bf16_to_dev(X), rot, 8)
    assert np.array_equal(q.cpu().numpy(), q_ref) and np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("M,K", [(8, 64), (300, 1152), (4608, 3072)])
def test_fluctuation_metric(lrq, M, K):
    """J = ||X||_F / sqrt(M K) (Method, Eq. J); the sum order differs from numpy's, so 1e-13 relative."""
    X = synth.make_activations(M, K, (906, M, K), 0.05, 4, 40.0)
    J = float(lrq.fluctuation_metric(bf16_to_dev(X)).cpu()[0])
    J_ref = oracle.fluctuation_J(X)
    assert abs(J - J_ref) <= 1e-13 * J_ref
    assert lrq.ars_select(J, 1.0) == {"hadamard": "hadamard", "outlier-aware": "blockperm"}[oracle.select_rotation(J_ref, 1.0)]
    J2 = float(lrq.fluctuation_metric(bf16_to_dev(X)).cpu()[0])
    assert J2 == J                                       # fixed summation order: same bits on every run


@pytest.mark.parametrize("alpha", [0.5, 0.3])
def test_smoothing_factor(lrq, alpha):
    """Per-channel smoothing factor with migration strength alpha (Experiment, "Implementation Details")."""
    T, N, K = 300, 200, 1152
    X = synth.make_activations(T, K, (907, 0, 0), 0.05, 5, 40.0)
    X[:, 17] = 0                                                     # a dead activation channel: factor 1
    W = synth.make_weights(N, K, (907, 0, 1))
    s_ref, inv_ref = oracle.smoothing_factor(X, W, alpha)
    s, inv, Ws = lrq.smooth_factor(bf16_to_dev(X), to_dev(W), alpha)
    s, inv, Ws = s.cpu().numpy(), inv.cpu().numpy(), Ws.cpu().numpy()
    if alpha == 0.5:                                                 # division and square root: correctly rounded on both sides
        assert np.array_equal(s, s_ref) and np.array_equal(inv, inv_ref)
    else:                                                            # pow comes from two different math libraries
        assert np.allclose(s, s_ref, rtol=2e-7, atol=0) and np.allclose(inv, inv_ref, rtol=2e-7, atol=0)
    assert s[17] == 1.0 and inv[17] == 1.0
    assert np.array_equal(Ws, oracle.smooth_weights(W, s))           # one fp32 multiplication per weight


@pytest.mark.parametrize("M,K,kind,h", [(70, 1152, "hadamard", 128), (130, 4608, "hadamard", 512), (33, 192, "hadamard", 64),
                                        (50, 4096, "hadamard", 4096), (64, 256, "none", 0), (90, 256, "dense", 0),
                                        (75, 192, "dense", 0), (3, 1152, "dense", 0), (140, 384, "blockperm", 128),
                                        (530, 12288, "hadamard", 4096)])      # persistent workgroups, single-round exchange
def test_prescaled_rotate_quant_bit_exact(lrq, M, K, kind, h):
    """The reciprocal smoothing factor multiplied into x ahead of every rotation kind."""
    print(f"case prescale M={M} K={K} {kind} h={h}", flush=True)
    X = _acts(M, K, 11 + K)
    ps = (0.25 + synth.rng_for(908, M, K).random(K) * 3.0).astype(np.float32)
    kw, okw = {}, {}
    if kind == "dense":
        R = synth.make_rotation(K, (908, K, 0))
        kw, okw = dict(R=bf16_to_dev(R)), dict(R_bits=R)
    if kind == "blockperm":
        bp, rot0 = _blockperm_inputs(lrq, K, h, M)
        kw, okw = dict(block=h, R1=rot0.R1, perm=rot0.perm, R2=rot0.R2), dict(blockperm=bp)
    rot = lrq.Rotation(kind, had_block=h if kind == "hadamard" else 0, prescale=to_dev(ps), **kw)
    for a_bits, asym in ((8, False), (4, True)):
        if asym:
            ref = oracle.ars_rotate_quant_asym(X, a_bits, kind, h, prescale=ps, **okw)
        else:
            ref = oracle.ars_rotate_quant(X, a_bits, kind, h, prescale=ps, **okw)
        got = lrq.ars_rotate_quant(bf16_to_dev(X), rot, a_bits, asym=asym)
        for g, r in zip(got, ref):
            assert np.array_equal(g.cpu().numpy(), r)


# ------------------------------------------------------------------ TLQ calibrate + pack
def _check_weight(lrq, W, bits, I=7, alpha=GRID, beta=GRID):
    p = oracle.tlq_calibrate(W, bits, alpha, beta)
    codes = oracle.tlq_encode(W, p)
    lut, wscale = oracle.tlq_lut(p, I)
    w = lrq.tlq_quantize_pack(to_dev(W), bits, I, to_dev(alpha), to_dev(beta))
    assert np.array_equal(w.codes.cpu().numpy(), oracle.pack_codes(codes, bits))          # bit-exact packed codes
    assert np.array_equal(w.z_pos.cpu().numpy(), p.z_pos) and np.array_equal(w.z_neg.cpu().numpy(), p.z_neg)
    assert np.array_equal(w.alpha.cpu().numpy(), p.alpha) and np.array_equal(w.beta.cpu().numpy(), p.beta)
    # scales come out of log2 / division chains evaluated by two different math libraries
    assert np.allclose(w.s_pos.cpu().numpy(), p.s_pos, rtol=1e-14, atol=0)
    assert np.allclose(w.s_neg.cpu().numpy(), p.s_neg, rtol=1e-14, atol=0)
    assert np.array_equal(w.lut.cpu().numpy()[:, :2 ** bits], lut)
    assert np.all(w.lut.cpu().numpy()[:, 2 ** bits:] == 0)
    ws_got = w.wscale.cpu().numpy()
    assert np.all(np.abs(ws_got.view(np.int32) - wscale.view(np.int32)) <= 1)          # at most one fp32 ulp (exp2 of two libraries)
    # the search objective at the chosen factors: same summation order on both sides, log2 / exp2 of two libraries
    assert np.allclose(w.err_pos.cpu().numpy(), p.err_pos, rtol=1e-12, atol=0)
    assert np.allclose(w.err_neg.cpu().numpy(), p.err_neg, rtol=1e-12, atol=0)
    return w, codes, lut, wscale


@pytest.mark.parametrize("N,K,bits,I", [(96, 1152, 4, 7), (40, 1152, 3, 7), (33, 256, 4, 6), (64, 4608, 3, 8),
                                        (17, 12288, 4, -1), (1152, 1152, 4, 7)])
def test_tlq_quantize_pack_bit_exact(lrq, N, K, bits, I):
    print(f"case tlq N={N} K={K} b={bits} I={I}", flush=True)
    W = synth.make_weights(N, K, (902, N, K))
    _check_weight(lrq, W, bits, I)


@pytest.mark.parametrize("N,K,bits", [(64, 1152, 4), (48, 1152, 3), (20, 4608, 4)])
def test_tlq_lower_clip_bit_exact(lrq, N, K, bits):
    """The search with a lower clip factor gamma (extension): codes, zero-points and all three chosen factors."""
    print(f"case tlq clip N={N} K={K} b={bits}", flush=True)
    W = synth.make_weights(N, K, (911, N, K))
    gam = np.arange(1.0, 0.29, -0.05).astype(np.float32)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID, gamma_grid=gam)
    codes = oracle.tlq_encode(W, p)
    lut, wscale = oracle.tlq_lut(p, 7)
    w = lrq.tlq_quantize_pack(to_dev(W), bits, 7, to_dev(GRID), to_dev(GRID), gamma_grid=to_dev(gam))
    assert np.array_equal(w.alpha.cpu().numpy(), p.alpha) and np.array_equal(w.beta.cpu().numpy(), p.beta)
    assert np.array_equal(w.gamma_pos.cpu().numpy(), p.gamma_pos) and np.array_equal(w.gamma_neg.cpu().numpy(), p.gamma_neg)
    assert np.array_equal(w.z_pos.cpu().numpy(), p.z_pos) and np.array_equal(w.z_neg.cpu().numpy(), p.z_neg)
    assert np.allclose(w.s_pos.cpu().numpy(), p.s_pos, rtol=1e-14, atol=0)
    assert np.array_equal(w.codes.cpu().numpy(), oracle.pack_codes(codes, bits))
    assert np.array_equal(w.lut.cpu().numpy()[:, :2 ** bits], lut)
    assert (p.gamma_pos < 1).any()                                   # the clip is actually in use on these weights
    # the grid {1} reproduces the plain entry point bit for bit
    w0 = lrq.tlq_quantize_pack(to_dev(W), bits, 7, to_dev(GRID), to_dev(GRID))
    w1 = lrq.tlq_quantize_pack(to_dev(W), bits, 7, to_dev(GRID), to_dev(GRID), gamma_grid=to_dev(np.array([1.0], np.float32)))
    assert torch_equal(w0.codes, w1.codes) and torch_equal(w0.lut, w1.lut) and torch_equal(w0.s_pos, w1.s_pos)


@pytest.mark.parametrize("N,K,bits", [(70, 192, 4), (48, 128, 3), (33, 64, 4)])
def test_gemm_code_tiling_matches_its_description(lrq, N, K, bits):
    """The GEMM's private copy of the weight codes: units of (32 channels x 64 k) stored [channel tile][K block], 64 slots
    of 16 bytes each; slot 16 kq + c holds k = 16 kq + [0, 16) of channel c (first 8 bytes) and of channel 16 + c (last 8
    bytes) of the tile, one nibble per code, byte j of a dword = code[k + j] | code[k + 4 + j] << 4.  Channels beyond N
    stay zero.  Built here from the oracle's codes."""
    W = synth.make_weights(N, K, (915, N, K))
    codes = oracle.tlq_encode(W, oracle.tlq_calibrate(W, bits, GRID, GRID)).astype(np.int64) & (2 ** bits - 1)
    w = lrq.tlq_quantize_pack(to_dev(W), bits, 7, to_dev(GRID), to_dev(GRID))
    tiles, kblocks = (N + 31) // 32, K // 64
    want = np.zeros((tiles, kblocks, 64, 16), dtype=np.uint8)
    for n in range(N):
        for k0 in range(0, K, 8):                       # one dword: 8 codes
            kb, kq, d = k0 // 64, (k0 % 64) // 16, (k0 % 16) // 8
            for j in range(4):
                want[n // 32, kb, 16 * kq + n % 16, ((n % 32) // 16) * 8 + d * 4 + j] = codes[n, k0 + j] | (codes[n, k0 + 4 + j] << 4)
    got = w.gemm_codes.cpu().numpy()
    assert got.size == want.size == lrq.lib().lrq_tlq_gemm_codes_bytes(N, K, bits)
    assert np.array_equal(got.reshape(want.shape), want)


def torch_equal(a, b):
    import torch
    return torch.equal(a, b)


def test_tlq_degenerate_channels(lrq):
    W = synth.make_weights(8, 128, (903, 0, 0))
    W[0] = 0.0
    W[1] = 0.25
    W[2, :64] = -0.5; W[2, 64:] = 0.0
    W[3] = 0.0; W[3, 0], W[3, 1] = 0.5, -0.125
    W[4] = np.abs(W[4])
    W[5] = -np.abs(W[5])
    for bits in (3, 4):
        _check_weight(lrq, W, bits)
    _check_weight(lrq, W, 4, 7, np.array([1.0], np.float32), np.array([1.0, 1.5], np.float32))
    # equal minima: all positive weights 4.0 are reproduced exactly by several factors; the first grid entry wins
    W[6, :64] = 4.0
    W[6, 64:] = -np.abs(W[6, 64:])
    for grid in ([1.5, 1.25, 2.0], [2.0, 1.5, 1.25]):
        for bits in (3, 4):
            w, *_ = _check_weight(lrq, W, bits, 7, np.array(grid, np.float32), GRID)
            assert float(w.alpha[6]) == grid[0]


# ------------------------------------------------------------------ GEMM + rescale
@pytest.mark.parametrize("M,N,K,w_bits,a_bits", [
    (256, 1152, 1152, 4, 8),      # config 1
    (300, 352, 1152, 4, 8),       # ragged M, N not a multiple of the workgroup tile
    (513, 200, 256, 3, 4),        # N not a multiple of 32, 3-bit weights
    (70, 4608, 128, 4, 4),
    (2, 6912, 1152, 3, 4),        # adaLN-shaped: two tokens (64-row tiles)
    (64, 200, 256, 4, 8),         # the largest M that takes the 64-row tiles, ragged N, exact-accumulator check
    (33, 1152, 4608, 4, 8),       # 64-row tiles, long K loop, half-empty second row tile
])
def test_qgemm_against_oracle(lrq, M, N, K, w_bits, a_bits):
    import torch
    print(f"case qgemm M={M} N={N} K={K} W{w_bits}A{a_bits}", flush=True)
    W = synth.make_weights(N, K, (904, N, K))
    w, codes, lut, wscale = _check_weight(lrq, W, w_bits)
    X = _acts(M, K, 5 + M)
    q, s = oracle.ars_rotate_quant(X, a_bits, "hadamard", synth.default_had_block(K))
    bias = synth.make_bias(N, (904, N, K))
    qd, sd = to_dev(q), to_dev(s)
    y_ref = oracle.qlinear_from_parts(q, s, codes, lut, wscale, w_bits, bias)
    y32 = lrq.qgemm(qd, sd, w, bias=to_dev(bias), out_dtype=torch.float32).cpu().numpy()
    assert rel_fro(y32, y_ref) <= 1e-3
    assert np.allclose(y32, y_ref, rtol=2e-6, atol=1e-6 * np.abs(y_ref).max())            # fp32 epilogue of an exact integer sum
    y_ref_nb = oracle.qlinear_from_parts(q, s, codes, lut, wscale, w_bits)
    y16 = bf16_bits_from_dev(lrq.qgemm(qd, sd, w, out_dtype=torch.bfloat16))
    ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(y_ref_nb))
    assert rel_fro(oracle.bf16_bits_to_f64(y16), ref16) <= 1e-3
    # the integer accumulators themselves: scale = wscale = 1 gives the exact int32 sums in fp32 (|acc| < 2^24 here)
    if K <= 256:
        ones_m, ones_n = torch.ones(M, device=qd.device), w.wscale.clone()
        w.wscale.fill_(1.0)
        acc = lrq.qgemm(qd, ones_m, w, out_dtype=torch.float32).cpu().numpy()
        w.wscale.copy_(ones_n)
        ref_acc = oracle.qlinear_from_parts(q, np.ones(M, np.float32), codes, lut, np.ones(N, np.float32), w_bits)
        assert np.array_equal(acc.astype(np.float64), ref_acc)


@pytest.mark.parametrize("M,N,K,w_bits,a_bits,I", [
    (256, 1152, 1152, 4, 8, 7),   # config 1
    (300, 352, 1152, 4, 8, 7),    # ragged M, N not a multiple of the workgroup tile
    (513, 200, 256, 3, 4, 7),     # N not a multiple of 32, 3-bit weights
    (2, 6912, 1152, 3, 4, 5),     # two tokens, fewer mantissa bits
    (130, 260, 64, 4, 4, 0),      # a single K block, N not a multiple of 8 (scalar stores), levels are powers of two
])
def test_levels_path_against_oracle(lrq, M, N, K, w_bits, a_bits, I):
    """The layer on the levels themselves (bf16 matrix cores): the level table bit for bit, outputs to the fp32
    accumulation of K exact products (relative Frobenius error <= 1e-3 is the stated bar; 1e-5 is what it gives)."""
    import torch
    print(f"case levels M={M} N={N} K={K} W{w_bits}A{a_bits} I={I}", flush=True)
    W = synth.make_weights(N, K, (906, N, K))
    w, codes, _, _ = _check_weight(lrq, W, w_bits, I)
    p = oracle.tlq_calibrate(W, w_bits, GRID, GRID)
    v = oracle.tlq_level_values(p, I)
    lv = w.levels.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(lv[:, :2 ** w_bits], oracle.f64_to_bf16_bits(v))
    assert np.all(lv[:, 2 ** w_bits:] == 0)
    X = _acts(M, K, 7 + M)
    q, s = oracle.ars_rotate_quant(X, a_bits, "hadamard", synth.default_had_block(K))
    bias = synth.make_bias(N, (906, N, K))
    qd, sd = to_dev(q), to_dev(s)
    y_ref = oracle.qlinear_levels_from_parts(q, s, codes, v, w_bits, bias)
    y32 = lrq.qgemm(qd, sd, w, bias=to_dev(bias), out_dtype=torch.float32, levels=True).cpu().numpy()
    assert rel_fro(y32, y_ref) <= 1e-5
    y_ref_nb = oracle.qlinear_levels_from_parts(q, s, codes, v, w_bits)
    y16 = bf16_bits_from_dev(lrq.qgemm(qd, sd, w, out_dtype=torch.bfloat16, levels=True))
    ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(y_ref_nb))
    assert rel_fro(oracle.bf16_bits_to_f64(y16), ref16) <= 1e-3
    # the fused call: same rotation + quantizer in front
    Y = lrq.qlinear(bf16_to_dev(X), lrq.Rotation("hadamard", synth.default_had_block(K)), a_bits, w, bias=to_dev(bias),
                    out_dtype=torch.float32, levels=True).cpu().numpy()
    assert rel_fro(Y, y_ref) <= 1e-5
    # and the int8-table path stays within its table rounding of it
    y_i8 = lrq.qgemm(qd, sd, w, bias=to_dev(bias), out_dtype=torch.float32).cpu().numpy()
    bound = (s.astype(np.float64)[:, None] * np.abs(q.astype(np.float64)).sum(axis=1)[:, None]
             * (w.wscale.cpu().numpy().astype(np.float64)[None, :] / 2))
    assert np.all(np.abs(y_i8 - y32) <= bound * (1 + 1e-3) + 1e-6 * np.abs(y_ref).max())


def test_extreme_shapes(lrq):
    """Smallest and largest shapes the entry points accept."""
    import torch
    gd = to_dev(GRID)
    # one token, eight output channels, one K block
    M, N, K = 1, 8, 64
    X = _acts(M, K, 41)
    W = synth.make_weights(N, K, (909, N, K))
    w = lrq.tlq_quantize_pack(to_dev(W), 4, 7, gd, gd)
    Y = lrq.qlinear(bf16_to_dev(X), lrq.Rotation("hadamard", 64), 8, w, out_dtype=torch.float32)
    ref = oracle.qlinear(X, W, 4, 8, "hadamard", 64, alpha_grid=GRID, beta_grid=GRID)
    assert rel_fro(Y.cpu().numpy(), ref["y"]) <= 1e-3
    # the widest row the rotate kernels take (K = 16384), every block size of the two-pass kernel
    K = 16384
    X = _acts(5, K, 42)
    for h in (16384, 16384 // 4, 2048, 256):
        q_ref, s_ref = oracle.ars_rotate_quant(X, 8, "hadamard", h)
        q, s = lrq.ars_rotate_quant(bf16_to_dev(X), lrq.Rotation("hadamard", h), 8)
        assert np.array_equal(q.cpu().numpy(), q_ref) and np.array_equal(s.cpu().numpy(), s_ref)
    # an all-zero activation matrix: codes and scales are zero, the output is the bias
    M, N, K = 40, 96, 256
    W = synth.make_weights(N, K, (909, N, K))
    w = lrq.tlq_quantize_pack(to_dev(W), 3, 7, gd, gd)
    bias = synth.make_bias(N, (909, N, K))
    Xz = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    Y = lrq.qlinear(Xz, lrq.Rotation("hadamard", 256), 4, w, bias=to_dev(bias), out_dtype=torch.float32)
    assert np.array_equal(Y.cpu().numpy(), np.broadcast_to(bias, (M, N)))


# ------------------------------------------------------------------ fused path
@pytest.mark.parametrize("cfg_case", ["config1", "dense", "w3a4", "w4a6"])
def test_qlinear_end_to_end(lrq, cfg_case):
    import torch
    print(f"case qlinear {cfg_case}", flush=True)
    if cfg_case == "config1":
        spec = synth.config_layers(1)[0]
    elif cfg_case == "dense":
        spec = synth.LayerSpec("d", 905, 0, 0, 150, 256, 96, 4, 8, "dense", 256, 0.05, 4, 40.0)
    elif cfg_case == "w4a6":
        spec = synth.LayerSpec("a6", 907, 0, 0, 201, 1152, 288, 4, 6, "hadamard", 128, 0.05, 8, 40.0)
    else:
        spec = synth.LayerSpec("w3", 906, 0, 0, 333, 1152, 416, 3, 4, "hadamard", 128, 0.05, 8, 40.0)
    X, W, R, bias = synth.layer_tensors(spec, with_bias=True)
    ref = oracle.qlinear(X, W, spec.w_bits, spec.a_bits, spec.rotation, spec.had_block, R, 7, GRID, GRID, bias)
    w = lrq.tlq_quantize_pack(to_dev(W), spec.w_bits, 7, to_dev(GRID), to_dev(GRID))
    rot = lrq.Rotation(spec.rotation, spec.had_block, None if R is None else bf16_to_dev(R))
    assert np.array_equal(w.codes.cpu().numpy(), oracle.pack_codes(ref["codes"], spec.w_bits))
    y = lrq.qlinear(bf16_to_dev(X), rot, spec.a_bits, w, bias=to_dev(bias), out_dtype=torch.float32).cpu().numpy()
    assert rel_fro(y, ref["y"]) <= 1e-3
    y16 = bf16_bits_from_dev(lrq.qlinear(bf16_to_dev(X), rot, spec.a_bits, w, bias=to_dev(bias), out_dtype=torch.bfloat16))
    ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(ref["y"]))
    assert rel_fro(oracle.bf16_bits_to_f64(y16), ref16) <= 1e-3
    # the activation codes inside the fused call are the standalone call's
    q, s = lrq.ars_rotate_quant(bf16_to_dev(X), rot, spec.a_bits)
    assert np.array_equal(q.cpu().numpy(), ref["q"]) and np.array_equal(s.cpu().numpy(), ref["scale"])


# ------------------------------------------------------------------ zero-point form of Eq. 1
@pytest.mark.parametrize("M,K,rotation,h,a_bits", [
    (256, 1152, "hadamard", 128, 8), (37, 1152, "hadamard", 128, 4), (9, 64, "hadamard", 4, 8),
    (70, 1536, "hadamard", 512, 8), (40, 3072, "hadamard", 1024, 4), (19, 12288, "hadamard", 4096, 8),
    (3, 16384, "hadamard", 16384, 8), (11, 256, "none", 0, 8), (70, 128, "dense", 0, 8), (64, 1152, "dense", 0, 4),
    (100, 1152, "hadamard", 128, 6), (30, 4608, "hadamard", 512, 6),
    (300, 1152, "dense", 0, 8), (200, 256, "dense", 0, 4), (129, 3072, "dense", 0, 6),      # the matrix-core evaluation
])
def test_zero_point_rotate_quant_bit_exact(lrq, M, K, rotation, h, a_bits):
    print(f"case asym M={M} K={K} {rotation} h={h} a={a_bits}", flush=True)
    X = oracle.bf16_bits_to_f64(_acts(M, K, 7 + K + M)).astype(np.float32)
    X += np.float32(0.75)                           # non-zero mean: the zero-points matter
    X[0] = 2.5                                      # constant token
    if M > 2:
        X[1] = 0.0                                  # all-zero token
        X[2] = -np.abs(X[2])                        # one-sided token
    Xb = synth.f32_to_bf16_bits(X)
    R = synth.make_rotation(K, (907, K, 0)) if rotation == "dense" else None
    q_ref, s_ref, z_ref = oracle.ars_rotate_quant_asym(Xb, a_bits, rotation, h, R)
    rot = lrq.Rotation(rotation, h, None if R is None else bf16_to_dev(R))
    q, s, z = lrq.ars_rotate_quant(bf16_to_dev(Xb), rot, a_bits, asym=True)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(z.cpu().numpy(), z_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("M,N,K,w_bits,a_bits", [(300, 352, 1152, 4, 8), (513, 200, 256, 3, 4), (256, 1152, 1152, 4, 8)])
def test_zero_point_qlinear_against_oracle(lrq, M, N, K, w_bits, a_bits):
    import torch
    print(f"case asym qlinear M={M} N={N} K={K} W{w_bits}A{a_bits}", flush=True)
    W = synth.make_weights(N, K, (908, N, K))
    w, codes, lut, wscale = _check_weight(lrq, W, w_bits)
    wv = np.take_along_axis(lut.astype(np.int64), codes.astype(np.int64) & (2 ** w_bits - 1), axis=1)
    assert np.array_equal(w.colsum.cpu().numpy(), wv.sum(axis=1).astype(np.int32))          # level sums, exact
    h = synth.default_had_block(K)
    Xb = synth.f32_to_bf16_bits(oracle.bf16_bits_to_f64(_acts(M, K, 9 + M)).astype(np.float32) + np.float32(1.25))
    bias = synth.make_bias(N, (908, N, K))
    q, s, z = oracle.ars_rotate_quant_asym(Xb, a_bits, "hadamard", h)
    y_ref = oracle.qlinear_from_parts_asym(q, s, z, codes, lut, wscale, w_bits, bias)
    rot = lrq.Rotation("hadamard", h)
    y32 = lrq.qlinear(bf16_to_dev(Xb), rot, a_bits, w, bias=to_dev(bias), out_dtype=torch.float32, asym=True).cpu().numpy()
    assert rel_fro(y32, y_ref) <= 1e-3
    assert np.allclose(y32, y_ref, rtol=3e-6, atol=2e-6 * np.abs(y_ref).max())
    y16 = bf16_bits_from_dev(lrq.qlinear(bf16_to_dev(Xb), rot, a_bits, w, bias=to_dev(bias), out_dtype=torch.bfloat16, asym=True))
    ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(y_ref))
    assert rel_fro(oracle.bf16_bits_to_f64(y16), ref16) <= 1e-3
    # the GEMM stage alone on oracle codes
    yg = lrq.qgemm(to_dev(q), to_dev(s), w, bias=to_dev(bias), out_dtype=torch.float32, zero=to_dev(z)).cpu().numpy()
    assert np.allclose(yg, y_ref, rtol=3e-6, atol=2e-6 * np.abs(y_ref).max())


def test_smoke_entry(lrq):
    import __graft_entry__
    __graft_entry__.smoke()


def test_qlinear_replays_from_a_hip_graph(lrq):
    """lrq_qlinear allocates nothing and synchronises nothing, so a captured call replays; every replay is checked
    against the eager result on fresh input contents, with eager work and synchronisation between replays."""
    import torch
    M, K, N = 300, 1152, 352
    gd = to_dev(GRID)
    W = synth.make_weights(N, K, (910, N, K))
    w = lrq.tlq_quantize_pack(to_dev(W), 4, 7, gd, gd)
    rot = lrq.Rotation("hadamard", 128)
    X_static = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    Y_static = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    ws = torch.zeros(lrq.workspace_bytes(M, N, K, rot, 8), dtype=torch.uint8, device="cuda")
    X0 = bf16_to_dev(_acts(M, K, 50))
    X_static.copy_(X0)
    lrq.qlinear(X_static, rot, 8, w, out=Y_static, workspace=ws)          # warm-up outside the capture (one-time set-up)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        lrq.qlinear(X_static, rot, 8, w, out=Y_static, workspace=ws)
    for rep in range(3):
        Xr = bf16_to_dev(_acts(M, K, 51 + rep))
        eager = lrq.qlinear(Xr, rot, 8, w)                                 # eager work between the replays
        torch.cuda.synchronize()
        X_static.copy_(Xr)
        Y_static.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y_static, eager), f"replay {rep} differs from the eager result"


def _random_case(seed):
    g = synth.rng_for(912, seed)
    K = int(g.choice([64, 128, 192, 256, 320, 384, 576, 1152, 2048, 2304]))
    M = int(g.integers(1, 400))
    N = int(g.integers(1, 700))
    w_bits, a_bits = int(g.choice([3, 4])), int(g.choice([4, 8]))
    kinds = ["hadamard", "hadamard", "none", "dense"] + (["blockperm"] if K % 128 == 0 else [])
    kind = str(g.choice(kinds))
    divs = [h for h in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048) if K % h == 0]
    h = int(g.choice(divs))
    return M, N, K, w_bits, a_bits, kind, h, bool(g.integers(0, 2)), bool(g.integers(0, 2)), bool(g.integers(0, 2))


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_end_to_end(lrq, seed):
    """Seeded random shapes, bit-widths, rotation kinds, quantizer forms, pre-scale and output types through
    lrq_qlinear: activation codes bit-exact, outputs within 1e-3 of the oracle."""
    import torch
    M, N, K, w_bits, a_bits, kind, h, asym, pre, fp32 = _random_case(seed)
    print(f"case random seed={seed} M={M} N={N} K={K} W{w_bits}A{a_bits} {kind} h={h} asym={asym} pre={pre} fp32={fp32}", flush=True)
    X = _acts(M, K, 600 + seed)
    W = synth.make_weights(N, K, (912, seed, 1))
    bias = synth.make_bias(N, (912, seed, 2))
    ps = (0.5 + synth.rng_for(912, seed, 3).random(K) * 2.0).astype(np.float32) if pre else None
    kw, okw = {}, {}
    if kind == "dense":
        R = synth.make_rotation(K, (912, seed, 4))
        kw, okw = dict(R=bf16_to_dev(R)), dict(R_bits=R)
    if kind == "blockperm":
        bp, rot0 = _blockperm_inputs(lrq, K, 128, seed)
        kw, okw = dict(block=128, R1=rot0.R1, perm=rot0.perm, R2=rot0.R2), dict(blockperm=bp)
    rot = lrq.Rotation(kind, had_block=h if kind == "hadamard" else 0, prescale=None if ps is None else to_dev(ps), **kw)
    gd = to_dev(GRID)
    w = lrq.tlq_quantize_pack(to_dev(W), w_bits, 7, gd, gd)
    p = oracle.tlq_calibrate(W, w_bits, GRID, GRID)
    codes = oracle.tlq_encode(W, p)
    lut, wscale = oracle.tlq_lut(p, 7)
    Xd = bf16_to_dev(X)
    out_dtype = torch.float32 if fp32 else torch.bfloat16
    Y = lrq.qlinear(Xd, rot, a_bits, w, bias=to_dev(bias), out_dtype=out_dtype, asym=asym)
    got = lrq.ars_rotate_quant(Xd, rot, a_bits, asym=asym)
    if asym:
        q_ref, s_ref, z_ref = oracle.ars_rotate_quant_asym(X, a_bits, kind, h, prescale=ps, **okw)
        assert np.array_equal(got[2].cpu().numpy(), z_ref)
        y_ref = oracle.qlinear_from_parts_asym(q_ref, s_ref, z_ref, codes, lut, wscale, w_bits, bias)
    else:
        q_ref, s_ref = oracle.ars_rotate_quant(X, a_bits, kind, h, prescale=ps, **okw)
        y_ref = oracle.qlinear_from_parts(q_ref, s_ref, codes, lut, wscale, w_bits, bias)
    assert np.array_equal(got[0].cpu().numpy(), q_ref) and np.array_equal(got[1].cpu().numpy(), s_ref)
    if fp32:
        assert rel_fro(Y.cpu().numpy(), y_ref) <= 1e-3
    else:
        ref16 = oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(y_ref))
        assert rel_fro(oracle.bf16_bits_to_f64(bf16_bits_from_dev(Y)), ref16) <= 1e-3
