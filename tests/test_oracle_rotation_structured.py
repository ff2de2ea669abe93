"""Pins for the oracle's structured outlier-aware rotation (Method, "Adaptive Rotation Scheme":
X . R1 . P . R2, greedy rotations R^i = E_c* R~ Q E_c*, staggered permutation P) - CPU only."""
import numpy as np
import pytest
import scipy.linalg

import oracle
import synth
from oracle import rotation as rot


def _rand_blocks(rng, nb, B):
    # bf16-valued, deliberately non-symmetric blocks
    bits = synth.f32_to_bf16_bits(rng.standard_normal((nb, B, B)).astype(np.float32))
    return oracle.bf16_bits_to_f64(bits)


def test_blockdiag_equals_block_diagonal_matrix_product():
    rng = np.random.default_rng(1)
    nb, B, M = 3, 8, 11
    Rb = _rand_blocks(rng, nb, B)
    x = rng.standard_normal((M, nb * B))
    D = scipy.linalg.block_diag(*Rb)
    assert np.allclose(rot.rotate_blockdiag(x, Rb), x @ D, rtol=0, atol=1e-12)


def test_identity_blocks_leave_only_the_permutation():
    rng = np.random.default_rng(2)
    nb, B, M = 4, 8, 5
    K = nb * B
    x = oracle.bf16_bits_to_f64(synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)))
    eye = np.broadcast_to(np.eye(B), (nb, B, B))
    perm = rng.permutation(K)
    assert np.array_equal(rot.rotate_blockperm(x, eye, perm, eye), x[:, perm])


def test_hadamard_blocks_reduce_to_the_hadamard_branch():
    rng = np.random.default_rng(3)
    nb, B, M = 3, 16, 7
    x = rng.integers(-100, 100, size=(M, nb * B)).astype(np.float64)      # integer values: fp32 rounding is exact
    H = np.broadcast_to(rot.hadamard_matrix(B), (nb, B, B))
    eye = np.broadcast_to(np.eye(B), (nb, B, B))
    got = rot.rotate_blockperm(x, H, np.arange(nb * B), eye)
    assert np.array_equal(got, rot.rotate_hadamard(x, B))
    # and as the second rotation
    assert np.array_equal(rot.rotate_blockperm(x, eye, np.arange(nb * B), H), rot.rotate_hadamard(x, B))


def test_equals_the_materialised_dense_product():
    # D = diag(R1) . P . diag(R2) with P[perm[j], j] = 1: catches a transposed block, an inverted permutation
    # and a swapped order of the two rotations
    rng = np.random.default_rng(4)
    nb, B, M = 3, 8, 9
    K = nb * B
    R1, R2 = _rand_blocks(rng, nb, B), _rand_blocks(rng, nb, B)
    perm = rng.permutation(K)
    P = np.zeros((K, K))
    P[perm, np.arange(K)] = 1.0
    D = scipy.linalg.block_diag(*R1) @ P @ scipy.linalg.block_diag(*R2)
    x = oracle.bf16_bits_to_f64(synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)))
    u = rot.rotate_blockperm(x, R1, perm, R2)
    assert np.allclose(u, x @ D, rtol=0, atol=1e-12 * np.abs(x @ D).max())     # fp64 round-off only
    wrong = x @ (scipy.linalg.block_diag(*R1) @ P.T @ scipy.linalg.block_diag(*R2))
    assert not np.allclose(u, wrong, rtol=0, atol=1e-2)


def test_nothing_is_rounded_between_the_two_stages():
    # second stage = identity: the result is the first block product itself, every fp64 bit of it
    rng = np.random.default_rng(5)
    nb, B = 2, 8
    R1 = _rand_blocks(rng, nb, B)
    eye = np.broadcast_to(np.eye(B), (nb, B, B))
    x = oracle.bf16_bits_to_f64(synth.f32_to_bf16_bits(rng.standard_normal((6, nb * B)).astype(np.float32)))
    z = rot.rotate_blockdiag(x, R1)
    u = rot.rotate_blockperm(x, R1, np.arange(nb * B), eye)
    assert np.array_equal(u, z)
    assert not np.array_equal(u, z.astype(np.float32).astype(np.float64))   # a narrower intermediate would show


def test_second_stage_sums_term_by_term_in_ascending_k():
    # scalar re-evaluation of one output: multiply and add rounded separately, k ascending within the block
    rng = np.random.default_rng(8)
    nb, B, M = 2, 8, 3
    K = nb * B
    R1, R2 = _rand_blocks(rng, nb, B), _rand_blocks(rng, nb, B)
    perm = rng.permutation(K)
    x = oracle.bf16_bits_to_f64(synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)))
    u = rot.rotate_blockperm(x, R1, perm, R2)
    for t, j in ((0, 0), (1, 9), (2, 15)):
        g, jj = divmod(j, B)
        acc = 0.0
        for k in range(B):
            src = int(perm[g * B + k])                   # channel of z that lands at position g*B + k
            gs, ks = divmod(src, B)
            zv = 0.0
            for i in range(B):
                zv = zv + float(x[t, gs * B + i]) * float(R1[gs, i, ks])
            acc = acc + zv * float(R2[g, k, jj])
        assert u[t, j] == acc


def test_rejects_a_non_permutation():
    eye = np.broadcast_to(np.eye(4), (2, 4, 4))
    with pytest.raises(AssertionError):
        rot.rotate_blockperm(np.zeros((1, 8)), eye, np.array([0, 1, 2, 3, 4, 5, 6, 6]), eye)


def test_zigzag_hand_example():
    # K = 6, two blocks of three.  Ranks (descending range): ch4, ch0, ch2, ch5, ch3, ch1.
    # first deal, left to right: ch4 -> block 0, ch0 -> block 1; second deal, right to left: ch2 -> block 1, ch5 -> block 0;
    # third deal, left to right: ch3 -> block 0, ch1 -> block 1.
    perm = rot.zigzag_permutation(np.array([5.0, 1.0, 4.0, 2.0, 6.0, 3.0]), 3)
    assert perm.tolist() == [4, 5, 3, 0, 2, 1]


def test_zigzag_deals_every_rank_group_across_all_blocks():
    rng = np.random.default_rng(6)
    K, B = 96, 8
    nb = K // B
    ranges = rng.random(K) * 10
    perm = rot.zigzag_permutation(ranges, B)
    assert sorted(perm.tolist()) == list(range(K))
    rank = np.empty(K, dtype=int)
    rank[np.argsort(-ranges, kind="stable")] = np.arange(K)
    for g in range(nb):
        ranks = rank[perm[g * B:(g + 1) * B]]
        assert sorted((ranks // nb).tolist()) == list(range(B))         # one channel of every rank group
    sums = ranges[perm].reshape(nb, B).sum(axis=1)
    contiguous = ranges.reshape(nb, B).sum(axis=1)
    assert sums.max() - sums.min() < contiguous.max() - contiguous.min()   # blocks are balanced
    # ties keep channel order
    assert rot.zigzag_permutation(np.ones(4), 2).tolist() == [0, 3, 1, 2]


def test_one_greedy_step_spreads_a_single_outlier_evenly():
    # Theoretical Analysis, Lemma: a vector dominated by one outlier has its max norm divided by sqrt(C)
    B, c, alpha = 16, 5, 48.0
    xb = np.zeros((1, B))
    xb[0, c] = alpha
    Rhat, y = rot.greedy_block_rotation(xb, synth.make_spreading_matrix(B), np.eye(B)[None])
    assert np.allclose(np.abs(y), alpha / np.sqrt(B), rtol=1e-14, atol=0)
    assert np.isclose(np.linalg.norm(y), alpha, rtol=1e-14)
    assert np.allclose(xb @ Rhat, y, rtol=0, atol=1e-13)


def test_one_greedy_step_is_the_printed_matrix_product():
    rng = np.random.default_rng(7)
    B, T = 8, 20
    xb = rng.standard_normal((T, B))
    xb[:, 3] *= 25.0
    Rt = synth.make_spreading_matrix(B)
    Q = synth.make_step_rotations(1, 1, B, (9, 9))[0]
    Rhat, y = rot.greedy_block_rotation(xb, Rt, Q)
    E = np.eye(B)
    E[:, [0, 3]] = E[:, [3, 0]]
    assert np.allclose(Rhat, E @ Rt @ Q[0] @ E, rtol=0, atol=1e-14)
    assert np.allclose(y, xb @ Rhat, rtol=0, atol=1e-12)


def test_greedy_product_is_orthogonal_and_consistent_with_the_rotated_data():
    rng = np.random.default_rng(8)
    B, T, n = 16, 64, 6
    xb = rng.standard_normal((T, B))
    xb[:, [2, 11]] *= 40.0
    Rhat, y = rot.greedy_block_rotation(xb, synth.make_spreading_matrix(B), synth.make_step_rotations(1, n, B, (1, 2))[0])
    assert np.allclose(Rhat @ Rhat.T, np.eye(B), rtol=0, atol=1e-13)
    assert np.allclose(y, xb @ Rhat, rtol=0, atol=1e-11)
    assert np.abs(y).max() < 0.7 * np.abs(xb).max()          # two outlier channels in a block of 16


def test_spreading_matrix_properties():
    for B in (8, 12, 128):
        Rt = synth.make_spreading_matrix(B)
        assert np.allclose(Rt @ Rt.T, np.eye(B), atol=1e-14)
        assert np.allclose(Rt[0], 1.0 / np.sqrt(B), rtol=1e-14)


def test_built_rotation_suppresses_salient_channels_and_keeps_the_norm():
    B, nb, T, n = 16, 4, 128, 4
    K = nb * B
    key = (5, 0, 0)
    X = oracle.bf16_bits_to_f64(synth.make_activations(T, K, key, 0.05, 2, 60.0))
    Rt = synth.make_spreading_matrix(B)
    R1, perm, R2 = rot.build_outlier_rotation(X, B, Rt, synth.make_step_rotations(nb, n, B, key, 0),
                                              synth.make_step_rotations(nb, n, B, key, 1))
    assert sorted(perm.tolist()) == list(range(K))
    for R in (R1, R2):
        for g in range(nb):
            assert np.allclose(R[g] @ R[g].T, np.eye(B), rtol=0, atol=2e-2)      # bf16-rounded entries
    u = rot.rotate_blockperm(X, R1, perm, R2)
    assert abs(np.linalg.norm(u) / np.linalg.norm(X) - 1.0) < 1e-2
    assert np.abs(u).max() < 0.5 * np.abs(X).max()
    # bf16-valued outputs
    for R in (R1, R2):
        assert np.array_equal(R, oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(R)))


def test_permutation_ranks_channels_by_max_minus_min_of_the_rotated_calibration_data():
    # identity rotations (R~ = Q = I) leave the data alone, so P must be the staggered dealing of the channels' ranges
    # max - min; a one-sided channel (large values, small spread) must rank by its spread, not by its magnitude
    rng = np.random.default_rng(11)
    B, nb, T = 4, 3, 40
    K = B * nb
    x = rng.standard_normal((T, K))
    x[:, 5] = 50.0 + 0.01 * rng.standard_normal(T)            # |x| large, range tiny
    x[:, 2] *= 9.0                                             # widest range
    eye = np.eye(B)
    Q = np.broadcast_to(eye, (nb, 1, B, B)).copy()
    R1, perm, R2 = rot.build_outlier_rotation(x, B, eye, Q, Q)
    assert np.array_equal(R1, np.broadcast_to(eye, (nb, B, B))) and np.array_equal(R2, R1)
    ranges = x.max(axis=0) - x.min(axis=0)
    assert perm.tolist() == rot.zigzag_permutation(ranges, B).tolist()
    assert perm[0] == 2                                        # the widest channel is dealt first
    assert perm.tolist() != rot.zigzag_permutation(np.abs(x).max(axis=0), B).tolist()
    assert list(perm).index(5) % B == B - 1                    # the one-sided channel lands in the last deal
