"""Pins for the oracle's Twin-Log Quantization (Method, "Twin-Log Quantization for Weights")."""
import math
import os

import numpy as np
import pytest

import oracle
import synth

GRID = synth.DEFAULT_GRID
ONE = np.array([1.0], np.float32)


def _weights(N, K, seed):
    return synth.make_weights(N, K, (77, 0, seed))


@pytest.mark.parametrize("bits", [3, 4])
def test_powers_of_two_are_reproduced_exactly(bits):
    # closed form: positive weights 2^-1 .. 2^-half with alpha = 1 give s+ = 1, z+ = -half and codes
    # half-1 .. 0; negative weights -2^-1 .. -2^-(half+1) give s- = 1, z- = -(half+1), codes -half .. -1
    # (the smallest negative falls on twin level 0 and is clamped up to level 1 under this reading)
    half = 2 ** (bits - 1)
    pos = [2.0 ** -k for k in range(1, half + 1)]
    neg = [-(2.0 ** -k) for k in range(1, half + 2)]
    W = np.array([pos + neg], dtype=np.float32)
    p = oracle.tlq_calibrate(W, bits, ONE, ONE)
    assert p.s_pos[0] == 1.0 and p.z_pos[0] == -half
    assert p.s_neg[0] == 1.0 and p.z_neg[0] == -(half + 1)
    codes = oracle.tlq_encode(W, p)
    assert codes[0, :half].tolist() == list(range(half - 1, -1, -1))
    assert codes[0, half:].tolist() == [-c for c in range(half, 0, -1)] + [-1]
    Wf = oracle.tlq_dequant(codes, p)
    assert np.array_equal(Wf[0, :-1], W[0, :-1].astype(np.float64))
    assert Wf[0, -1] == -(2.0 ** -half)
    # the printed clamp [0, 2^(b-1)] keeps the smallest negative on level 0 of its twin
    p0 = oracle.tlq_calibrate(W, bits, ONE, ONE, neg_lo=0)
    c0 = oracle.tlq_encode(W, p0, neg_lo=0)
    assert c0[0, -1] == 0


@pytest.mark.parametrize("bits", [3, 4])
def test_code_ranges_and_sign_recovers_mask(bits):
    W = _weights(12, 512, bits)
    W[0, :5] = 0.0
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    c = oracle.tlq_encode(W, p)
    half = 2 ** (bits - 1)
    assert c.min() >= -half and c.max() <= half - 1
    assert np.all(c[W > 0] >= 0) and np.all(c[W < 0] < 0) and np.all(c[W == 0] == 0)


@pytest.mark.parametrize("bits", [3, 4])
def test_scale_and_zero_point_closed_forms(bits):
    W = _weights(8, 300, 10 + bits)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    half = 2 ** (bits - 1)
    for n in range(W.shape[0]):
        lp = [math.log2(float(w)) for w in W[n] if w > 0]
        ln = [math.log2(-float(w)) for w in W[n] if w < 0]
        sp = (float(p.alpha[n]) * max(lp) - min(lp)) / (half - 1)
        sn = (float(p.beta[n]) * max(ln) - min(ln)) / half
        assert p.s_pos[n] == pytest.approx(sp, rel=1e-14) and p.s_neg[n] == pytest.approx(sn, rel=1e-14)
        assert p.z_pos[n] == round(min(lp) / sp) and p.z_neg[n] == round(min(ln) / sn)
        assert float(p.alpha[n]) in [float(g) for g in GRID]


@pytest.mark.parametrize("bits", [3, 4])
def test_encode_is_nearest_level_in_log_distance(bits):
    # brute force over the admissible twin levels: the code minimises |log2|w| - s (q + z)|
    W = _weights(4, 96, 20 + bits)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    c = oracle.tlq_encode(W, p)
    half = 2 ** (bits - 1)
    for n in range(W.shape[0]):
        for k in range(W.shape[1]):
            w = float(W[n, k])
            ell = math.log2(abs(w))
            if w > 0:
                cand = [(abs(ell - p.s_pos[n] * (q + int(p.z_pos[n]))), q) for q in range(0, half)]
            else:
                cand = [(abs(ell - p.s_neg[n] * (q + int(p.z_neg[n]))), -q) for q in range(1, half + 1)]
            cand.sort()
            if cand[1][0] - cand[0][0] > 1e-9:                       # skip numerical ties
                assert c[n, k] == cand[0][1]


@pytest.mark.parametrize("bits", [3, 4])
def test_idempotent(bits):
    W = _weights(16, 256, 30 + bits)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    c = oracle.tlq_encode(W, p)
    Wf = oracle.tlq_dequant(c, p)
    assert np.array_equal(oracle.tlq_encode(Wf, p), c)
    assert np.array_equal(np.sign(Wf), np.sign(np.where(W == 0, 1.0, W)))


def _scalar_side_error(ws, factor, n_int, lo, hi):
    """Independent scalar re-evaluation of one clip candidate (plain python floats)."""
    ls = [math.log2(w) for w in ws]
    T = factor * max(ls)
    if not T > min(ls):
        return None
    s = (T - min(ls)) / n_int
    z = round(min(ls) / s)
    err = 0.0
    for w, ell in zip(ws, ls):
        q = min(max(round(ell / s) - z, lo), hi)
        err += (2.0 ** (s * (q + z)) - w) ** 2
    return err


@pytest.mark.parametrize("bits", [3, 4])
def test_search_picks_the_first_minimum_of_the_grid(bits):
    W = _weights(6, 200, 40 + bits)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    half = 2 ** (bits - 1)
    for n in range(W.shape[0]):
        for ws, chosen, n_int, lo, hi in (
                ([float(w) for w in W[n] if w > 0], p.alpha[n], half - 1, 0, half - 1),
                ([-float(w) for w in W[n] if w < 0], p.beta[n], half, 1, half)):
            errs = [(_scalar_side_error(ws, float(g), n_int, lo, hi), float(g)) for g in GRID]
            errs = [(e, g) for e, g in errs if e is not None]
            emin = min(e for e, _ in errs)
            chosen_err = dict((g, e) for e, g in errs)[float(chosen)]
            assert chosen_err <= emin * (1 + 1e-9)
            firsts = [g for e, g in errs if e <= emin * (1 + 1e-9)]
            assert float(chosen) == firsts[0]


@pytest.mark.parametrize("K", [1, 255, 256, 257, 600, 1152])
def test_objective_is_summed_in_its_stated_order(K):
    # 256 interleaved partial sums over ascending k, then partial 0, 1, ..., 255: a scalar loop in that order gives
    # the same bits; values of very different magnitude make any other association visible
    rng = np.random.default_rng(K)
    v = (rng.random((3, K)) * 10.0 ** rng.integers(-12, 4, size=(3, K)))
    got = oracle.tlq._ordered_sum(v)
    for n in range(3):
        part = [0.0] * 256
        for k in range(K):
            part[k % 256] = part[k % 256] + float(v[n, k])
        tot = 0.0
        for j in range(256):
            tot = tot + part[j]
        assert got[n] == tot
    if K >= 600:
        ascending = [sum(float(x) for x in v[n]) for n in range(3)]       # plain left-to-right sum: other bits
        assert any(got[n] != ascending[n] for n in range(3))
        assert np.allclose(got, ascending, rtol=1e-12, atol=0)


def test_reported_objective_is_the_ordered_sum_at_the_chosen_factors():
    W = _weights(4, 600, 77)
    p = oracle.tlq_calibrate(W, 4, GRID, GRID)
    for n in range(4):
        for sel, s, z, lo, hi, want in ((W[n] > 0, p.s_pos[n], p.z_pos[n], 0, 7, p.err_pos[n]),
                                        (W[n] < 0, p.s_neg[n], p.z_neg[n], 1, 8, p.err_neg[n])):
            part = [0.0] * 256
            for k in range(600):
                if sel[k]:
                    w = abs(float(W[n, k]))
                    q = min(max(round(math.log2(w) / s) - int(z), lo), hi)
                    d = 2.0 ** (s * (q + int(z))) - w
                    part[k % 256] = part[k % 256] + d * d
            tot = 0.0
            for j in range(256):
                tot = tot + part[j]
            assert want == pytest.approx(tot, rel=1e-13)       # log2 / exp2 of two libraries; the order is pinned above


def test_equal_minima_keep_the_first_grid_entry():
    # a side whose weights are all 4.0 is reproduced exactly by several clip factors (zero error each):
    # the factor that comes first in the caller's grid order wins
    W = np.full((2, 64), 4.0, dtype=np.float32)
    W[:, 32:] = -np.abs(_weights(2, 32, 99))
    for bits in (3, 4):
        for grid, want in (([1.5, 1.25, 2.0], 1.5), ([2.0, 1.5, 1.25], 2.0), ([1.25, 2.0], 1.25)):
            g = np.array(grid, dtype=np.float32)
            p = oracle.tlq_calibrate(W, bits, g, GRID)
            assert np.all(p.alpha == np.float32(want))
            codes = oracle.tlq_encode(W, p)
            assert np.array_equal(oracle.tlq_dequant(codes, p)[:, :32], W[:, :32].astype(np.float64))


# ------------------------------------------------------------------ lower clip factor gamma (extension)
GAMMAS = np.array([1.0, 0.9, 0.8, 0.7, 0.6, 0.5, 0.4], dtype=np.float32)


def _scalar_side_error_clip(ws, alpha, gamma, n_int, lo, hi):
    ls = [math.log2(w) for w in ws]
    T, B = alpha * max(ls), gamma * min(ls)
    if not T > B:
        return None
    s = (T - B) / n_int
    z = round(B / s)
    err = 0.0
    for w, ell in zip(ws, ls):
        q = min(max(round(ell / s) - z, lo), hi)
        err += (2.0 ** (s * (q + z)) - w) ** 2
    return err


def test_gamma_grid_of_one_is_the_paper_formula():
    W = _weights(6, 300, 71)
    for bits in (3, 4):
        p0 = oracle.tlq_calibrate(W, bits, GRID, GRID)
        p1 = oracle.tlq_calibrate(W, bits, GRID, GRID, gamma_grid=np.array([1.0], np.float32))
        for a, b in ((p0.s_pos, p1.s_pos), (p0.s_neg, p1.s_neg), (p0.z_pos, p1.z_pos), (p0.z_neg, p1.z_neg),
                     (p0.alpha, p1.alpha), (p0.beta, p1.beta)):
            assert np.array_equal(a, b)
        assert np.all(p1.gamma_pos == 1) and np.all(p1.gamma_neg == 1)


@pytest.mark.parametrize("bits", [3, 4])
def test_joint_search_picks_the_first_minimum_alpha_outer_gamma_inner(bits):
    W = _weights(4, 160, 72 + bits)
    grid = GRID[::4]
    p = oracle.tlq_calibrate(W, bits, grid, grid, gamma_grid=GAMMAS)
    half = 2 ** (bits - 1)
    for n in range(W.shape[0]):
        for ws, ca, cg, s_got, z_got, n_int, lo, hi in (
                ([float(w) for w in W[n] if w > 0], p.alpha[n], p.gamma_pos[n], p.s_pos[n], p.z_pos[n], half - 1, 0, half - 1),
                ([-float(w) for w in W[n] if w < 0], p.beta[n], p.gamma_neg[n], p.s_neg[n], p.z_neg[n], half, 1, half)):
            cands = [(_scalar_side_error_clip(ws, float(a), float(g), n_int, lo, hi), float(a), float(g))
                     for a in grid for g in GAMMAS]
            cands = [c for c in cands if c[0] is not None]
            emin = min(c[0] for c in cands)
            first = [c for c in cands if c[0] <= emin * (1 + 1e-9)][0]
            assert (float(ca), float(cg)) == first[1:]
            ls = [math.log2(w) for w in ws]                    # scale and zero-point recomputed from the printed-style formulas
            s_ref = (float(ca) * max(ls) - float(cg) * min(ls)) / n_int
            assert math.isclose(s_got, s_ref, rel_tol=1e-13) and z_got == round(float(cg) * min(ls) / s_ref)


def test_lower_clip_reduces_the_weight_error_and_clamps_small_magnitudes():
    W = synth.make_weights(32, 1152, (7, 7, 7))
    for bits in (3, 4):
        p0 = oracle.tlq_calibrate(W, bits, GRID, GRID)
        p1 = oracle.tlq_calibrate(W, bits, GRID, GRID, gamma_grid=np.arange(1.0, 0.29, -0.05).astype(np.float32))
        e0 = np.linalg.norm(oracle.tlq_dequant(oracle.tlq_encode(W, p0), p0) - W) / np.linalg.norm(W)
        e1 = np.linalg.norm(oracle.tlq_dequant(oracle.tlq_encode(W, p1), p1) - W) / np.linalg.norm(W)
        assert e1 < 0.6 * e0
        codes = oracle.tlq_encode(W, p1)
        n = 0                                                  # weights below the raised lower end take the lowest level
        lim = 2.0 ** (p1.s_pos[n] * p1.z_pos[n])
        small = (W[n] > 0) & (W[n] < lim * 0.5)
        assert small.any() and np.all(codes[n][small] == 0)


def test_alpha_one_is_plain_min_max_log_quantization():
    W = _weights(5, 400, 50)
    p = oracle.tlq_calibrate(W, 4, ONE, ONE)
    e, _ = oracle.tlq_exponents(p)
    for n in range(5):
        lp = np.log2(W[n][W[n] > 0].astype(np.float64))
        ln = np.log2(-W[n][W[n] < 0].astype(np.float64))
        assert abs(e[n, 0] - lp.min()) <= p.s_pos[n] / 2 + 1e-12     # lowest positive level sits at the minimum
        assert abs(e[n, 7] - lp.max()) <= p.s_pos[n] / 2 + 1e-12     # highest at the maximum
        assert abs(e[n, (-8) & 15] - ln.max()) <= p.s_neg[n] / 2 + 1e-12
        assert np.all(p.alpha == 1) and np.all(p.beta == 1)


def test_clipping_never_hurts_and_suppresses_a_long_tail():
    W = _weights(8, 1024, 60)
    e1 = ((oracle.tlq_dequant(oracle.tlq_encode(W, p1 := oracle.tlq_calibrate(W, 3, ONE, ONE)), p1) - W) ** 2).sum(axis=1)
    e2 = ((oracle.tlq_dequant(oracle.tlq_encode(W, p2 := oracle.tlq_calibrate(W, 3, GRID, GRID)), p2) - W) ** 2).sum(axis=1)
    assert np.all(e2 <= e1 * (1 + 1e-12))


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("I", [6, 7, 8])
def test_level_values_and_lut(bits, I):
    W = _weights(32, 512, 70 + bits)
    p = oracle.tlq_calibrate(W, bits, GRID, GRID)
    nlev, half = 2 ** bits, 2 ** (bits - 1)
    order = [c & (nlev - 1) for c in range(-half, half)]             # ascending signed code
    e, sign = oracle.tlq_exponents(p)
    exact = oracle.tlq_level_values(p, -1)
    # exact levels are strictly monotone in the signed code: v(-half) < ... < v(-1) < 0 < v(0) < ... < v(half-1)
    assert np.all(np.diff(exact[:, order], axis=1) > 0)
    assert np.all(exact[:, order[half - 1]] < 0) and np.all(exact[:, order[half]] > 0)
    # I < 0 is Eq. dequant itself
    assert np.allclose(np.abs(exact), np.exp2(e), rtol=1e-15)
    # exponent split: 2^f 2^r = 2^e with r in [0, 1); integer mantissa in [2^I, 2^(I+1)] within half a unit
    v = oracle.tlq_level_values(p, I)
    f = np.floor(e)
    mant = np.abs(v) / np.exp2(f - I)
    assert np.all(mant == np.rint(mant)) and mant.min() >= 2 ** I and mant.max() <= 2 ** (I + 1)
    assert np.all(np.abs(mant * 2.0 ** -I - np.exp2(e - f)) <= 2.0 ** -(I + 1) + 1e-15)
    assert np.all(np.abs(v / exact - 1) <= 2.0 ** -(I + 1) + 1e-12)
    # int8 table: monotone non-decreasing, the largest level is +-127, rounding error within half a unit
    lut, wscale = oracle.tlq_lut(p, I)
    assert lut.dtype == np.int8 and wscale.dtype == np.float32
    assert np.all(np.diff(lut[:, order].astype(int), axis=1) >= 0)
    assert np.all(np.abs(lut).max(axis=1) == 127)
    assert np.all(np.abs(lut * wscale.astype(np.float64)[:, None] - v) <= wscale[:, None] * 0.5 * (1 + 1e-6))


def test_pack_examples_from_fixture():
    path = os.path.join(os.path.dirname(__file__), "golden", "pack_examples.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        bits, codes, hexes = [f.strip() for f in line.split("|")]
        codes = np.array([[int(c) for c in codes.split()]], dtype=np.int8)
        want = np.array([[int(h, 16) for h in hexes.split()]], dtype=np.uint8)
        got = oracle.pack_codes(codes, int(bits))
        assert np.array_equal(got, want)
        assert np.array_equal(oracle.unpack_codes(want, int(bits), codes.shape[1]), codes)
        n += 1
    assert n == 3


@pytest.mark.parametrize("bits", [3, 4])
def test_pack_round_trip(bits):
    rng = np.random.default_rng(bits)
    half = 2 ** (bits - 1)
    c = rng.integers(-half, half, size=(7, 64)).astype(np.int8)
    pk = oracle.pack_codes(c, bits)
    assert pk.shape == (7, 64 * bits // 8) and pk.dtype == np.uint8
    assert np.array_equal(oracle.unpack_codes(pk, bits, 64), c)


def test_degenerate_channels():
    W = np.zeros((4, 16), np.float32)
    W[1, :] = 0.25                      # one value only: zero range, positive side only
    W[2, :8] = -0.5                     # negative side only (+ zeros)
    W[3, 0], W[3, 1] = 0.5, -0.125      # one element per side
    p = oracle.tlq_calibrate(W, 4, GRID, GRID)
    c = oracle.tlq_encode(W, p)
    assert np.all(c[0] == 0)
    assert p.s_pos[1] == 1.0 and p.z_pos[1] == -2 and np.all(c[1] == 0)
    assert p.s_neg[2] == 1.0 and p.z_neg[2] == -1 and np.all(c[2, :8] == -1) and np.all(c[2, 8:] == 0)
    assert p.s_pos[0] == 1.0 and p.z_pos[0] == 0 and p.s_neg[0] == 1.0 and p.z_neg[0] == 0
    assert np.all(np.isfinite(oracle.tlq_lut(p, 7)[1]))
