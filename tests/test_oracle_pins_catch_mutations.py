"""The pins are only worth something if a plausible mistake in the oracle breaks one of them.  Each case below plants one
mistake in the oracle (on the CPU, by swapping a function for a wrong copy), re-runs the pins that are supposed to guard
that function, and requires at least one of them to fail.  CPU only."""
import importlib
import pkgutil

import numpy as np
import pytest

import oracle
import oracle.actquant
import oracle.bf16
import oracle.calib
import oracle.fp8
import oracle.rotation
import oracle.tlq
import test_oracle_actquant as t_act
import test_oracle_actquant_asym as t_asym
import test_oracle_calib as t_cal
import test_oracle_fp8 as t_fp8
import test_oracle_levels as t_lev
import test_oracle_qlinear as t_ql
import test_oracle_rotation as t_rot
import test_oracle_rotation_structured as t_str
import test_oracle_tlq as t_tlq

_qlinear_mod = importlib.import_module("oracle.qlinear")      # the package re-exports a function of the same name
_MODULES = [oracle] + [importlib.import_module("oracle." + m.name) for m in pkgutil.iter_modules(oracle.__path__)]


def _plant(monkeypatch, original, wrong):
    """Replace `original` by `wrong` in every oracle module that holds a reference to it."""
    hit = 0
    for mod in _MODULES:
        for name, val in list(vars(mod).items()):
            if val is original:
                monkeypatch.setattr(mod, name, wrong)
                hit += 1
    assert hit, "nothing to replace"


def _some_pin_fails(pins):
    failed = 0
    for fn, args in pins:
        try:
            fn(*args)
        except Exception:        # an assertion, or the wrong function tripping over its own output
            failed += 1
    return failed > 0


# ---- wrong copies -------------------------------------------------------------------------------------------------
def _fwht_swapped_outputs(x, h):
    x = np.asarray(x, dtype=np.float64)
    K = x.shape[-1]
    lead = x.shape[:-1]
    u = x.reshape(*lead, K // h, h).copy()
    s = 1
    while s < h:
        v = u.reshape(*lead, K // h, h // (2 * s), 2, s)
        a, b = v[..., 0, :].copy(), v[..., 1, :].copy()
        v[..., 0, :] = a - b                       # (a - b, a + b) instead of (a + b, a - b)
        v[..., 1, :] = a + b
        s *= 2
    return u.reshape(*lead, K)


def _fwht_descending(x, h):
    # mathematically the same transform, stages in descending stride order: must still pass the exact-value pins
    x = np.asarray(x, dtype=np.float64)
    K = x.shape[-1]
    lead = x.shape[:-1]
    u = x.reshape(*lead, K // h, h).copy()
    s = h // 2
    while s >= 1:
        v = u.reshape(*lead, K // h, h // (2 * s), 2, s)
        a, b = v[..., 0, :].copy(), v[..., 1, :].copy()
        v[..., 0, :] = a + b
        v[..., 1, :] = a - b
        s //= 2
    return u.reshape(*lead, K)


def _dense_transposed(x, R):
    return _DENSE(x, np.asarray(R).T)


def _quant_qmax_off_by_one(u, a_bits, norm=1.0):
    u = np.asarray(u, dtype=np.float64)
    qmax = float(2 ** (a_bits - 1))               # 128 / 8 instead of 127 / 7
    amax = np.max(np.abs(u), axis=1)
    inv = np.where(amax > 0, qmax / np.where(amax > 0, amax, 1.0), 0.0)
    q = np.clip(np.rint(u * inv[:, None]), -qmax, qmax - 1).astype(np.int8)
    return q, (amax / (qmax * np.float64(norm))).astype(np.float32)


def _quant_truncating(u, a_bits, norm=1.0):
    u = np.asarray(u, dtype=np.float64)
    qmax = float(2 ** (a_bits - 1) - 1)
    amax = np.max(np.abs(u), axis=1)
    inv = np.where(amax > 0, qmax / np.where(amax > 0, amax, 1.0), 0.0)
    q = np.clip(np.trunc(u * inv[:, None]), -qmax, qmax).astype(np.int8)     # truncation instead of rounding
    return q, (amax / (qmax * np.float64(norm))).astype(np.float32)


def _quant_half_away(u, a_bits, norm=1.0):
    u = np.asarray(u, dtype=np.float64)
    qmax = float(2 ** (a_bits - 1) - 1)
    amax = np.max(np.abs(u), axis=1)
    inv = np.where(amax > 0, qmax / np.where(amax > 0, amax, 1.0), 0.0)
    t = u * inv[:, None]
    q = np.clip(np.sign(t) * np.floor(np.abs(t) + 0.5), -qmax, qmax).astype(np.int8)   # ties away from zero
    return q, (amax / (qmax * np.float64(norm))).astype(np.float32)


def _asym_zero_point_floor(u, a_bits, norm=1.0):
    q, scale, zero = _ASYM(u, a_bits, norm)
    u = np.asarray(u, dtype=np.float64)
    L = float(2 ** a_bits - 1)
    rng = u.max(axis=1) - u.min(axis=1)
    inv = np.where(rng > 0, L / np.where(rng > 0, rng, 1.0), 0.0)
    z = np.floor(u.min(axis=1) * inv)              # floor instead of round
    xq = np.clip(np.rint(u * inv[:, None]) - z[:, None], 0.0, L)
    half = 2 ** (a_bits - 1)
    return (xq - half).astype(np.int8), scale, (z + half).astype(np.int32)


def _encode_side_no_zero_point(ell, s, z, lo, hi):
    return np.clip(np.rint(ell / s[:, None]), lo, hi)                        # "- z" dropped


def _lut_128(p, I=7):
    v = oracle.tlq.tlq_level_values(p, I)
    wscale = (np.max(np.abs(v), axis=1) / 128.0).astype(np.float32)          # 128 instead of 127
    return np.clip(np.rint(v / wscale.astype(np.float64)[:, None]), -127, 127).astype(np.int8), wscale


def _pack_swapped_nibbles(codes, bits):
    out = _PACK(codes, bits)
    if bits == 4:
        out = ((out >> 4) | (out << 4)).astype(np.uint8)
    else:
        out = out[:, ::-1].copy()
    return out


def _zigzag_without_turning(ranges, B):
    ranges = np.asarray(ranges, dtype=np.float64)
    K = ranges.shape[0]
    nb = K // B
    order = np.argsort(-ranges, kind="stable")
    perm = np.empty(K, dtype=np.int32)
    for r in range(K):
        rnd, pos = divmod(r, nb)
        perm[pos * B + rnd] = order[r]             # always left to right
    return perm


def _blockperm_scatter(x, R1, perm, R2):
    z = oracle.rotation.rotate_blockdiag(x, R1)
    zp = np.empty_like(z)
    zp[:, np.asarray(perm)] = z                    # scatter instead of gather
    return oracle.rotation.rotate_blockdiag(zp, R2)


def _blockperm_narrow_intermediate(x, R1, perm, R2):
    z = oracle.rotation.rotate_blockdiag(x, R1).astype(np.float32).astype(np.float64)   # a storage format leaking in
    return oracle.rotation.rotate_blockdiag(z[:, np.asarray(perm)], R2)


def _e4m3_rounding_towards_zero(x):
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), 448.0)
    pos = oracle.fp8.e4m3_bits_to_f64(np.arange(0x7f, dtype=np.uint8))
    idx = np.searchsorted(pos, a, side="right") - 1               # largest representable magnitude <= |x|: truncation
    return (np.arange(0x7f, dtype=np.uint8)[idx] | (np.signbit(x).astype(np.uint8) << 7)).astype(np.uint8)


def _lut_fp8_top_level_at_448(p):
    v = oracle.tlq.tlq_level_values(p, 3)
    wscale = np.max(np.abs(v), axis=1) / 448.0                    # uses the whole range, but is no power of two
    return oracle.fp8.f64_to_e4m3_bits(v / wscale[:, None]), wscale.astype(np.float32)


def _pack_act_adjacent_pairs(q):
    q = np.asarray(q).astype(np.int64) + 8
    return (q[:, 0::2] | (q[:, 1::2] << 4)).astype(np.uint8)        # neighbours share a byte instead of j and 4 + j


def _blockdiag_transposed(x, Rb):
    return _BLOCKDIAG(x, np.transpose(np.asarray(Rb), (0, 2, 1)))


def _qlinear_without_wscale(q, scale, codes, lut, wscale, bits, bias=None):
    return _QLP(q, scale, codes, lut, np.ones_like(wscale), bits, bias)


def _J_per_channel_only(X_bits):
    x = oracle.bf16_bits_to_f64(X_bits)
    return float(np.sqrt(np.sum(x * x)) / np.sqrt(np.float64(x.shape[1])))   # forgets the token count


def _smoothing_product(X_bits, W, alpha=0.5):
    a = np.max(np.abs(oracle.bf16_bits_to_f64(X_bits)), axis=0)
    w = np.max(np.abs(np.asarray(W, dtype=np.float64)), axis=0)
    ok = (a > 0) & (w > 0)
    s = np.where(ok, np.power(np.where(ok, a, 1.0), alpha) * np.power(np.where(ok, w, 1.0), 1.0 - alpha), 1.0)
    return s.astype(np.float32), (1.0 / s).astype(np.float32)



def _search_side_last_minimum(ell, absw, mask, grid, n_intervals, q_lo, q_hi, gamma_grid=(1.0,)):
    # scanning the grid backwards keeps the last of several equal minima instead of the first
    return _SEARCH(ell, absw, mask, np.asarray(grid)[::-1], n_intervals, q_lo, q_hi, gamma_grid)


def _level_values_floor_mantissa(p, I=7):
    e, sign = oracle.tlq.tlq_exponents(p)
    if I < 0:
        return sign[None, :] * np.exp2(e)
    f = np.floor(e)
    mant = np.floor(np.exp2(e - f) * 2.0 ** I)      # floor instead of round
    return sign[None, :] * mant * np.exp2(f - I)


def _calibrate_same_intervals_for_both_twins(W, bits, alpha_grid, beta_grid, neg_lo=1, chunk=256, gamma_grid=None):
    p = _CALIB(W, bits, alpha_grid, beta_grid, neg_lo, chunk, gamma_grid)
    half = 2 ** (bits - 1)
    p.s_neg = p.s_neg * half / (half - 1)             # as if the negative twin had 2^(b-1) - 1 intervals too
    return p


def _greedy_without_swapping_back(xb, Rtilde, Q):
    x = np.array(xb, dtype=np.float64)
    B = x.shape[1]
    Rhat = np.eye(B)
    for i in range(Q.shape[0]):
        c = int(np.argmax(np.max(np.abs(x), axis=0)))
        for m in (x, Rhat):
            m[:, [0, c]] = m[:, [c, 0]]
        x = (x @ Rtilde) @ Q[i]
        Rhat = (Rhat @ Rtilde) @ Q[i]                 # second exchange forgotten
    return Rhat, x


def _asym_linear_wrong_sign(q, scale, zero, codes, lut, wscale, bits, bias=None):
    return _QLPA(q, scale, -np.asarray(zero), codes, lut, wscale, bits, bias)

def _bf16_truncating(x):
    x = np.asarray(x, dtype=np.float64)
    f = x.astype(np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)             # chops instead of rounding to nearest even


def _asym_constant_row_scale_zero(u, a_bits, norm=1.0):
    q, scale, zero = _ASYM(u, a_bits, norm)
    u = np.asarray(u, dtype=np.float64)
    const = u.max(axis=1) == u.min(axis=1)
    return q, np.where(const, np.float32(0.0), scale).astype(np.float32), zero   # a constant token loses its value


def _exponents_negative_twin_sign(p):
    e, sign = _EXPO(p)
    nlev = 2 ** p.bits
    half = nlev // 2
    for c in range(-half, 0):
        e[:, c & (nlev - 1)] = p.s_neg * (c + p.z_neg.astype(np.float64))    # +c instead of -c for the negative twin
    return e, sign


def _build_with_absmax_ranks(xcal, B, Rtilde, Q1, Q2):
    x = np.asarray(xcal, dtype=np.float64)
    nb = x.shape[1] // B
    R1 = np.empty((nb, B, B))
    y = np.empty_like(x)
    for g in range(nb):
        R1[g], y[:, g * B:(g + 1) * B] = oracle.rotation.greedy_block_rotation(x[:, g * B:(g + 1) * B], Rtilde, Q1[g])
    perm = oracle.rotation.zigzag_permutation(np.max(np.abs(y), axis=0), B)   # magnitude instead of max - min
    yp = y[:, perm]
    R2 = np.empty((nb, B, B))
    for g in range(nb):
        R2[g], _ = oracle.rotation.greedy_block_rotation(yp[:, g * B:(g + 1) * B], Rtilde, Q2[g])
    rnd = lambda R: oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(R))
    return rnd(R1), perm, rnd(R2)


def _select_with_inclusive_threshold(J, threshold=1.0):
    return "hadamard" if J <= threshold else "outlier-aware"


def _levels_layer_bias_scaled(q, scale, codes, levels, bits, bias=None):
    idx = codes.astype(np.int64) & (2 ** bits - 1)
    wv = np.take_along_axis(np.asarray(levels, dtype=np.float64), idx, axis=1)
    y = q.astype(np.float64) @ wv.T
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y * scale.astype(np.float64)[:, None]            # the bias must not take the token's scale


def _levels_layer_by_signed_code_magnitude(q, scale, codes, levels, bits, bias=None):
    idx = np.abs(codes.astype(np.int64))                     # a negative code must select its own (negative) level
    wv = np.take_along_axis(np.asarray(levels, dtype=np.float64), np.minimum(idx, 2 ** bits - 1), axis=1)
    y = (q.astype(np.float64) @ wv.T) * scale.astype(np.float64)[:, None]
    return y if bias is None else y + np.asarray(bias, dtype=np.float64)[None, :]


_ASYM = oracle.actquant.quantize_per_token_asym
_EXPO = oracle.tlq.tlq_exponents
_SEARCH = oracle.tlq._search_side
_CALIB = oracle.tlq.tlq_calibrate
_QLPA = _qlinear_mod.qlinear_from_parts_asym
_DENSE = oracle.rotation.rotate_dense
_PACK = oracle.tlq.pack_codes
_BLOCKDIAG = oracle.rotation.rotate_blockdiag
_QLP = _qlinear_mod.qlinear_from_parts

CASES = {
    "butterfly outputs swapped": (oracle.rotation.fwht_blocks, _fwht_swapped_outputs,
                                  [(t_rot.test_butterfly_equals_matrix_form_exactly, (8, 24)),
                                   (t_rot.test_one_hot_outlier_is_spread_evenly, ())]),
    "dense rotation transposed": (oracle.rotation.rotate_dense, _dense_transposed,
                                  [(t_rot.test_dense_rotation_exact_on_integers_and_not_transposed, ())]),
    "quantizer range off by one": (oracle.actquant.quantize_per_token, _quant_qmax_off_by_one,
                                   [(t_act.test_worked_example_by_hand, ()), (t_act.test_properties, (8,))]),
    "quantizer truncates": (oracle.actquant.quantize_per_token, _quant_truncating,
                            [(t_act.test_brute_force_nearest_grid_point, (8,))]),
    "ties rounded away from zero": (oracle.actquant.quantize_per_token, _quant_half_away,
                                    [(t_act.test_worked_example_by_hand, ())]),
    "zero-point floored": (oracle.actquant.quantize_per_token_asym, _asym_zero_point_floor,
                           [(t_asym.test_worked_example_by_hand, ()), (t_asym.test_brute_force_eq1_in_exact_rationals, (8,))]),
    "TLQ zero-point dropped": (oracle.tlq._encode_side, _encode_side_no_zero_point,
                               [(t_tlq.test_powers_of_two_are_reproduced_exactly, (4,)),
                                (t_tlq.test_encode_is_nearest_level_in_log_distance, (4,))]),
    "level table normalised by 128": (oracle.tlq.tlq_lut, _lut_128, [(t_tlq.test_level_values_and_lut, (4, 7))]),
    "packed codes in the wrong order": (oracle.tlq.pack_codes, _pack_swapped_nibbles,
                                        [(t_tlq.test_pack_examples_from_fixture, ())]),
    "staggered dealing never turns": (oracle.rotation.zigzag_permutation, _zigzag_without_turning,
                                      [(t_str.test_zigzag_hand_example, ())]),
    "permutation applied as a scatter": (oracle.rotation.rotate_blockperm, _blockperm_scatter,
                                         [(t_str.test_equals_the_materialised_dense_product, ()),
                                          (t_str.test_identity_blocks_leave_only_the_permutation, ())]),
    "intermediate of the structured rotation rounded to fp32": (
        oracle.rotation.rotate_blockperm, _blockperm_narrow_intermediate,
        [(t_str.test_nothing_is_rounded_between_the_two_stages, ()),
         (t_str.test_equals_the_materialised_dense_product, ())]),
    "FP8 conversion truncates": (oracle.fp8.f64_to_e4m3_bits, _e4m3_rounding_towards_zero,
                                 [(t_fp8.test_conversion_is_the_nearest_value_ties_to_even_and_saturates, ())]),
    "FP8 level table scaled by a non power of two": (oracle.tlq.tlq_lut_fp8, _lut_fp8_top_level_at_448,
                                                     [(t_fp8.test_fp8_level_table, (4,))]),
    "packed activation codes pair neighbours": (oracle.actquant.pack_act_codes4, _pack_act_adjacent_pairs,
                                                [(t_act.test_packed_4bit_codes_hand_example_and_round_trip, ())]),
    "rotation blocks transposed": (oracle.rotation.rotate_blockdiag, _blockdiag_transposed,
                                   [(t_str.test_blockdiag_equals_block_diagonal_matrix_product, ()),
                                    (t_str.test_equals_the_materialised_dense_product, ())]),
    "weight scale forgotten": (_qlinear_mod.qlinear_from_parts, _qlinear_without_wscale,
                               [(t_ql.test_end_to_end_equals_fake_quant_product, (4, 8))]),
    "J without the token count": (oracle.calib.fluctuation_J, _J_per_channel_only,
                                  [(t_cal.test_J_of_a_constant_tensor_is_its_magnitude, ()), (t_cal.test_J_of_a_single_spike, ())]),
    "search keeps the last minimum": (oracle.tlq._search_side, _search_side_last_minimum,
                                      [(t_tlq.test_equal_minima_keep_the_first_grid_entry, ())]),
    "mantissa floored": (oracle.tlq.tlq_level_values, _level_values_floor_mantissa, [(t_tlq.test_level_values_and_lut, (4, 7))]),
    "negative twin with the positive twin's interval count": (oracle.tlq.tlq_calibrate, _calibrate_same_intervals_for_both_twins,
                                                              [(t_tlq.test_scale_and_zero_point_closed_forms, (4,))]),
    "second channel exchange forgotten": (oracle.rotation.greedy_block_rotation, _greedy_without_swapping_back,
                                          [(t_str.test_one_greedy_step_is_the_printed_matrix_product, ())]),
    "zero-point term with the wrong sign": (_qlinear_mod.qlinear_from_parts_asym, _asym_linear_wrong_sign,
                                            [(t_asym.test_linear_layer_with_zero_point_equals_fake_quant_product, ())]),
    "bf16 conversion truncates": (oracle.bf16.f64_to_bf16_bits, _bf16_truncating, [(t_rot.test_bf16_round_trip_against_torch, ())]),
    "constant token loses its value": (oracle.actquant.quantize_per_token_asym, _asym_constant_row_scale_zero,
                                       [(t_asym.test_constant_rows, ())]),
    "negative twin's exponent with the wrong sign": (oracle.tlq.tlq_exponents, _exponents_negative_twin_sign,
                                                    [(t_tlq.test_powers_of_two_are_reproduced_exactly, (4,)),
                                                     (t_tlq.test_idempotent, (4,))]),
    "permutation ranked by magnitude": (oracle.rotation.build_outlier_rotation, _build_with_absmax_ranks,
                                        [(t_str.test_permutation_ranks_channels_by_max_minus_min_of_the_rotated_calibration_data, ())]),
    "levels layer scales the bias": (_qlinear_mod.qlinear_levels_from_parts, _levels_layer_bias_scaled,
                                     [(t_lev.test_against_exact_rational_arithmetic, (4,))]),
    "levels layer drops the code's sign": (_qlinear_mod.qlinear_levels_from_parts, _levels_layer_by_signed_code_magnitude,
                                           [(t_lev.test_reduces_to_the_fake_quant_product_with_dequantized_weights, ()),
                                            (t_lev.test_distance_to_the_int8_table_path_is_the_table_rounding, (4,))]),
    "threshold rule inclusive": (oracle.calib.select_rotation, _select_with_inclusive_threshold, [(t_cal.test_threshold_rule, ())]),
    "smoothing factor as a product": (oracle.calib.smoothing_factor, _smoothing_product,
                                      [(t_cal.test_half_migration_equalises_activation_and_weight_ranges, ()),
                                       (t_cal.test_migration_extremes, ())]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_a_planted_mistake_fails_a_pin(monkeypatch, name):
    original, wrong, pins = CASES[name]
    assert not _some_pin_fails(pins), "the pins must pass on the unmodified oracle"
    _plant(monkeypatch, original, wrong)
    assert _some_pin_fails(pins), f"no pin noticed: {name}"


def test_an_equivalent_rewrite_passes_the_exact_pins(monkeypatch):
    # control: a butterfly with its stages in the opposite order computes the same exact sums on the pins' integer data
    _plant(monkeypatch, oracle.rotation.fwht_blocks, _fwht_descending)
    t_rot.test_butterfly_equals_matrix_form_exactly(8, 24)
    t_rot.test_one_hot_outlier_is_spread_evenly()
