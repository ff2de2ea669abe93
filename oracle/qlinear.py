"""The W-A-quantized linear layer assembled from the oracle's parts (test infrastructure, fp64).

Y[t, n] = scale_t * wscale_n * sum_k q[t, k] * lut_n[code[n, k]]  (+ bias_n)

which is the integer-times-scale form of the last equation of "Hardware Implementation"
(I^X the activation integers, s^X their scale) with the per-channel int8 level table standing
in for the shift datapath, and per-token / per-channel granularity as in Experiment,
"Implementation Details".
"""
import numpy as np

from .actquant import quantize_per_token, quantize_per_token_asym
from .bf16 import bf16_bits_to_f64
from .rotation import rotate_blockperm, rotate_dense, rotate_hadamard
from .tlq import TLQParams, tlq_calibrate, tlq_encode, tlq_lut


def _rotate(X_bits, rotation, had_block, R_bits, blockperm=None, prescale=None):
    """(u fp64 [M, K], norm) for the layer's rotation choice (Method, ARS case equation).
    rotation: "none" | "hadamard" | "dense" (R_bits: bf16 bit patterns [K, K]) | "blockperm" (blockperm =
    (R1_bits [nb, B, B], perm [K], R2_bits [nb, B, B]): the structured form X . R1 . P . R2).
    prescale: optional fp32 [K], the reciprocal smoothing factor; x is multiplied by it channel-wise first (each
    product of a bf16 and an fp32 value is exact in fp64)."""
    x = bf16_bits_to_f64(X_bits)
    if prescale is not None:
        x = x * np.asarray(prescale, dtype=np.float32).astype(np.float64)[None, :]
    if rotation == "hadamard":
        return rotate_hadamard(x, had_block), np.sqrt(np.float64(had_block))
    if rotation == "dense":
        return rotate_dense(x, bf16_bits_to_f64(R_bits)), 1.0
    if rotation == "blockperm":
        R1_bits, perm, R2_bits = blockperm
        return rotate_blockperm(x, bf16_bits_to_f64(R1_bits), perm, bf16_bits_to_f64(R2_bits)), 1.0
    assert rotation == "none"
    return x, 1.0


def ars_rotate_quant(X_bits, a_bits, rotation, had_block=None, R_bits=None, blockperm=None, prescale=None):
    """(Smooth,) rotate (per-layer choice) and quantize per token.
    X_bits: bf16 bit patterns [M, K].  Returns (q int8 [M, K], scale fp32 [M])."""
    u, norm = _rotate(X_bits, rotation, had_block, R_bits, blockperm, prescale)
    return quantize_per_token(u, a_bits, norm)


def ars_rotate_quant_asym(X_bits, a_bits, rotation, had_block=None, R_bits=None, blockperm=None, prescale=None):
    """(Smooth,) rotate and quantize per token with the zero-point form of Eq. 1.
    Returns (q int8 [M, K], scale fp32 [M], zero int32 [M]) with x_f = scale * (q + zero)."""
    u, norm = _rotate(X_bits, rotation, had_block, R_bits, blockperm, prescale)
    return quantize_per_token_asym(u, a_bits, norm)


def qlinear_from_parts_asym(q, scale, zero, codes, lut, wscale, bits, bias=None):
    """Y[t, n] = scale_t wscale_n (sum_k q[t,k] lut_n[code[n,k]] + zero_t sum_k lut_n[code[n,k]]) (+ bias_n):
    the zero-point of Eq. 1 contributes a per-token multiple of each channel's level sum."""
    idx = codes.astype(np.int64) & (2 ** bits - 1)
    wv = np.take_along_axis(lut.astype(np.float64), idx, axis=1)
    acc = q.astype(np.float64) @ wv.T + zero.astype(np.float64)[:, None] * wv.sum(axis=1)[None, :]
    y = (acc * scale.astype(np.float64)[:, None]) * wscale.astype(np.float64)[None, :]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


def qlinear_from_parts(q, scale, codes, lut, wscale, bits, bias=None):
    """fp64 Y [M, N] from activation codes, weight codes and the per-channel level table.
    The integer sum is taken by an fp64 matmul of integer-valued matrices: every partial sum is
    an integer below 2^53, so the result is the exact integer whatever the summation order."""
    idx = codes.astype(np.int64) & (2 ** bits - 1)
    wv = np.take_along_axis(lut.astype(np.float64), idx, axis=1)          # [N, K] decoded int8 values
    acc = q.astype(np.float64) @ wv.T                                      # exact integers
    y = (acc * scale.astype(np.float64)[:, None]) * wscale.astype(np.float64)[None, :]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


def qlinear_levels_from_parts(q, scale, codes, levels, bits, bias=None):
    """The layer on the levels themselves ("Hardware Implementation": value of a code = +-round(2^r 2^I) 2^(f-I)),
    without the per-channel int8 table: Y[t, n] = scale_t sum_k q[t, k] levels[n, code[n, k]] (+ bias_n), fp64.
    levels: fp64 [N, 2^bits] indexed by the code's low bits (tlq_level_values)."""
    idx = codes.astype(np.int64) & (2 ** bits - 1)
    wv = np.take_along_axis(np.asarray(levels, dtype=np.float64), idx, axis=1)          # [N, K]
    y = (q.astype(np.float64) @ wv.T) * scale.astype(np.float64)[:, None]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


def act_codes_to_e4m3(q):
    """4-bit activation codes (integers in [-7, 7]) as FP8 E4M3 bit patterns: every such integer has at most three
    significant bits, so the conversion is exact."""
    from .fp8 import e4m3_bits_to_f64, f64_to_e4m3_bits
    q = np.asarray(q)
    assert np.abs(q).max(initial=0) <= 7
    bits = f64_to_e4m3_bits(q.astype(np.float64))
    assert np.array_equal(e4m3_bits_to_f64(bits), q.astype(np.float64))
    return bits


def qlinear_fp8_from_parts(q, scale, codes, lut_fp8, wscale_fp8, bits, bias=None):
    """The layer with FP8 E4M3 operands on both sides (4-bit activation codes; levels from tlq_lut_fp8):
    Y[t, n] = scale_t wscale_n sum_k q[t, k] value(lut_fp8[n, code[n, k]]) (+ bias_n), the sum exact in fp64
    (a product has at most seven significant bits)."""
    from .fp8 import e4m3_bits_to_f64
    idx = codes.astype(np.int64) & (2 ** bits - 1)
    wv = np.take_along_axis(e4m3_bits_to_f64(lut_fp8), idx, axis=1)                      # [N, K]
    y = (q.astype(np.float64) @ wv.T) * scale.astype(np.float64)[:, None] * np.asarray(wscale_fp8, dtype=np.float64)[None, :]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


def qlinear(X_bits, W, w_bits, a_bits, rotation, had_block=None, R_bits=None, I=7,
            alpha_grid=None, beta_grid=None, bias=None):
    """Whole path: TLQ calibrate + encode the (already rotated) weights, rotate + quantize the
    activations, integer GEMM, rescale.  Returns a dict with every intermediate."""
    p = tlq_calibrate(W, w_bits, alpha_grid, beta_grid)
    codes = tlq_encode(W, p)
    lut, wscale = tlq_lut(p, I)
    q, scale = ars_rotate_quant(X_bits, a_bits, rotation, had_block, R_bits)
    y = qlinear_from_parts(q, scale, codes, lut, wscale, w_bits, bias)
    return dict(params=p, codes=codes, lut=lut, wscale=wscale, q=q, scale=scale, y=y)


def reference_linear(X_bits, W, rotation, had_block=None, R_bits=None):
    """Unquantized product in the rotated basis, (X.Rot)(W)^T in fp64 with the normalised
    rotation: the quantity the quantized layer approximates (diagnostic only)."""
    x = bf16_bits_to_f64(X_bits)
    if rotation == "hadamard":
        u = rotate_hadamard(x, had_block) / np.sqrt(np.float64(had_block))
    elif rotation == "dense":
        u = x @ bf16_bits_to_f64(R_bits)
    else:
        u = x
    return u @ np.asarray(W, dtype=np.float64).T
