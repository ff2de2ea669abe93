"""Twin-Log Quantization of weights (test infrastructure, fp64).

Follows Method, "Twin-Log Quantization for Weights":
  W' = log2|W|, split by the sign masks M+ / M-            (paragraph "Twin-Log Quantization")
  W_q+ = clamp(round(W+/s+) - z+, 0, 2^(b-1)-1)
  W_q- = clamp(round(W-/s-) - z-, 0, 2^(b-1)),  W_q = W_q+ - W_q-      (Eq. log-based quantizer)
  s+ = (alpha*W+max - W+min)/(2^(b-1)-1), z+ = round(W+min/s+)
  s- = (beta *W-max - W-min)/ 2^(b-1),    z- = round(W-min/s-)         (Eq. hyperparameters clip)
  W_f = 2^(s+(W_q+ + z+)) M+  -  2^(s-(W_q- + z-)) M-                  (Eq. dequant)
  f = floor(e), r = e - f, 2^r ~ round(2^r * 2^I) * 2^-I               ("Hardware Implementation")

Readings of what the paper leaves open (all per output channel, weights per-channel static):
  * rounding is round-half-to-even;
  * min / max run over the masked positions only; exact zeros are left out of the
    statistics and take code 0;
  * the negative twin is clamped to [1, 2^(b-1)] instead of [0, 2^(b-1)], so that
    W_q = W_q+ - W_q- in [-2^(b-1), 2^(b-1)-1] is a true b-bit two's-complement code whose
    sign alone recovers the mask (with the printed lower bound 0 both twins map to W_q = 0 and
    the masks would have to be stored beside the codes).  `neg_lo=0` gives the printed clamp
    as a diagnostic;
  * alpha, beta come from caller-supplied grids scanned in the given order; a candidate whose
    clipped maximum does not exceed the minimum is skipped; the objective is the per-channel,
    per-sign squared error sum (W_f - W)^2 with the exact Eq. dequant levels, summed in a stated
    order (_ordered_sum: 256 interleaved partial sums over ascending k, then the partials in
    ascending order) so that which of two close candidates is smaller does not depend on who adds;
    the first minimum wins; a side with no element or no valid candidate takes s = 1,
    z = round(W_min) (0 if empty);
  * optional extension, not in the paper: a lower clip factor gamma on W_min, searched jointly with alpha (beta):
        s = (alpha * W_max - gamma * W_min) / intervals,  z = round(gamma * W_min / s)
    (log2 values are negative for |w| < 1, so gamma < 1 raises the lower end; smaller magnitudes clamp to the lowest
    level of their twin).  The grid {1} is the paper's formula; the search scans alpha in the outer loop and gamma
    in the inner loop, first minimum wins;
  * the MFMA operand of a code is an int8: v(c) = +-round(2^r 2^I) 2^(f-I) (I < 0: exactly
    2^e), divided by wscale_n = fp32(max_c |v(c)| / 127) and rounded.  This int8
    normalisation is not in the paper (its datapath shifts inside the reduction).
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class TLQParams:
    bits: int
    s_pos: np.ndarray   # fp64 [N]
    z_pos: np.ndarray   # int32 [N]
    s_neg: np.ndarray   # fp64 [N]
    z_neg: np.ndarray   # int32 [N]
    alpha: np.ndarray   # fp32 [N]  chosen clip factor of the positive side
    beta: np.ndarray    # fp32 [N]  chosen clip factor of the negative side
    gamma_pos: np.ndarray = None   # fp32 [N]  chosen lower clip factors (all ones without the extension)
    gamma_neg: np.ndarray = None
    err_pos: np.ndarray = None     # fp64 [N]  the search objective at the chosen factors (inf: no valid candidate)
    err_neg: np.ndarray = None


def _log2_abs(W):
    absw = np.abs(W)
    ell = np.zeros_like(absw)
    nz = absw > 0
    ell[nz] = np.log2(absw[nz])
    return absw, ell


def _encode_side(ell, s, z, lo, hi):
    return np.clip(np.rint(ell / s[:, None]) - z[:, None], lo, hi)


_STRIDE = 256


def _ordered_sum(v):
    """Row sums of v [N, K] in the order the search objective is defined in: partial sum j (j = 0..255) adds
    v[:, j], v[:, j + 256], v[:, j + 512], ... one after the other; the total adds partial 0, 1, ..., 255 one
    after the other.  Every step is one fp64 addition (positions past K contribute nothing)."""
    N, K = v.shape
    part = np.zeros((N, _STRIDE))
    for a in range(0, K, _STRIDE):
        blk = v[:, a:a + _STRIDE]
        part[:, :blk.shape[1]] = part[:, :blk.shape[1]] + blk
    tot = np.zeros(N)
    for j in range(_STRIDE):
        tot = tot + part[:, j]
    return tot


def _search_side(ell, absw, mask, grid, n_intervals, q_lo, q_hi, gamma_grid=(1.0,)):
    """Grid search of one clip factor (and the optional lower clip) for one sign.
    Returns (s, z, chosen_factor, chosen_gamma, objective at the choice)."""
    N = ell.shape[0]
    has = mask.any(axis=1)
    wmax = np.max(np.where(mask, ell, -np.inf), axis=1)
    wmin = np.min(np.where(mask, ell, np.inf), axis=1)
    wmax = np.where(has, wmax, 0.0)
    wmin = np.where(has, wmin, 0.0)
    best_err = np.full(N, np.inf)
    best_s = np.ones(N)
    best_z = np.rint(wmin)
    best_c = np.ones(N, dtype=np.float32)
    best_g = np.ones(N, dtype=np.float32)
    for c32 in np.asarray(grid, dtype=np.float32):
        T = np.float64(c32) * wmax
        for g32 in np.asarray(gamma_grid, dtype=np.float32):
            B = np.float64(g32) * wmin
            valid = has & (T > B)
            s = np.where(valid, (T - B) / n_intervals, 1.0)
            z = np.rint(B / s)
            q = _encode_side(ell, s, z, q_lo, q_hi)
            lev = np.exp2(s[:, None] * (q + z[:, None]))
            d = np.where(mask, lev - absw, 0.0)
            err = _ordered_sum(d * d)
            better = valid & (err < best_err)
            best_err = np.where(better, err, best_err)
            best_s = np.where(better, s, best_s)
            best_z = np.where(better, z, best_z)
            best_c = np.where(better, c32, best_c)
            best_g = np.where(better, g32, best_g)
    return best_s, best_z.astype(np.int32), best_c, best_g, best_err


def tlq_calibrate(W, bits, alpha_grid, beta_grid, neg_lo=1, chunk=256, gamma_grid=None):
    """Search-based clipping per output channel.  W fp32/fp64 [N, K] -> TLQParams.
    gamma_grid: None (the paper's formula) or the grid of the lower clip factor (extension)."""
    assert bits in (3, 4)
    W = np.asarray(W, dtype=np.float64)
    N = W.shape[0]
    half = 2 ** (bits - 1)
    gg = (1.0,) if gamma_grid is None else gamma_grid
    out = [np.empty(N), np.empty(N, np.int32), np.empty(N), np.empty(N, np.int32),
           np.empty(N, np.float32), np.empty(N, np.float32), np.empty(N, np.float32), np.empty(N, np.float32),
           np.empty(N), np.empty(N)]
    for a in range(0, N, chunk):
        w = W[a:a + chunk]
        absw, ell = _log2_abs(w)
        sp, zp, al, gp, ep = _search_side(ell, absw, w > 0, alpha_grid, float(half - 1), 0.0, float(half - 1), gg)
        sn, zn, be, gn, en = _search_side(ell, absw, w < 0, beta_grid, float(half), float(neg_lo), float(half), gg)
        for dst, src in zip(out, (sp, zp, sn, zn, al, be, gp, gn, ep, en)):
            dst[a:a + chunk] = src
    return TLQParams(bits, *out)


def tlq_encode(W, p: TLQParams, neg_lo=1, chunk=256):
    """Signed b-bit codes W_q = W_q+ - W_q- (int8 [N, K]) under fixed parameters."""
    W = np.asarray(W, dtype=np.float64)
    half = 2 ** (p.bits - 1)
    codes = np.zeros(W.shape, dtype=np.int8)
    for a in range(0, W.shape[0], chunk):
        w = W[a:a + chunk]
        sl = slice(a, a + chunk)
        _, ell = _log2_abs(w)
        qp = _encode_side(ell, p.s_pos[sl], p.z_pos[sl].astype(np.float64), 0.0, float(half - 1))
        qn = _encode_side(ell, p.s_neg[sl], p.z_neg[sl].astype(np.float64), float(neg_lo), float(half))
        codes[sl] = np.where(w > 0, qp, np.where(w < 0, -qn, 0.0)).astype(np.int8)
    return codes


def tlq_exponents(p: TLQParams):
    """e[n, c & (2^b - 1)] = exponent of the level of signed code c: s+(c + z+) for c >= 0,
    s-(-c + z-) for c < 0.  Returns (e fp64 [N, 2^b], sign fp64 [2^b])."""
    nlev = 2 ** p.bits
    half = nlev // 2
    e = np.empty((len(p.s_pos), nlev))
    sign = np.empty(nlev)
    for c in range(-half, half):
        idx = c & (nlev - 1)
        if c >= 0:
            e[:, idx] = p.s_pos * (c + p.z_pos.astype(np.float64))
            sign[idx] = 1.0
        else:
            e[:, idx] = p.s_neg * (-c + p.z_neg.astype(np.float64))
            sign[idx] = -1.0
    return e, sign


def tlq_level_values(p: TLQParams, I=7):
    """Real value of every code, [N, 2^b] indexed by c & (2^b - 1).  I >= 0: the integerised
    form round(2^r 2^I) 2^(f - I) of "Hardware Implementation"; I < 0: exactly 2^e (Eq. dequant)."""
    e, sign = tlq_exponents(p)
    if I < 0:
        return sign[None, :] * np.exp2(e)
    f = np.floor(e)
    r = e - f
    mant = np.rint(np.exp2(r) * float(2 ** I))
    return sign[None, :] * np.ldexp(mant, (f - I).astype(np.int64))


def tlq_lut(p: TLQParams, I=7):
    """(lut int8 [N, 2^b], wscale fp32 [N]): lut = round(v / wscale), wscale = fp32(max|v| / 127)."""
    v = tlq_level_values(p, I)
    wscale = (np.max(np.abs(v), axis=1) / 127.0).astype(np.float32)
    lut = np.clip(np.rint(v / wscale.astype(np.float64)[:, None]), -127, 127).astype(np.int8)
    return lut, wscale


def tlq_lut_fp8(p: TLQParams):
    """The levels as FP8 E4M3 operands ("Hardware Implementation" with I = 3: a level round(2^r 2^3) 2^(f-3) has four
    significant bits, an E4M3 number's worth).  Per channel the levels are divided by a power of two
    wscale = 2^(floor(log2 max|v|) - 7), which puts the largest one in [128, 256) - inside E4M3's range (448) - and
    then rounded to E4M3 (nearest even): exact for every level within 2^13 of the largest, rounded to the subnormal
    spacing 2^-9 below that, zero below 2^-10.  Returns (lut uint8 [N, 2^b] of E4M3 bit patterns indexed by
    c & (2^b - 1), wscale fp32 [N]).  This normalisation is not in the paper (its datapath shifts per element)."""
    from .fp8 import f64_to_e4m3_bits
    v = tlq_level_values(p, 3)
    vmax = np.max(np.abs(v), axis=1)
    e = np.floor(np.log2(np.where(vmax > 0, vmax, 1.0))) - 7.0
    wscale = np.exp2(e)
    return f64_to_e4m3_bits(v / wscale[:, None]), wscale.astype(np.float32)


def tlq_dequant(codes, p: TLQParams):
    """W_f of Eq. dequant from signed codes (sign of the code = mask)."""
    v = tlq_level_values(p, I=-1)
    idx = codes.astype(np.int64) & (2 ** p.bits - 1)
    return np.take_along_axis(v, idx, axis=1)


def pack_codes(codes, bits):
    """Canonical packed layout, row n = K codes, each the low b bits of W_q.
    W4: byte j = code[2j] | code[2j+1] << 4.  W3: every 8 codes form a 24-bit little-endian
    group with code i at bits [3i, 3i+3)."""
    c = codes.astype(np.int64) & (2 ** bits - 1)
    N, K = c.shape
    if bits == 4:
        assert K % 2 == 0
        return (c[:, 0::2] | (c[:, 1::2] << 4)).astype(np.uint8)
    assert bits == 3 and K % 8 == 0
    g = c.reshape(N, K // 8, 8)
    v = np.zeros((N, K // 8), dtype=np.int64)
    for i in range(8):
        v |= g[:, :, i] << (3 * i)
    out = np.stack([v & 255, (v >> 8) & 255, (v >> 16) & 255], axis=-1)
    return out.reshape(N, K // 8 * 3).astype(np.uint8)


def unpack_codes(packed, bits, K):
    """Inverse of pack_codes: signed codes int8 [N, K]."""
    p = packed.astype(np.int64)
    N = p.shape[0]
    if bits == 4:
        c = np.empty((N, K), dtype=np.int64)
        c[:, 0::2] = p & 15
        c[:, 1::2] = p >> 4
    else:
        g = p.reshape(N, K // 8, 3)
        v = g[:, :, 0] | (g[:, :, 1] << 8) | (g[:, :, 2] << 16)
        c = np.stack([(v >> (3 * i)) & 7 for i in range(8)], axis=-1).reshape(N, K)
    half = 2 ** (bits - 1)
    return np.where(c >= half, c - 2 * half, c).astype(np.int8)
