"""Per-token dynamic uniform activation quantizer (test infrastructure, fp64).

The paper's uniform quantizer (Preliminaries, Eq. 1) maps x to round(x / s) with a scale
from the observed range, and activations are quantized per token, dynamically (Experiment,
"Implementation Details").  This build uses the symmetric absmax form of that quantizer:
signed codes in [-qmax, qmax], qmax = 2^(a-1) - 1, no zero-point, so that the rescale after
the integer GEMM is a pure per-token x per-channel scale.  Rounding is round-half-to-even.

Arithmetic (fixed so that an fp64 implementation elsewhere reproduces it bit for bit):
    amax_t = max_k |u[t, k]|
    inv_t  = qmax / amax_t             one IEEE fp64 division   (amax = 0 -> inv = 0)
    q[t,k] = clamp(rint(u[t,k] * inv_t), -qmax, qmax)   one fp64 multiply per element
    scale_t = fp32(amax_t / (qmax * norm))               norm = sqrt(h) for the unnormalised
                                                         Hadamard transform, 1 for a dense R
"""
import numpy as np


def quantize_per_token(u: np.ndarray, a_bits: int, norm: float = 1.0):
    """u fp64 [M, K] -> (q int8 [M, K], scale fp32 [M])."""
    assert a_bits in (4, 6, 8)           # the bit-widths of the paper's tables
    u = np.asarray(u, dtype=np.float64)
    qmax = float(2 ** (a_bits - 1) - 1)
    amax = np.max(np.abs(u), axis=1)
    inv = np.zeros_like(amax)
    nz = amax > 0
    inv[nz] = qmax / amax[nz]
    q = np.clip(np.rint(u * inv[:, None]), -qmax, qmax).astype(np.int8)
    scale = (amax / (qmax * np.float64(norm))).astype(np.float32)
    return q, scale


def quantize_per_token_asym(u: np.ndarray, a_bits: int, norm: float = 1.0):
    """The paper's uniform quantizer with zero-point (Preliminaries, Eq. 1), per token:
        s = (x_max - x_min) / (2^b - 1),  z = round(x_min / s),  x_q = clamp(round(x / s) - z, 0, 2^b - 1),
        x_f = s (x_q + z).
    Arithmetic (fixed so that an fp64 implementation elsewhere reproduces it bit for bit): with
    L = 2^b - 1 and range = x_max - x_min, the quotients x / s are taken as products with one
    reciprocal, inv = L / range (one fp64 division): z = rint(x_min * inv), x_q = clamp(rint(x * inv) - z, 0, L);
    s = range / L.  A constant token (range = 0, value c) takes inv = 0, x_q = 0 and (s, z) = (|c|, sign c)
    (s = 1, z = 0 for c = 0), so that s (x_q + z) = c exactly.
    Returned in the form the integer GEMM consumes: q = x_q - 2^(b-1) (int8), zero = z + 2^(b-1) (int32), so that
    x_f = scale * (q + zero) with scale = fp32(s / norm).  u fp64 [M, K] -> (q int8 [M, K], scale fp32 [M],
    zero int32 [M])."""
    assert a_bits in (4, 6, 8)           # the bit-widths of the paper's tables
    u = np.asarray(u, dtype=np.float64)
    L = float(2 ** a_bits - 1)
    half = 2 ** (a_bits - 1)
    umax, umin = np.max(u, axis=1), np.min(u, axis=1)
    rng = umax - umin
    pos = rng > 0
    inv = np.zeros_like(rng)
    inv[pos] = L / rng[pos]
    s = np.where(pos, rng / L, np.where(umin != 0, np.abs(umin), 1.0))
    z = np.where(pos, np.rint(umin * inv), np.sign(umin))
    xq = np.clip(np.rint(u * inv[:, None]) - z[:, None], 0.0, L)
    xq = np.where(pos[:, None], xq, 0.0)
    q = (xq - half).astype(np.int8)
    zero = (z + half).astype(np.int32)
    scale = (s / np.float64(norm)).astype(np.float32)
    return q, scale, zero


def pack_act_codes4(q: np.ndarray) -> np.ndarray:
    """Storage of 4-bit activation codes two per byte (the paper's W4A4 / W3A4 settings; it leaves the storage open,
    this is the build's format): q int8 [M, K] with values in [-7, 7], K a multiple of 8 -> uint8 [M, K/2].
    Every 8 consecutive codes of a token make 4 bytes; byte j of the group holds q[j] + 8 in its low nibble and
    q[4 + j] + 8 in its high nibble."""
    q = np.asarray(q)
    M, K = q.shape
    assert K % 8 == 0 and q.min(initial=0) >= -7 and q.max(initial=0) <= 7
    g = q.astype(np.int64).reshape(M, K // 8, 8) + 8
    return (g[:, :, :4] | (g[:, :, 4:] << 4)).astype(np.uint8).reshape(M, K // 2)


def unpack_act_codes4(q4: np.ndarray) -> np.ndarray:
    """Inverse of pack_act_codes4: uint8 [M, K/2] -> int8 [M, K]."""
    q4 = np.asarray(q4, dtype=np.uint8)
    M, H = q4.shape
    g = q4.astype(np.int64).reshape(M, H // 4, 4)
    out = np.concatenate([(g & 15) - 8, (g >> 4) - 8], axis=2)
    return out.reshape(M, 2 * H).astype(np.int8)
