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
    assert a_bits in (4, 8)
    u = np.asarray(u, dtype=np.float64)
    qmax = float(2 ** (a_bits - 1) - 1)
    amax = np.max(np.abs(u), axis=1)
    inv = np.zeros_like(amax)
    nz = amax > 0
    inv[nz] = qmax / amax[nz]
    q = np.clip(np.rint(u * inv[:, None]), -qmax, qmax).astype(np.int8)
    scale = (amax / (qmax * np.float64(norm))).astype(np.float32)
    return q, scale
