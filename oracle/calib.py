"""Calibration-time quantities of the Adaptive Rotation Scheme (test infrastructure, fp64).

fluctuation_J: the adaptive metric J = ||X||_F / sqrt(B N C) of a layer's input activations with shape B x N x C
(Method, Eq. J); here the activations arrive flattened to [M, K] = [B N, C].
select_rotation: the case equation that follows it - Hadamard below the threshold, the outlier-aware dual
transformation at or above it; the paper reports that a threshold of 1 works in practice.
"""
import numpy as np

from .bf16 import bf16_bits_to_f64


def fluctuation_J(X_bits: np.ndarray) -> float:
    x = bf16_bits_to_f64(X_bits)
    return float(np.sqrt(np.sum(x * x)) / np.sqrt(np.float64(x.size)))


def select_rotation(J: float, threshold: float = 1.0) -> str:
    return "hadamard" if J < threshold else "outlier-aware"


def smoothing_factor(X_bits: np.ndarray, W: np.ndarray, alpha: float = 0.5):
    """Per-channel smoothing factor that moves quantization difficulty from activations to weights with migration
    strength alpha (Experiment, "Implementation Details": migration strength 0.5; the factor itself is the cited
    SmoothQuant one): s_c = max_t |x[t,c]|^alpha / max_n |w[n,c]|^(1-alpha); activations are divided by s, the
    weight columns multiplied by it.  alpha = 0.5 is evaluated as sqrt(a / w) (two correctly rounded operations);
    a channel whose activations or weights are all zero takes s = 1.
    X_bits bf16 bit patterns [T, K] (calibration activations), W fp32 [N, K].
    Returns (s fp32 [K], inv_s fp32 [K]) = (fp32(s), fp32(1 / s)), both rounded from the fp64 factor."""
    a = np.max(np.abs(bf16_bits_to_f64(X_bits)), axis=0)
    w = np.max(np.abs(np.asarray(W, dtype=np.float32).astype(np.float64)), axis=0)
    ok = (a > 0) & (w > 0)
    a1, w1 = np.where(ok, a, 1.0), np.where(ok, w, 1.0)
    if alpha == 0.5:
        s = np.sqrt(a1 / w1)
    else:
        s = np.power(a1, alpha) / np.power(w1, 1.0 - alpha)
    s = np.where(ok, s, 1.0)
    return s.astype(np.float32), (1.0 / s).astype(np.float32)


def smooth_weights(W: np.ndarray, s: np.ndarray) -> np.ndarray:
    """W'[n, c] = fp32(W[n, c] * s[c]): one fp32 multiplication per weight."""
    return (np.asarray(W, dtype=np.float32) * np.asarray(s, dtype=np.float32)[None, :]).astype(np.float32)
