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
