"""bfloat16 <-> fp64 for the oracle (test infrastructure; independent of the HIP path)."""
import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp64 exactly."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(y: np.ndarray) -> np.ndarray:
    """Round fp64 to the nearest bf16 (ties to even) in ONE rounding, return bit patterns.

    A bf16 has 8 significant bits: write y = m * 2^e with m in [0.5, 1), round m * 2^8 to an
    integer with rint (half-even), and rebuild.  Values in the normal bf16 range only."""
    y = np.asarray(y, dtype=np.float64)
    m, e = np.frexp(y)
    r = np.ldexp(np.rint(m * 256.0) / 256.0, e)
    f = r.astype(np.float32)           # exact: r has <= 8 significant bits
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
