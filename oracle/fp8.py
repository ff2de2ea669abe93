"""FP8 E4M3 (the OCP 8-bit float: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest
finite value 448, subnormals down to 2^-9) - test infrastructure.

The paper's "Hardware Implementation" approximates 2^r by an integer of I + 1 bits times 2^-I; with I = 3 a level
+-round(2^r 2^3) 2^(f-3) has four significant bits, which is exactly what an E4M3 number holds, so on matrix cores
that multiply FP8 operands the levels can be fed as they are (up to a per-channel power-of-two scale that moves
them into the format's exponent range) instead of going through an int8 table.
"""
import numpy as np


def e4m3_bits_to_f64(b) -> np.ndarray:
    """Value of every E4M3 bit pattern in b (uint8).  0x7f / 0xff (NaN) map to NaN."""
    b = np.asarray(b, dtype=np.uint8).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e = (b >> 3) & 15
    m = b & 7
    normal = np.ldexp(1.0 + m / 8.0, e - 7)
    sub = np.ldexp(m / 8.0, -6)
    v = np.where(e == 0, sub, normal)
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return sign * v


def f64_to_e4m3_bits(x) -> np.ndarray:
    """Round-to-nearest-even conversion to E4M3, saturating at +-448."""
    x = np.asarray(x, dtype=np.float64)
    s = np.signbit(x)
    a = np.minimum(np.abs(x), 448.0)
    # exponent of the E4M3 binade that holds a: normals 2^-6 .. 2^8, everything smaller shares the subnormal spacing
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6, 8)
    step = np.exp2(e - 3)                        # spacing of representable values in that binade (2^-9 for subnormals)
    n = np.rint(a / step)                        # ties to even; n * step is the rounded magnitude (exact arithmetic)
    r = np.minimum(n * step, 448.0)
    # encode r (exactly representable by now)
    with np.errstate(divide="ignore"):
        er = np.floor(np.log2(np.where(r > 0, r, 1.0)))
    is_sub = r < 2.0 ** -6
    ebits = np.where(is_sub, 0, er + 7).astype(np.int64)
    mbits = np.where(is_sub, np.rint(r * 2.0 ** 9), np.rint((r / np.exp2(er) - 1.0) * 8.0)).astype(np.int64)
    return ((s.astype(np.int64) << 7) | (ebits << 3) | mbits).astype(np.uint8)
