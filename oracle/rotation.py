"""Rotations of the Adaptive Rotation Scheme (test infrastructure, fp64).

Hadamard branch: the paper defines H_2 = [[1,1],[1,-1]]/sqrt(2) and
H_{2^n} = H_2 (x) H_{2^(n-1)} (Preliminaries, Eq. hadamard).  The oracle works with the
*unnormalised* +-1 matrix; the 1/sqrt(h) factor is a per-token constant and is folded into
the activation scale so that it never touches a rounding decision.  For a hidden size K that
is not a power of two the rotation is block-diagonal, I (x) H_h, with h a power of two
dividing K (the paper only defines sizes 2^n).

Dense branch: X.R for an arbitrary orthogonal R (the paper's outlier-aware product
R1.P.R2 materialised is one such R; Method, ARS case equation).
"""
import numpy as np


def hadamard_matrix(h: int) -> np.ndarray:
    """Unnormalised Sylvester Hadamard matrix (entries +-1) by the Kronecker recursion."""
    assert h >= 1 and (h & (h - 1)) == 0, "Hadamard size must be a power of two"
    H2 = np.array([[1.0, 1.0], [1.0, -1.0]])
    H = np.ones((1, 1))
    while H.shape[0] < h:
        H = np.kron(H2, H)
    return H


def fwht_blocks(x: np.ndarray, h: int) -> np.ndarray:
    """u = x . (I (x) H_h) along the last axis, unnormalised, by the butterfly that the
    Kronecker recursion unrolls into: log2(h) stages, stage s pairs elements 2^s apart and
    replaces (a, b) by (a + b, a - b).  Stages run in ascending stride order; every
    operation is one IEEE fp64 add or subtract (exact whenever the exponents involved span
    less than 53 - 8 - log2(h) binades, which bf16 inputs of any realistic range satisfy)."""
    assert h >= 1 and (h & (h - 1)) == 0
    x = np.asarray(x, dtype=np.float64)
    K = x.shape[-1]
    assert K % h == 0
    lead = x.shape[:-1]
    u = x.reshape(*lead, K // h, h).copy()
    s = 1
    while s < h:
        v = u.reshape(*lead, K // h, h // (2 * s), 2, s)
        a = v[..., 0, :].copy()
        b = v[..., 1, :].copy()
        v[..., 0, :] = a + b
        v[..., 1, :] = a - b
        s *= 2
    return u.reshape(*lead, K)


def rotate_hadamard(x: np.ndarray, h: int) -> np.ndarray:
    """Unnormalised block-Hadamard rotation of fp64 activations [M, K]."""
    return fwht_blocks(x, h)


def rotate_dense(x: np.ndarray, R: np.ndarray) -> np.ndarray:
    """u = x . R with x [M, K], R [K, K], fp64.  The sum over k is taken term by term in
    ascending k, u += x[:, k] * R[k, :], so the result is defined bit for bit (each product
    of two bf16-valued numbers is exact in fp64; each accumulation is one IEEE fp64 add)."""
    x = np.asarray(x, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    M, K = x.shape
    assert R.shape == (K, K)
    u = np.zeros((M, K), dtype=np.float64)
    for k in range(K):
        u += x[:, k:k + 1] * R[k:k + 1, :]
    return u
