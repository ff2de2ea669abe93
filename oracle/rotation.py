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


# --------------------------------------------------------------------------------------------------
# Outlier-aware branch in its structured form (Method, "Adaptive Rotation Scheme": X . R1 . P . R2 with
# block-wise greedy rotations R1, R2 and the staggered channel permutation P).

def rotate_blockdiag(x: np.ndarray, Rb: np.ndarray) -> np.ndarray:
    """u = x . diag(Rb[0], ..., Rb[nb-1]) with x [M, K] fp64 and Rb [nb, B, B], K = nb * B.
    Within a block the sum over k is taken term by term in ascending k (one multiply, one add)."""
    x = np.asarray(x, dtype=np.float64)
    Rb = np.asarray(Rb, dtype=np.float64)
    nb, B, B2 = Rb.shape
    M, K = x.shape
    assert B == B2 and K == nb * B
    u = np.zeros((M, K), dtype=np.float64)
    for g in range(nb):
        xs = x[:, g * B:(g + 1) * B]
        acc = np.zeros((M, B), dtype=np.float64)
        for k in range(B):
            acc += xs[:, k:k + 1] * Rb[g, k:k + 1, :]
        u[:, g * B:(g + 1) * B] = acc
    return u


def rotate_blockperm(x: np.ndarray, R1: np.ndarray, perm: np.ndarray, R2: np.ndarray) -> np.ndarray:
    """u = ((x . R1) . P) . R2 with block-diagonal R1, R2 ([nb, B, B] each, bf16-valued) and the channel
    permutation P in gather form, (z . P)[:, j] = z[:, perm[j]] (Method, ARS case equation, second branch).
    Both block products are the plain fp64 sums of rotate_blockdiag (ascending k, one rounded multiply and one
    rounded add per term); nothing is rounded between the stages."""
    perm = np.asarray(perm)
    K = x.shape[1]
    assert perm.shape == (K,) and np.array_equal(np.sort(perm), np.arange(K)), "perm must be a permutation of 0..K-1"
    z = rotate_blockdiag(x, R1)
    return rotate_blockdiag(z[:, perm], R2)


def zigzag_permutation(ranges: np.ndarray, B: int) -> np.ndarray:
    """The staggered reordering P: channels are sorted by their numerical range (descending, ties by channel
    index) and dealt across the nb = K / B blocks alternately - left to right on even rounds, right to left on
    odd rounds - so that every block receives one channel of each group of nb consecutive ranks.
    Returns perm (gather form): new channel j takes old channel perm[j]."""
    ranges = np.asarray(ranges, dtype=np.float64)
    K = ranges.shape[0]
    assert K % B == 0
    nb = K // B
    order = np.argsort(-ranges, kind="stable")
    perm = np.empty(K, dtype=np.int32)
    for r in range(K):
        rnd, pos = divmod(r, nb)
        blk = pos if rnd % 2 == 0 else nb - 1 - pos
        perm[blk * B + rnd] = order[r]
    return perm


def _seq_matmul(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """a [T, B] . b [B, B] with the sum over k taken in ascending k, one rounded multiply and one rounded add
    per term (no fused multiply-add)."""
    out = np.zeros((a.shape[0], b.shape[1]), dtype=np.float64)
    for k in range(a.shape[1]):
        out += a[:, k:k + 1] * b[k:k + 1, :]
    return out


def greedy_block_rotation(xb: np.ndarray, Rtilde: np.ndarray, Q: np.ndarray):
    """Greedy outlier-aware rotation of one block of B channels (Method, equation R^i = E_c* R~ Q E_c*,
    R^ = prod_i R^i).  xb [T, B] calibration activations of the block, Rtilde [B, B] the initial orthogonal
    matrix (its job is to spread channel 0 over all channels), Q [n, B, B] one orthogonal matrix per greedy
    step.  Step i: c* = the channel with the largest |value| over the calibration tokens (first one on ties);
    E swaps channels 0 and c*; the block's activations and the running product are multiplied, left to
    right, by E, R~, Q[i], E.  Returns (R^ [B, B] fp64, rotated activations [T, B])."""
    x = np.array(xb, dtype=np.float64)
    B = x.shape[1]
    Rhat = np.eye(B)
    for i in range(Q.shape[0]):
        c = int(np.argmax(np.max(np.abs(x), axis=0)))
        for m in (x, Rhat):
            m[:, [0, c]] = m[:, [c, 0]]
        x = _seq_matmul(_seq_matmul(x, Rtilde), Q[i])
        Rhat = _seq_matmul(_seq_matmul(Rhat, Rtilde), Q[i])
        for m in (x, Rhat):
            m[:, [0, c]] = m[:, [c, 0]]
    return Rhat, x


def build_outlier_rotation(xcal: np.ndarray, B: int, Rtilde: np.ndarray, Q1: np.ndarray, Q2: np.ndarray):
    """Calibration of the outlier-aware branch: R1 (greedy, per block) on the calibration activations
    xcal [T, K]; P from the per-channel ranges max - min of xcal . R1; R2 (greedy, per block) on the permuted
    result.  Q1, Q2 [nb, n, B, B]: the per-step orthogonal matrices of every block.
    Returns (R1 bf16-rounded fp64 [nb, B, B], perm int32 [K], R2 likewise): the rotations as the runtime stores
    them.  The working state stays in fp64 throughout (the rounding to bf16 is applied to the outputs only)."""
    from .bf16 import bf16_bits_to_f64, f64_to_bf16_bits
    x = np.asarray(xcal, dtype=np.float64)
    T, K = x.shape
    nb = K // B
    assert K == nb * B
    R1 = np.empty((nb, B, B))
    y = np.empty_like(x)
    for g in range(nb):
        R1[g], y[:, g * B:(g + 1) * B] = greedy_block_rotation(x[:, g * B:(g + 1) * B], Rtilde, Q1[g])
    perm = zigzag_permutation(np.max(y, axis=0) - np.min(y, axis=0), B)
    yp = y[:, perm]
    R2 = np.empty((nb, B, B))
    for g in range(nb):
        R2[g], _ = greedy_block_rotation(yp[:, g * B:(g + 1) * B], Rtilde, Q2[g])
    rnd = lambda R: bf16_bits_to_f64(f64_to_bf16_bits(R))
    return rnd(R1), perm, rnd(R2)
