"""Seeded synthetic inputs for the quantized-linear hot path of LRQ-DiT.

This module only *draws inputs* (activations, weights, rotation matrices, layer
shape lists).  It holds none of the method's arithmetic (no Hadamard transform,
no quantizer, no TLQ): both the CPU oracle and the HIP path consume the buffers
made here, and neither imports the other.

The paper's real workloads are PixArt / FLUX / OpenSORA activations and weights
(Experiment section, "Models and Prompt sets"); none of those are available, so
the generators reproduce the *described* statistics instead:

* weights: zero-mean, Gaussian-like with long tails on both sides (Method,
  "Twin-Log Quantization for Weights", Motivation) -> Student-t(nu=4) * 0.02;
* activations: N(0,1) body, "mild" outliers that rarely exceed ~5 and "salient"
  outliers confined to a few fixed channels across all tokens, reaching the
  hundreds (Method, "Adaptive Rotation Scheme", Motivation) -> a Bernoulli(p)
  mask scaled x4 and S fixed channels scaled x g.

All draws come from numpy's PCG64 seeded by SeedSequence([MASTER, *key]); rows of
an activation matrix are drawn in independent chunks of ROW_CHUNK rows so any row
range of a very large matrix can be regenerated without drawing the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

MASTER_SEED = 20250803
ROW_CHUNK = 256

# stream ids keep the different tensors of one layer statistically independent
_STREAM_X, _STREAM_W, _STREAM_R, _STREAM_CH, _STREAM_BIAS, _STREAM_J = 1, 2, 3, 4, 5, 6


def rng_for(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([MASTER_SEED, *key])))


# --------------------------------------------------------------------------- bf16 storage helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even.  Storage
    conversion of generated inputs only."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- layer descriptions
@dataclass(frozen=True)
class LayerSpec:
    name: str
    config: int          # 1..5, the workload it belongs to
    block: int           # transformer block index (0 for single-block configs)
    layer: int           # index of the linear inside the block
    M: int               # tokens
    K: int               # input features (hidden dimension that is rotated)
    N: int               # output features
    w_bits: int          # 3 | 4
    a_bits: int          # 4 | 8
    rotation: str        # "hadamard" | "dense"
    had_block: int       # Hadamard block size h (power of two dividing K)
    p_mild: float        # fraction of mildly outlying entries (x4)
    n_salient: int       # number of salient channels
    gain: float          # salient channel gain
    J: float = 0.0       # seeded stand-in for the fluctuation score of the layer

    @property
    def key(self) -> Tuple[int, int, int]:
        return (self.config, self.block, self.layer)

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K


def default_had_block(K: int) -> int:
    """Largest power of two dividing K."""
    return K & (-K)


# --------------------------------------------------------------------------- tensors
def salient_channels(K: int, n_salient: int, key: Sequence[int]) -> np.ndarray:
    return np.sort(rng_for(*key, _STREAM_CH).choice(K, size=n_salient, replace=False))


def make_activations(M: int, K: int, key: Sequence[int], p_mild: float, n_salient: int,
                     gain: float, rows: Optional[Tuple[int, int]] = None) -> np.ndarray:
    """bf16 bit patterns (uint16) of X[r0:r1, :K] for the layer identified by `key`."""
    r0, r1 = (0, M) if rows is None else rows
    assert 0 <= r0 <= r1 <= M
    ch = salient_channels(K, n_salient, key) if n_salient > 0 else np.zeros(0, np.int64)
    out = np.empty((r1 - r0, K), np.uint16)
    c0, c1 = r0 // ROW_CHUNK, (r1 + ROW_CHUNK - 1) // ROW_CHUNK
    for c in range(c0, c1):
        lo, hi = c * ROW_CHUNK, min((c + 1) * ROW_CHUNK, M)
        g = rng_for(*key, _STREAM_X, c)
        x = g.standard_normal((hi - lo, K), dtype=np.float32)
        mild = g.random((hi - lo, K), dtype=np.float32) < np.float32(p_mild)
        x = np.where(mild, x * np.float32(4.0), x)
        if len(ch):
            x[:, ch] *= np.float32(gain)
        a, b = max(lo, r0), min(hi, r1)
        out[a - r0:b - r0] = f32_to_bf16_bits(x[a - lo:b - lo])
    return out


def make_weights(N: int, K: int, key: Sequence[int]) -> np.ndarray:
    """fp32 W[N,K] (already in the rotated basis): Student-t(nu=4) * 0.02."""
    g = rng_for(*key, _STREAM_W)
    return (g.standard_t(4.0, size=(N, K)) * 0.02).astype(np.float32)


def make_bias(N: int, key: Sequence[int]) -> np.ndarray:
    return (rng_for(*key, _STREAM_BIAS).standard_normal(N) * 0.1).astype(np.float32)


def make_rotation(K: int, key: Sequence[int]) -> np.ndarray:
    """bf16 bit patterns of a dense K x K rotation: Q factor of a seeded Gaussian with
    the sign convention diag(R_qr) > 0.  The bf16-rounded matrix (only approximately
    orthogonal) is *the input*: both sides use it exactly as stored."""
    g = rng_for(*key, _STREAM_R)
    a = g.standard_normal((K, K))
    q, r = np.linalg.qr(a)
    q = q * np.sign(np.diag(r))[None, :]
    return f32_to_bf16_bits(q.astype(np.float32))


def make_block_rotations(K: int, B: int, key: Sequence[int], which: int = 0) -> np.ndarray:
    """bf16 bit patterns [K/B, B, B] of a block-diagonal rotation: one seeded QR factor per block (sign
    convention diag(R_qr) > 0); `which` separates the two rotations of a layer."""
    out = np.empty((K // B, B, B), dtype=np.uint16)
    for g in range(K // B):
        a = rng_for(*key, _STREAM_R, 1 + which, g).standard_normal((B, B))
        q, r = np.linalg.qr(a)
        out[g] = f32_to_bf16_bits((q * np.sign(np.diag(r))[None, :]).astype(np.float32))
    return out


def make_channel_permutation(K: int, key: Sequence[int]) -> np.ndarray:
    """A seeded permutation of the K channels (int32, gather form)."""
    return rng_for(*key, _STREAM_R, 7).permutation(K).astype(np.int32)


def make_spreading_matrix(B: int) -> np.ndarray:
    """fp64 [B, B] orthogonal, symmetric matrix whose first row is 1/sqrt(B) everywhere (the Householder
    reflection that maps e_0 to the uniform unit vector): an initial matrix for the greedy rotation builder."""
    v = -np.full(B, 1.0 / np.sqrt(B))
    v[0] += 1.0
    return np.eye(B) - 2.0 * np.outer(v, v) / float(v @ v)


def make_step_rotations(nb: int, n: int, B: int, key: Sequence[int], which: int = 0) -> np.ndarray:
    """fp64 [nb, n, B, B]: per block and greedy step an orthogonal matrix diag(1, Q') with Q' the QR factor of
    a seeded (B-1) x (B-1) Gaussian - the random rotations the greedy builder takes as an input."""
    out = np.zeros((nb, n, B, B))
    for g in range(nb):
        for i in range(n):
            a = rng_for(*key, _STREAM_R, 11 + which, g, i).standard_normal((B - 1, B - 1))
            q, r = np.linalg.qr(a)
            out[g, i, 0, 0] = 1.0
            out[g, i, 1:, 1:] = q * np.sign(np.diag(r))[None, :]
    return out


def layer_tensors(spec: LayerSpec, rows: Optional[Tuple[int, int]] = None, with_bias: bool = False):
    """(X bf16 bits [rows,K], W fp32 [N,K], R bf16 bits [K,K] or None, bias or None)."""
    X = make_activations(spec.M, spec.K, spec.key, spec.p_mild, spec.n_salient, spec.gain, rows)
    W = make_weights(spec.N, spec.K, spec.key)
    R = make_rotation(spec.K, spec.key) if spec.rotation == "dense" else None
    b = make_bias(spec.N, spec.key) if with_bias else None
    return X, W, R, b


# --------------------------------------------------------------------------- the five workloads
_PIXART = [("qkv", 1152, 3456), ("proj", 1152, 1152), ("fc1", 1152, 4608), ("fc2", 4608, 1152)]
_FLUX = [("qkv", 3072, 9216), ("proj", 3072, 3072), ("mlp_up", 3072, 12288), ("mlp_down", 12288, 3072)]


def _seeded_mix(key: Sequence[int]):
    g = rng_for(*key, _STREAM_J)
    p = float(g.uniform(0.02, 0.08))
    S = int(g.integers(4, 33))
    gain = float(g.uniform(20.0, 80.0))
    J = float(g.uniform(0.0, 2.0))
    return p, S, gain, J


def config_layers(cfg: int) -> List[LayerSpec]:
    """Layer list of workload `cfg` (1-based, as listed in the benchmark description)."""
    out: List[LayerSpec] = []
    if cfg == 1:
        out.append(LayerSpec("single", 1, 0, 0, 256, 1152, 1152, 4, 8, "hadamard", 128, 0.05, 8, 40.0))
    elif cfg == 2:
        for i, (nm, K, N) in enumerate(_PIXART):
            out.append(LayerSpec(nm, 2, 0, i, 8192, K, N, 4, 8, "hadamard", default_had_block(K), 0.05, 8, 40.0))
    elif cfg == 3:
        for i, (nm, K, N) in enumerate(_FLUX):
            out.append(LayerSpec(nm, 3, 0, i, 4608, K, N, 4, 4, "hadamard", default_had_block(K), 0.05, 16, 60.0))
    elif cfg == 4:
        # per-layer seeded outlier mix and score J; the K=3072 layers are ranked by J and
        # the upper half takes the dense rotation, the rest (and K=12288) take Hadamard.
        mixes = [_seeded_mix((4, 0, i)) for i in range(len(_FLUX))]
        k3072 = [i for i, (_, K, _) in enumerate(_FLUX) if K == 3072]
        ranked = sorted(k3072, key=lambda i: -mixes[i][3])
        dense = set(ranked[: (len(k3072) + 1) // 2])
        for i, (nm, K, N) in enumerate(_FLUX):
            p, S, gain, J = mixes[i]
            rot = "dense" if i in dense else "hadamard"
            out.append(LayerSpec(nm, 4, 0, i, 35100, K, N, 4, 8, rot, default_had_block(K), p, S, gain, J))
    elif cfg == 5:
        for blk in range(28):
            specs = _PIXART + [("adaLN", 1152, 6912)]
            for i, (nm, K, N) in enumerate(specs):
                M = 2 if nm == "adaLN" else 8192
                g = rng_for(5, blk, i, _STREAM_J)
                # J ~ lognormal centred below the threshold 1 so that roughly 5-10 % of the
                # layers exceed it (the paper applies the extra rotation to about 5 %).
                J = float(np.exp(g.normal(-0.75, 0.5)))
                rot = "dense" if (J >= 1.0 and K == 1152) else "hadamard"
                out.append(LayerSpec(f"b{blk}.{nm}", 5, blk, i, M, K, N, 3, 4, rot,
                                     default_had_block(K), 0.05, 8, 40.0, J))
    else:
        raise ValueError(f"unknown config {cfg}")
    return out


DEFAULT_GRID = np.arange(21, dtype=np.float32) * np.float32(0.05) + np.float32(1.0)  # 1.00 .. 2.00
