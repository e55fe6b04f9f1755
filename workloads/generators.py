"""Seeded generators for activations X, weights W and rotation blocks R.

Recipe (all draws from numpy's counter-based Philox generator, keyed by a base
seed and a stream name, so every consumer reproduces the same buffers):

* X [T, K]: standard normal fp32; outlier structure is injected by multiplying
  already-drawn values (whole channels = "normal outliers", a few channels in a
  few tokens = "massive outliers", the taxonomy of Sec. 4.1 of the paper); the
  result is rounded to bf16 (round-to-nearest-even) and returned as uint16 bits.
* W [N, K]: normal with the given standard deviation, rounded to bf16.
* R [G, 32, 32]: per block, the Q factor of a seeded fp64 Gaussian 32x32 matrix
  with columns sign-fixed by the diagonal of the triangular factor (Haar
  distributed), rounded to fp32.  Stored R[j][r][c], r = input channel of block
  j, c = output channel, so that y = x . R (row-vector convention of Eq. 5).

These stand in for LLaMA-3 activations/weights and for calibrated rotations,
none of which are available offline.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 0x260417789
BLOCK = 32


def stream_seed(*names) -> int:
    """64-bit stream id derived from the base seed and a tuple of names."""
    h = hashlib.sha256(("|".join(str(n) for n in names)).encode()).digest()
    return (int.from_bytes(h[:8], "little") ^ BASE_SEED) & 0xFFFFFFFFFFFFFFFF


def _rng(*names) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=stream_seed(*names)))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class OutlierSpec:
    """`n_channels` seeded channels multiplied by `factor`, in `n_tokens` seeded
    tokens (None = every token)."""
    n_channels: int
    factor: float
    n_tokens: Optional[int] = None


def make_activations(name: str, T: int, K: int, outliers: Tuple[OutlierSpec, ...] = ()) -> np.ndarray:
    """X [T, K] as bf16 bit patterns (uint16)."""
    rng = _rng(name, "X", T, K)
    x = rng.standard_normal((T, K), dtype=np.float32)
    if outliers:
        pick = _rng(name, "X-outliers", T, K)
        total = sum(o.n_channels for o in outliers)
        chans = pick.choice(K, size=total, replace=False)
        at = 0
        for o in outliers:
            c = np.sort(chans[at:at + o.n_channels])
            at += o.n_channels
            if o.n_tokens is None or o.n_tokens >= T:
                x[:, c] *= np.float32(o.factor)
            else:
                t = np.sort(pick.choice(T, size=o.n_tokens, replace=False))
                x[np.ix_(t, c)] *= np.float32(o.factor)
    return f32_to_bf16_bits(x)


def make_weights(name: str, N: int, K: int, std: float) -> np.ndarray:
    """W [N, K] (the layout of a Linear's weight: row n = output channel n) as bf16 bits."""
    rng = _rng(name, "W", N, K)
    out = np.empty((N, K), dtype=np.uint16)
    step = max(1, (1 << 24) // K)
    for n0 in range(0, N, step):  # chunked so the fp32 temporary stays small
        n1 = min(N, n0 + step)
        w = rng.standard_normal((n1 - n0, K), dtype=np.float32) * np.float32(std)
        out[n0:n1] = f32_to_bf16_bits(w)
    return out


def make_rotation_blocks(name: str, G: int) -> np.ndarray:
    """R [G, 32, 32] fp32, each block orthogonal (sign-fixed QR of a Gaussian)."""
    rng = _rng(name, "R", G)
    g = rng.standard_normal((G, BLOCK, BLOCK))
    q, r = np.linalg.qr(g)
    d = np.sign(np.diagonal(r, axis1=1, axis2=2))
    d[d == 0] = 1.0
    q = q * d[:, None, :]
    return np.ascontiguousarray(q.astype(np.float32))


def make_orthogonal_steps(name: str, steps: int, n: int = BLOCK - 1) -> np.ndarray:
    """[steps, n, n] fp64 orthogonal matrices (sign-fixed QR of seeded Gaussians): the random draws of the greedy
    construction of a rotation block, handed to the oracle and to the library alike."""
    rng = _rng(name, "Qsteps", steps, n)
    g = rng.standard_normal((steps, n, n))
    q, r = np.linalg.qr(g)
    d = np.sign(np.diagonal(r, axis1=1, axis2=2))
    d[d == 0] = 1.0
    return np.ascontiguousarray(q * d[:, None, :])


def make_smoothing_scales(name: str, K: int, spread: float = 2.0) -> np.ndarray:
    """A synthetic smoothing diagonal [K] fp32: log-uniform in [2^-spread, 2^spread].  Stands in for scales
    calibrated on real activations and weights, which are not available."""
    rng = _rng(name, "lambda", K)
    return np.exp2(rng.uniform(-spread, spread, size=K)).astype(np.float32)


def identity_blocks(G: int) -> np.ndarray:
    return np.ascontiguousarray(np.broadcast_to(np.eye(BLOCK, dtype=np.float32), (G, BLOCK, BLOCK)))


def hadamard_blocks(G: int) -> np.ndarray:
    """Normalised Sylvester-Hadamard H32 / sqrt(32) repeated G times (a closed-form
    orthogonal block used by tests)."""
    h = np.array([[1.0]])
    while h.shape[0] < BLOCK:
        h = np.block([[h, h], [h, -h]])
    h = (h / np.sqrt(float(BLOCK))).astype(np.float32)
    return np.ascontiguousarray(np.broadcast_to(h, (G, BLOCK, BLOCK)))


# Workload configurations (shapes from LLaMA-3-8B / 70B linear layers).
CONFIGS: Dict[str, dict] = {
    # q_proj shape, small enough for the oracle to finish in seconds
    "c1_qproj_T64": dict(T=64, K=4096, N=4096, w_std=0.02, out="f32",
                         outliers=(OutlierSpec(8, 50.0),)),
    # LLaMA-3-8B down_proj prefill: the headline workload
    "c2_8b_down_prefill": dict(T=2048, K=14336, N=4096, w_std=0.02, out="bf16",
                               outliers=(OutlierSpec(4, 1000.0, 8), OutlierSpec(32, 20.0))),
    # LLaMA-3-70B down_proj prefill
    "c4_70b_down_prefill": dict(T=4096, K=28672, N=8192, w_std=0.01, out="f32",
                                outliers=(OutlierSpec(8, 1000.0, 16),)),
}
# decode shapes (generators as c1)
for _T in (1, 4, 16):
    CONFIGS[f"c3_decode_gateup_T{_T}"] = dict(T=_T, K=4096, N=14336, w_std=0.02, out="f32",
                                               outliers=(OutlierSpec(8, 50.0),))
    CONFIGS[f"c3_decode_down_T{_T}"] = dict(T=_T, K=14336, N=4096, w_std=0.02, out="f32",
                                             outliers=(OutlierSpec(8, 50.0),))

# LLaMA-3-8B decoder-layer linear set (T = 8192 in the full configuration):
# (name, K, N, has_outliers)
LAYER_SET_8B: List[Tuple[str, int, int, bool]] = [
    ("q", 4096, 4096, False),
    ("k", 4096, 1024, False),
    ("v", 4096, 1024, False),
    ("o", 4096, 4096, True),
    ("gate", 4096, 14336, False),
    ("up", 4096, 14336, False),
    ("down", 14336, 4096, True),
]
# the whole set as one workload: T tokens through all seven linears, each with its own rotation; inputs of
# the linears marked True carry 8 seeded outlier channels x100, outputs are bf16
LAYER_SET_CONFIGS = {
    "c5_8b_layer_set_T8192": dict(T=8192, layers=LAYER_SET_8B, w_std=0.02, out="bf16",
                                  outliers=(OutlierSpec(8, 100.0),)),
}
