"""W4A4 MXFP4 matrix product (paper Eq. 5: Y^ = Q(X^) . Q(W^)).

Both operands are MXFP4 along K; the result is the plain inner product of the values
the codes stand for, Y[t, n] = sum_k val_a[t, k] * val_b[n, k], taken in fp64.
"""
import numpy as np

from . import mxfp4


def mxfp4_gemm(a_codes, a_scales, b_codes, b_scales) -> np.ndarray:
    """A codes [T, K/2] + scales [T, K/32]; B codes [N, K/2] + scales [N, K/32] -> Y [T, N] fp64."""
    a = mxfp4.dequantize(a_codes, a_scales)
    b = mxfp4.dequantize(b_codes, b_scales)
    return a @ b.T


def round_to_bf16_bits(y32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (the bf16 output epilogue)."""
    u = np.ascontiguousarray(y32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = u + 0x7FFF + ((u >> 16) & 1)
    return (r >> 16).astype(np.uint16)
