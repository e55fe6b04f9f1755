"""The library's entry points composed from the oracle's steps (paper Eq. 5).

    rotate_quantize   X^ = X . R^ , then Eq. 2            (online, activations)
    quantize_weights  W^ = R^T W  , then Eq. 2            (offline, weights stored [N, K])
    rotq_gemm         Q(X . R^) . Q(W^)                   (fused form: same codes, same product)
With `lam` (the diagonal of Eq. 3) the operands are X Lambda^-1 R^ and R^T Lambda W, as Eq. 5 is written.
"""
import numpy as np

from . import linear, mxfp4, rotation, smoothing


def _as_real(x):
    """Inputs arrive as bf16 bit patterns (uint16) or as float arrays."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << 16).view(np.float32)
    return x


def rotate_quantize(x, R, lam=None):
    """Returns (codes, scales, y_rot fp32)."""
    x = _as_real(x)
    if lam is not None:
        x = smoothing.apply(x, lam, inverse=True)
    y = rotation.rotate(x, R)
    codes, scales = mxfp4.quantize(y)
    return codes, scales, y


def quantize_weights(w, R, lam=None):
    """w [N, K]: each row (scaled by Lambda when given) rotated like a token, then quantised along K."""
    w = _as_real(w)
    if lam is not None:
        w = smoothing.apply(w, lam, inverse=False)
    y = rotation.rotate(w, R)
    codes, scales = mxfp4.quantize(y)
    return codes, scales, y


def rotq_gemm(x, R, b_codes, b_scales):
    a_codes, a_scales, _ = rotate_quantize(x, R)
    return linear.mxfp4_gemm(a_codes, a_scales, b_codes, b_scales)


def per_group_normalised_errors(y32, codes, scales):
    """Fig. 1 statistic before its mean: ||Q(x) - x||_2 / ||x||_2 of every group of 32, as an array [rows, K/32];
    a group without norm has no ratio and reads -1."""
    y = np.asarray(y32, dtype=np.float64)
    d = mxfp4.dequantize(codes, scales) - y
    G = y.shape[1] // 32
    num = np.linalg.norm(d.reshape(y.shape[0], G, 32), axis=-1)
    den = np.linalg.norm(y.reshape(y.shape[0], G, 32), axis=-1)
    ok = den > 0
    out = np.full(den.shape, -1.0)
    out[ok] = num[ok] / den[ok]
    return out


def per_group_normalised_error(y32, codes, scales):
    """Fig. 1 statistic: ||Q(x) - x||_2 / ||x||_2 per group of 32, averaged over groups
    with non-zero norm."""
    r = per_group_normalised_errors(y32, codes, scales)
    return float(np.mean(r[r >= 0]))
