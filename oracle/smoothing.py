"""Per-channel smoothing (paper Sec. 4.2, Eq. 3, and its place in Eq. 5).

Eq. 3 rewrites Y = X W as (X Lambda^-1)(Lambda W) with a diagonal Lambda over the reduction axis,
Lambda_j = max|X_j|^alpha / max|W_j|^(1 - alpha); Eq. 5 puts the rotation after it:
X^ = X Lambda^-1 R^ and W^ = R^T Lambda W.  With W stored [N, K] (row n = output channel n) both
operands are rows over K: a token becomes (x / lambda) . R^ and a weight row (w * lambda) . R^.

A diagonal matrix times a block-diagonal one is block-diagonal, so the two factors can be merged
offline into one (no longer orthogonal) 32x32 block per group:
    (x / lambda) . R_j  =  x . (diag(1 / lambda_j) R_j),     (w * lambda) . R_j  =  w . (diag(lambda_j) R_j)
`fold_into_rotation` writes those merged blocks; `apply` is the definition itself, kept for checking them.
"""
import numpy as np

from . import rotation

BLOCK = rotation.BLOCK


def smoothing_scales(x, w, alpha=0.5):
    """Eq. 3: lambda[k] = max_t |x[t, k]|^alpha / max_n |w[n, k]|^(1 - alpha), fp64.  x [T, K], w [N, K]."""
    ax = np.max(np.abs(np.asarray(x, dtype=np.float64)), axis=0)
    aw = np.max(np.abs(np.asarray(w, dtype=np.float64)), axis=0)
    return ax ** alpha / aw ** (1.0 - alpha)


def apply(x, lam, inverse):
    """x Lambda^-1 (inverse=True, activations) or x Lambda (inverse=False, weight rows), fp64."""
    x = np.asarray(x, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    return x / lam[None, :] if inverse else x * lam[None, :]


def fold_into_rotation(R, lam):
    """R [G or 1, 32, 32], lam [K] -> (R_act, R_wgt), each fp32 [G, 32, 32]:
    R_act[j][r][c] = R[j][r][c] / lam[32 j + r],  R_wgt[j][r][c] = R[j][r][c] * lam[32 j + r]
    (r is the input channel of block j).  A shared block expands to one block per group."""
    R = np.asarray(R, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    G = lam.shape[0] // BLOCK
    assert lam.shape[0] % BLOCK == 0 and R.shape[1:] == (BLOCK, BLOCK) and R.shape[0] in (1, G)
    Rg = R if R.shape[0] == G else np.broadcast_to(R, (G, BLOCK, BLOCK))
    l = lam.reshape(G, BLOCK, 1)
    return (Rg / l).astype(np.float32), (Rg * l).astype(np.float32)
