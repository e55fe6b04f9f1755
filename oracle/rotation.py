"""Block-diagonal rotation (paper Sec. 4.2, Eq. 4 and the X . R^ factor of Eq. 5).

R^ = BlockDiag(R_1 .. R_G) with 32x32 orthogonal blocks aligned to the MXFP4 groups.
Row-vector convention: for a row x and block j, y[32j + c] = sum_r x[32j + r] * R[j][r][c].
A weight stored [N, K] (row n = output channel n, i.e. the transpose of the paper's
[C_in, C_out] W) is rotated row by row in the same way, which is W^ = R^T W of Eq. 5.
With a single block (R.shape[0] == 1) every group shares it (the variant of Sec. 4.2
where all blocks equal the one built from the group with the largest outlier).
"""
import numpy as np

BLOCK = 32


def rotate(x: np.ndarray, R: np.ndarray) -> np.ndarray:
    """x [rows, K] (any real dtype, taken exactly), R [G or 1, 32, 32] fp32.
    Accumulates each 32-term dot product in fp64 and rounds once to fp32."""
    x = np.asarray(x, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    rows, K = x.shape
    G = K // BLOCK
    assert K % BLOCK == 0 and R.shape[1:] == (BLOCK, BLOCK) and R.shape[0] in (1, G)
    y = np.empty((rows, K), dtype=np.float64)
    for j in range(G):
        Rj = R[j if R.shape[0] == G else 0]
        y[:, BLOCK * j:BLOCK * (j + 1)] = x[:, BLOCK * j:BLOCK * (j + 1)] @ Rj
    return y.astype(np.float32)
