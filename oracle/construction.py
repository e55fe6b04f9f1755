"""Greedy outlier-aware construction of the shared 32x32 rotation block (paper Sec. 4.2, paragraph
"Fine-grained Block-diagonal Rotation": steps (1)-(3), and the statement that all blocks share the matrix built
from the block containing the largest outlier).

The paper gives the construction as a three-step sketch and defers the details to the DuQuant paper, which is
not at hand; what follows is this build's reading of the sketch.  PARITY UNPINNED: no number in the paper pins
it; the tests pin it to its own invariants only (orthogonality, the search state equals X . R, the peak never
rises, closed forms for single spikes).

Reading.  Calibration activations X [T, K].  b* = the block of 32 channels that holds the largest |x| (the
smallest index among equals).  Z_0 = X[:, block b*], R^(0) = I.  For t = 1 .. steps:
  (1) d = the channel of Z_{t-1} with the largest magnitude (smallest index among equals);
  (2) R_t = E_d . H . Q_t . E_d, where E_d exchanges coordinates 0 and d (the identity for d = 0), H is the
      normalised Sylvester-Hadamard matrix, whose first row is uniform (1/sqrt(32) everywhere: what sits in
      coordinate 0 is spread evenly over all 32), and Q_t = diag(1, Q'_t) with a caller-drawn orthogonal
      31 x 31 matrix Q'_t that varies the remaining directions from step to step;
  (3) Z_t = Z_{t-1} . R_t,  R^(t) = R^(t-1) . R_t,  peak_t = max |Z_t|.
The result is R^(t*) with t* the step count of the smallest peak (the smallest t among equals, t = 0 allowed:
then no rotation helps and the identity is kept), rounded to fp32.

Arithmetic: fp64; every dot product is accumulated in index order from zero with one rounding per multiply and
per add (no fused multiply-add), so that an implementation following the same order takes the same argmax and
argmin decisions and reproduces R bit for bit.
"""
import numpy as np

BLOCK = 32
S = 0.17677669529663687          # 1 / sqrt(32) as a double


def hadamard():
    """H[i][k] = (-1)^popcount(i & k) / sqrt(32), fp64."""
    i = np.arange(BLOCK)
    bits = i[:, None] & i[None, :]
    pop = np.zeros_like(bits)
    for b in range(5):
        pop += (bits >> b) & 1
    return np.where(pop % 2 == 0, S, -S).astype(np.float64)


def _dot_rows(A, B):
    """A [m, n] . B [n, p] in fp64, accumulated over n in index order from zero, unfused."""
    acc = np.zeros((A.shape[0], B.shape[1]), dtype=np.float64)
    for r in range(A.shape[1]):
        acc = acc + A[:, r:r + 1] * B[r:r + 1, :]
    return acc


def step_matrix(d, q_prime):
    """R_t of step (2) for outlier channel d and the step's orthogonal 31 x 31 matrix."""
    H = hadamard()
    M = np.empty((BLOCK, BLOCK), dtype=np.float64)
    M[:, 0] = H[:, 0]                                        # Q = diag(1, Q'): column 0 passes through
    M[:, 1:] = _dot_rows(H[:, 1:], np.asarray(q_prime, dtype=np.float64))   # terms k = 1 .. 31 in order
    sigma = np.arange(BLOCK)
    sigma[0], sigma[d] = d, 0                                # E_d as an index exchange
    return M[np.ix_(sigma, sigma)]


def select_block(x):
    """Index of the block of 32 channels holding the largest |x| (smallest index among equals)."""
    a = np.abs(np.asarray(x, dtype=np.float64))
    G = a.shape[1] // BLOCK
    per_block = a.reshape(a.shape[0], G, BLOCK).max(axis=(0, 2))
    return int(np.argmax(per_block))                         # argmax returns the first maximum


def greedy_rotation(x, q_steps):
    """x [T, K] calibration activations (taken exactly), q_steps [steps, 31, 31] fp64 orthogonal.
    Returns dict(R fp32 [32, 32], block, steps, peaks fp64 [steps + 1], channels [steps], Z fp64 [T, 32] at the
    kept step)."""
    x = np.asarray(x, dtype=np.float64)
    q_steps = np.asarray(q_steps, dtype=np.float64)
    assert x.shape[1] % BLOCK == 0 and q_steps.shape[1:] == (BLOCK - 1, BLOCK - 1)
    b = select_block(x)
    Z = x[:, BLOCK * b:BLOCK * (b + 1)].copy()
    R = np.eye(BLOCK, dtype=np.float64)
    peaks = [float(np.max(np.abs(Z)))]
    hist = [(R, Z)]
    channels = []
    for t in range(q_steps.shape[0]):
        d = int(np.argmax(np.max(np.abs(Z), axis=0)))        # step (1)
        Rt = step_matrix(d, q_steps[t])                      # step (2)
        Z = _dot_rows(Z, Rt)                                 # step (3)
        R = _dot_rows(R, Rt)
        channels.append(d)
        peaks.append(float(np.max(np.abs(Z))))
        hist.append((R, Z))
    best = int(np.argmin(np.asarray(peaks)))                 # first minimum
    return dict(R=hist[best][0].astype(np.float32), block=b, steps=best, peaks=np.asarray(peaks),
                channels=channels, Z=hist[best][1])
