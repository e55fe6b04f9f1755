"""CPU oracle for the DuQuant++ online hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the path computes, written from the
paper (Sec. 3.2 Eq. 2, Sec. 4.2 Eq. 4 and Eq. 5) and the OCP Microscaling fixed
points.  It shares no code with the HIP library and must never be imported by
the product package; only the tests, the smoke check and the bench's CPU
baseline leg call it.

    rotation.rotate              Eq. 4 / Eq. 5  (block-diagonal X . R)
    mxfp4.quantize / dequantize  Eq. 2          (E8M0 scale + E2M1 codes)
    linear.mxfp4_gemm            Eq. 5          (Q(X^) . Q(W^))
    smoothing.*                  Eq. 3          (diagonal Lambda, and its merge into the rotation blocks)
    construction.*               Sec. 4.2       (greedy construction of the shared rotation block; parity unpinned)
    pipeline.*                   the library's entry points composed from the above

Pinned by tests/test_oracle_*.py (hand-worked groups, exact rational brute force,
closed forms, invariants).  Not pinned by any number printed in the paper: the
paper prints no worked numeric example for these equations.
"""
from . import construction, linear, mxfp4, pipeline, rotation, smoothing  # noqa: F401
