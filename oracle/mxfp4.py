"""MXFP4 encoding (paper Sec. 3.2, Eq. 2): groups of 32 values share one E8M0
power-of-two scale; each value is stored as a 4-bit E2M1 code.

Readings taken where Eq. 2 is silent or garbled (listed in the design notes):
  * the exponent offset b is the E2M1 maximum exponent, 2: s = 2^(floor(log2 amax) - 2);
  * rounding to the nearest value of the format = one round-to-nearest on the E2M1 grid with ties
    to the code whose mantissa bit is 0, then saturation at +-6;
  * groups run along the last (reduction) axis;
  * an all-zero group gets scale byte 0; the exponent is clamped to [-127, 127];
  * the sign bit of the input is kept even when the magnitude rounds to zero.
"""
import numpy as np

GROUP = 32
E2M1_MAGNITUDES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64)
E2M1_EMAX = 2
E8M0_BIAS = 127


def group_exponent(y32: np.ndarray) -> np.ndarray:
    """Shared exponent e per group of 32 along the last axis: floor(log2 amax) - 2,
    clamped to the E8M0 range; e = -127 for an all-zero group.  Returns int64 [..., G]."""
    y = np.asarray(y32, dtype=np.float64)
    assert y.shape[-1] % GROUP == 0
    g = y.reshape(y.shape[:-1] + (y.shape[-1] // GROUP, GROUP))
    amax = np.max(np.abs(g), axis=-1)
    mant, ex = np.frexp(amax)              # amax = mant * 2^ex, mant in [0.5, 1)
    floor_log2 = ex.astype(np.int64) - 1
    e = floor_log2 - E2M1_EMAX
    e = np.clip(e, -127, 127)
    e = np.where(amax == 0.0, -127, e)
    return e.astype(np.int64)


def e2m1_magnitude_code(v: np.ndarray) -> np.ndarray:
    """Magnitude code 0..7 of v >= 0 (already divided by the group scale): nearest of
    {0, .5, 1, 1.5, 2, 3, 4, 6}, ties to the even code, everything above 5 -> 6."""
    v = np.asarray(v, dtype=np.float64)
    code = np.zeros(v.shape, dtype=np.uint8)            # v <= 0.25            -> 0
    code[(v > 0.25) & (v < 0.75)] = 1                    # (0.25, 0.75)         -> 0.5
    code[(v >= 0.75) & (v <= 1.25)] = 2                  # [0.75, 1.25]         -> 1
    code[(v > 1.25) & (v < 1.75)] = 3                    # (1.25, 1.75)         -> 1.5
    code[(v >= 1.75) & (v <= 2.5)] = 4                   # [1.75, 2.5]          -> 2
    code[(v > 2.5) & (v < 3.5)] = 5                      # (2.5, 3.5)           -> 3
    code[(v >= 3.5) & (v <= 5.0)] = 6                    # [3.5, 5]             -> 4
    code[v > 5.0] = 7                                    # > 5 (saturating)     -> 6
    return code


def quantize(y32: np.ndarray):
    """Eq. 2 on fp32 input [rows, K] (K % 32 == 0), groups along K.
    Returns (codes uint8 [rows, K/2], scales uint8 [rows, K/32]); element 2i sits in
    the low nibble of byte i, element 2i+1 in the high nibble; scale byte = e + 127."""
    y32 = np.asarray(y32)
    assert y32.dtype == np.float32 and y32.ndim == 2 and y32.shape[1] % GROUP == 0
    rows, K = y32.shape
    e = group_exponent(y32)                                    # [rows, G]
    y = y32.astype(np.float64)
    v = np.ldexp(np.abs(y), -np.repeat(e, GROUP, axis=1))      # |y| / s, exact in fp64
    mag = e2m1_magnitude_code(v)
    code = mag | (np.signbit(y32).astype(np.uint8) << 3)
    packed = (code[:, 0::2] | (code[:, 1::2] << 4)).astype(np.uint8)
    scales = (e + E8M0_BIAS).astype(np.uint8)
    return packed, scales


def unpack_codes(codes: np.ndarray) -> np.ndarray:
    """[rows, K/2] packed bytes -> [rows, K] 4-bit codes."""
    codes = np.asarray(codes, dtype=np.uint8)
    out = np.empty((codes.shape[0], codes.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = codes & 0xF
    out[:, 1::2] = codes >> 4
    return out


def dequantize(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """Values the encoding stands for, exact in fp64: (-1)^s * magnitude * 2^(byte-127)."""
    c = unpack_codes(codes)
    mag = E2M1_MAGNITUDES[c & 7]
    val = np.where((c & 8) != 0, -mag, mag)
    ex = np.repeat(np.asarray(scales, dtype=np.int64) - E8M0_BIAS, GROUP, axis=1)
    return np.ldexp(val, ex)
