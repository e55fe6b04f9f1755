"""The GPU tests' own checkers, exercised on the CPU with planted deviations (in oracle-made codes, never on a
device): a checker that accepts everything would make the GPU parity tests vacuous."""
import numpy as np
import pytest

from oracle import mxfp4
from helpers import assert_codes_differ_only_at_boundaries, per_element_gemm_bound


def _group(vals):
    y = np.zeros((1, 32), dtype=np.float32)
    y[0, :len(vals)] = vals
    return y


def _check(y_dev, y_ref, x_norm=8.0, **kw):
    """Codes of y_dev ("device") against codes of y_ref (oracle); the block's input is one value of size x_norm."""
    c, s = mxfp4.quantize(y_dev)
    c_ref, s_ref = mxfp4.quantize(y_ref)
    x = np.zeros_like(y_ref)
    x[:, 0::32] = x_norm
    return assert_codes_differ_only_at_boundaries(c, s, c_ref, s_ref, y_ref, x, **kw)


def test_flip_at_a_rounding_boundary_is_accepted():
    # 4.0 holds the scale at 1; 2.5 is the tie between codes 2 and 3: one ulp either side flips the code
    up, down = np.nextafter(np.float32(2.5), np.float32(3)), np.nextafter(np.float32(2.5), np.float32(2))
    assert _check(_group([4.0, up]), _group([4.0, down])) == (1, 0)
    # and a sign flip of a vanishing value
    assert _check(_group([4.0, down, -1e-7]), _group([4.0, up, 1e-7]), max_fraction=0.1) == (2, 0)


def test_flip_away_from_a_boundary_is_rejected():
    with pytest.raises(AssertionError):
        _check(_group([4.0, 2.6]), _group([4.0, 2.4]))          # 0.1 from the tie with a slack of 8e-5
    with pytest.raises(AssertionError):
        _check(_group([4.0, 3.6]), _group([4.0, 2.4]))          # two codes apart
    with pytest.raises(AssertionError):
        _check(_group([4.0, -0.3]), _group([4.0, 0.3]))         # a sign flip of a value that is not small


def test_scale_change_needs_a_group_maximum_at_a_power_of_two():
    below = np.nextafter(np.float32(8.0), np.float32(0))
    assert _check(_group([8.0, 1.0]), _group([below, 1.0])) == (0, 1)
    with pytest.raises(AssertionError):
        _check(_group([8.5, 1.0]), _group([7.5, 1.0]))
    with pytest.raises(AssertionError):
        _check(_group([33.0, 1.0]), _group([7.9999, 1.0]))      # two scale steps apart


def test_too_many_differences_are_rejected():
    up, down = np.nextafter(np.float32(2.5), np.float32(3)), np.nextafter(np.float32(2.5), np.float32(2))
    y_dev = np.tile(_group([4.0, up, up, up]), (4, 1))
    y_ref = np.tile(_group([4.0, down, down, down]), (4, 1))
    with pytest.raises(AssertionError):
        _check(y_dev, y_ref)                                    # 12 of 128 codes
    assert _check(y_dev, y_ref, max_fraction=0.1) == (12, 0)


def test_per_element_gemm_bound_is_the_sum_of_magnitudes():
    rng = np.random.default_rng(5)
    ac = rng.integers(0, 256, size=(3, 32)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(2, 32)).astype(np.uint8)
    asc = rng.integers(120, 130, size=(3, 2)).astype(np.uint8)
    bsc = rng.integers(120, 130, size=(2, 2)).astype(np.uint8)
    bound = per_element_gemm_bound(ac, asc, bc, bsc, mxfp4.dequantize)
    a, b = mxfp4.dequantize(ac, asc), mxfp4.dequantize(bc, bsc)
    for t in range(3):
        for n in range(2):
            assert bound[t, n] == sum(abs(a[t, k]) * abs(b[n, k]) for k in range(64))
            assert abs(sum(a[t, k] * b[n, k] for k in range(64))) <= bound[t, n]
