"""Pins of the oracle's smoothing step (paper Sec. 4.2, Eq. 3, and the smoothed form of Eq. 5).
CPU only.  What fixes it from outside: a hand-worked example, the balance property of the scaling rule,
the identity (X L^-1 R)(R^T L W) = X W, and the reduction to the unsmoothed path at L = I."""
import numpy as np
import pytest

import workloads as wl
from oracle import mxfp4, pipeline, rotation, smoothing


def _blockdiag(R, G):
    M = np.zeros((32 * G, 32 * G))
    for j in range(G):
        M[32 * j:32 * j + 32, 32 * j:32 * j + 32] = R[j if R.shape[0] == G else 0]
    return M


def test_scales_hand_worked():
    # two channels: column maxima of |X| are 4 and 9, of |W| 1 and 4; alpha = 1/2 gives sqrt(4/1), sqrt(9/4)
    x = np.array([[4.0, -1.0], [-2.0, 9.0], [0.5, 3.0]])
    w = np.array([[0.5, 4.0], [-1.0, 2.0]])
    np.testing.assert_allclose(smoothing.smoothing_scales(x, w, 0.5), [2.0, 1.5], rtol=1e-15)
    # alpha = 1 moves everything to the weights (lambda = max|X|), alpha = 0 nothing of X (lambda = 1 / max|W|)
    np.testing.assert_allclose(smoothing.smoothing_scales(x, w, 1.0), [4.0, 9.0], rtol=1e-15)
    np.testing.assert_allclose(smoothing.smoothing_scales(x, w, 0.0), [1.0, 0.25], rtol=1e-15)


@pytest.mark.parametrize("alpha", [0.3, 0.5, 0.8])
def test_scaling_rule_balances_channel_maxima(alpha):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((50, 64)) * np.exp(rng.standard_normal(64) * 2)   # strong per-channel spread
    w = rng.standard_normal((40, 64)) * 0.02
    lam = smoothing.smoothing_scales(x, w, alpha)
    ax, aw = np.max(np.abs(x), axis=0), np.max(np.abs(w), axis=0)
    xs, ws = smoothing.apply(x, lam, inverse=True), smoothing.apply(w, lam, inverse=False)
    np.testing.assert_allclose(np.max(np.abs(xs), axis=0), ax ** (1 - alpha) * aw ** (1 - alpha), rtol=1e-12)
    np.testing.assert_allclose(np.max(np.abs(ws), axis=0), ax ** alpha * aw ** alpha, rtol=1e-12)
    if alpha == 0.5:      # the two operands end up with the same maximum in every channel
        np.testing.assert_allclose(np.max(np.abs(xs), axis=0), np.max(np.abs(ws), axis=0), rtol=1e-12)


@pytest.mark.parametrize("shared", [False, True])
def test_smoothed_rotated_product_is_lossless(shared):
    """(X L^-1 R^)(R^T L W) = X W (Eq. 5), for the definition and for the merged blocks alike.  Scaling by the
    output channel of a block instead of its input channel, or swapping the two factors, breaks it."""
    rng = np.random.default_rng(11)
    T, N, K = 7, 5, 96
    G = K // 32
    x, w = rng.standard_normal((T, K)), rng.standard_normal((N, K))
    lam = np.exp(rng.uniform(-2, 2, K))
    R = wl.make_rotation_blocks("smooth-lossless", 1 if shared else G).astype(np.float64)
    exact = x @ w.T
    Rhat = _blockdiag(R, G)
    # the definition
    xa = smoothing.apply(x, lam, inverse=True) @ Rhat
    wa = smoothing.apply(w, lam, inverse=False) @ Rhat
    assert np.linalg.norm(xa @ wa.T - exact) <= 1e-6 * np.linalg.norm(exact)      # R is orthogonal to fp32 accuracy
    # the merged blocks (fp32 entries)
    Ra, Rw = smoothing.fold_into_rotation(R, lam)
    assert Ra.shape == (G, 32, 32) and Ra.dtype == np.float32
    xb, wb = x @ _blockdiag(Ra.astype(np.float64), G), w @ _blockdiag(Rw.astype(np.float64), G)
    assert np.linalg.norm(xb @ wb.T - exact) <= 1e-6 * np.linalg.norm(exact)
    np.testing.assert_allclose(xb, xa, rtol=0, atol=2e-7 * np.max(np.abs(xa)))
    # planted mistakes
    Rbad = np.stack([R[j if not shared else 0] / lam[32 * j:32 * j + 32][None, :] for j in range(G)])   # scaled by c, not r
    assert np.linalg.norm((x @ _blockdiag(Rbad, G)) @ wb.T - exact) > 1e-2 * np.linalg.norm(exact)
    assert np.linalg.norm((x @ _blockdiag(Rw.astype(np.float64), G)) @ wb.T - exact) > 1e-2 * np.linalg.norm(exact)


def test_merged_block_entries():
    R = wl.make_rotation_blocks("smooth-entries", 2)
    lam = np.arange(1, 65, dtype=np.float64) / 8.0
    Ra, Rw = smoothing.fold_into_rotation(R, lam)
    for (j, r, c) in [(0, 0, 0), (0, 31, 5), (1, 3, 31), (1, 17, 17)]:
        assert Ra[j, r, c] == np.float32(np.float64(R[j, r, c]) / lam[32 * j + r])
        assert Rw[j, r, c] == np.float32(np.float64(R[j, r, c]) * lam[32 * j + r])
    # a shared block expands to one block per group, each with its own slice of lambda
    Ra1, Rw1 = smoothing.fold_into_rotation(R[:1], lam)
    np.testing.assert_array_equal(Ra1[0], Ra[0])
    assert Ra1.shape == (2, 32, 32) and Rw1[1, 4, 9] == np.float32(np.float64(R[0, 4, 9]) * lam[36])


def test_unit_lambda_is_the_unsmoothed_path():
    T, K = 9, 128
    xb = wl.make_activations("smooth-unit", T, K, (wl.OutlierSpec(2, 50.0),))
    R = wl.make_rotation_blocks("smooth-unit", K // 32)
    one = np.ones(K)
    Ra, Rw = smoothing.fold_into_rotation(R, one)
    np.testing.assert_array_equal(Ra, R)
    np.testing.assert_array_equal(Rw, R)
    c0, s0, y0 = pipeline.rotate_quantize(xb, R)
    c1, s1, y1 = pipeline.rotate_quantize(xb, R, lam=one)
    np.testing.assert_array_equal(y0, y1)
    np.testing.assert_array_equal(c0, c1)
    np.testing.assert_array_equal(s0, s1)


def test_pipeline_with_lambda_follows_the_definition_and_the_merged_blocks():
    T, N, K = 12, 6, 160
    xb = wl.make_activations("smooth-pipe", T, K, (wl.OutlierSpec(3, 50.0),))
    wb = wl.make_weights("smooth-pipe", N, K, 0.02)
    R = wl.make_rotation_blocks("smooth-pipe", K // 32)
    xf, wf = wl.bf16_bits_to_f32(xb), wl.bf16_bits_to_f32(wb)
    lam = smoothing.smoothing_scales(xf, wf, 0.5)
    c, s, y = pipeline.rotate_quantize(xb, R, lam=lam)
    y_def = rotation.rotate(xf.astype(np.float64) / lam[None, :], R)
    np.testing.assert_array_equal(y, y_def)
    c2, s2 = mxfp4.quantize(y_def)
    np.testing.assert_array_equal(c, c2)
    np.testing.assert_array_equal(s, s2)
    # the same operand from the merged blocks: equal up to the fp32 rounding of their entries
    Ra, Rw = smoothing.fold_into_rotation(R, lam)
    y_m = rotation.rotate(xf, Ra)
    nrm = np.linalg.norm((xf.astype(np.float64) / lam).reshape(T, K // 32, 32), axis=-1)
    err = np.abs(y_m.astype(np.float64) - y_def).reshape(T, K // 32, 32).max(axis=-1)
    assert np.all(err <= 1e-6 * nrm)
    cw, sw, yw = pipeline.quantize_weights(wb, R, lam=lam)
    np.testing.assert_array_equal(yw, rotation.rotate(wf.astype(np.float64) * lam[None, :], R))
    # the smoothed, rotated, quantised product still approximates X W^T (ungraded sanity)
    approx = mxfp4.dequantize(c, s) @ mxfp4.dequantize(cw, sw).T
    exact = xf.astype(np.float64) @ wf.astype(np.float64).T
    assert np.linalg.norm(approx - exact) < 0.5 * np.linalg.norm(exact)
