"""Pins of the oracle's greedy construction of the shared rotation block (Sec. 4.2, steps (1)-(3)).

The paper prints no number for this construction and gives it as a sketch: PARITY UNPINNED beyond what the
mathematics fixes.  The pins below are invariants, closed forms and an independent restatement through library
matrix products; each planted mistake (a transposed step matrix, a dropped exchange, a wrong channel, a step
kept too late) fails at least one of them."""
import numpy as np
import pytest

import workloads as wl
from oracle import construction as C
from oracle import mxfp4, pipeline, rotation


def _calib(name, T=256, K=256, massive=True):
    specs = (wl.OutlierSpec(3, 1000.0, 4), wl.OutlierSpec(6, 20.0)) if massive else (wl.OutlierSpec(6, 20.0),)
    return wl.bf16_bits_to_f32(wl.make_activations(name, T, K, specs)).astype(np.float64)


def test_hadamard_closed_form():
    H = C.hadamard()
    assert np.all(H[0] == C.S) and np.all(H[:, 0] == C.S)            # uniform first row and column
    assert np.array_equal(H, H.T)
    assert np.max(np.abs(H @ H.T - np.eye(32))) < 1e-15
    assert H[5, 3] == -C.S and H[5, 2] == C.S                        # popcount(5 & 3) = 1, popcount(5 & 2) = 0
    np.testing.assert_array_equal(H.astype(np.float32), wl.hadamard_blocks(1)[0])


@pytest.mark.parametrize("d", [0, 1, 17, 31])
def test_step_matrix_is_orthogonal_and_spreads_channel_d(d):
    q = wl.make_orthogonal_steps("pin-step", 3)
    Rt = C.step_matrix(d, q[1])
    assert np.max(np.abs(Rt.T @ Rt - np.eye(32))) < 1e-14
    assert np.max(np.abs(Rt @ Rt.T - np.eye(32))) < 1e-14
    # a spike in channel d: coordinate d of the image is a / sqrt(32), and the image has the spike's norm
    y = (7.0 * np.eye(32)[d]) @ Rt
    assert abs(y[d] - 7.0 * C.S) < 1e-15
    assert abs(np.linalg.norm(y) - 7.0) < 1e-13
    # with Q' = I the spike is spread evenly over all 32 channels: |y_c| = a / sqrt(32) for every c
    y = (7.0 * np.eye(32)[d]) @ C.step_matrix(d, np.eye(31))
    np.testing.assert_allclose(np.abs(y), 7.0 * C.S, rtol=0, atol=1e-15)
    # restated through library products: E_d H diag(1, Q') E_d
    E = np.eye(32)
    E[[0, d]] = E[[d, 0]]
    Q = np.eye(32)
    Q[1:, 1:] = q[1]
    np.testing.assert_allclose(Rt, E @ C.hadamard() @ Q @ E, rtol=0, atol=1e-15)


def test_channel_and_block_selection():
    x = np.zeros((8, 96))
    x[3, 40] = -9.0
    x[5, 70] = 9.0                                                    # equal magnitudes: the smaller block index wins
    x[2, 5] = 8.0
    assert C.select_block(x) == 1
    out = C.greedy_rotation(x, np.eye(31)[None])
    assert out["block"] == 1 and out["channels"] == [8]               # channel 40 is channel 8 of block 1
    # one step with Q' = I spreads the single spike evenly: peak 9 -> 9 / sqrt(32), kept
    assert out["steps"] == 1
    np.testing.assert_allclose(out["peaks"], [9.0, 9.0 * C.S], rtol=0, atol=1e-15)
    z = np.abs(out["Z"][3])
    np.testing.assert_allclose(z, 9.0 * C.S, rtol=0, atol=1e-15)
    # ties between channels: the smaller channel index
    x = np.zeros((4, 32))
    x[0, 20] = 3.0
    x[1, 11] = -3.0
    assert C.greedy_rotation(x, np.eye(31)[None])["channels"] == [11]


def test_kept_step_minimises_the_peak_and_identity_is_allowed():
    x = _calib("pin-min")
    q = wl.make_orthogonal_steps("pin-min", 40)
    out = C.greedy_rotation(x, q)
    peaks = out["peaks"]
    assert len(peaks) == 41 and out["steps"] == int(np.argmin(peaks))
    assert peaks[out["steps"]] <= peaks[0]                            # never worse than no rotation
    assert np.all(peaks[:out["steps"]] > peaks[out["steps"]])         # the first minimum
    assert peaks[out["steps"]] < 0.5 * peaks[0]                       # massive outliers are dispersed
    # data whose peak no rotation lowers: all |x| equal in one channel pattern H already spreads -> identity kept
    flat = np.full((4, 32), 1.0)
    flat[:, 1::2] = -1.0
    out = C.greedy_rotation(flat, wl.make_orthogonal_steps("pin-flat", 5))
    assert out["steps"] == 0 and np.array_equal(out["R"], np.eye(32, dtype=np.float32))


def test_search_state_equals_x_times_r_and_r_is_orthogonal():
    x = _calib("pin-state", T=300, K=512)
    q = wl.make_orthogonal_steps("pin-state", 30)
    out = C.greedy_rotation(x, q)
    b, R = out["block"], out["R"].astype(np.float64)
    assert np.max(np.abs(R.T @ R - np.eye(32))) < 1e-6                # the orthogonality bar of every rotation block
    xb = x[:, 32 * b:32 * b + 32]
    # the state of the search is X . R^(t*): independent restatement through library products of the step matrices
    P = np.eye(32)
    for t in range(out["steps"]):
        P = P @ C.step_matrix(out["channels"][t], q[t])
    np.testing.assert_allclose(out["Z"], xb @ P, rtol=0, atol=1e-9 * np.max(np.abs(xb)))
    np.testing.assert_allclose(R, P, rtol=0, atol=1e-7)
    assert abs(np.max(np.abs(xb @ P)) - out["peaks"][out["steps"]]) < 1e-9 * out["peaks"][0]
    # planted mistakes: the transposed step matrix, or the exchange left out, break that identity
    Pt = np.eye(32)
    Pn = np.eye(32)
    for t in range(out["steps"]):
        Pt = Pt @ C.step_matrix(out["channels"][t], q[t]).T
        Pn = Pn @ C.step_matrix(0, q[t])
    assert np.max(np.abs(out["Z"] - xb @ Pt)) > 1e-3 * np.max(np.abs(xb))
    assert np.max(np.abs(out["Z"] - xb @ Pn)) > 1e-3 * np.max(np.abs(xb))
    # every recorded channel is the argmax of the state before its step
    Zt = xb.copy()
    for t in range(len(out["channels"])):
        assert out["channels"][t] == int(np.argmax(np.max(np.abs(Zt), axis=0)))
        Zt = Zt @ C.step_matrix(out["channels"][t], q[t])


def test_constructed_block_is_lossless_and_usable_as_shared_rotation():
    """(X R^)(W R^)^T = X W^T with the constructed block shared by all groups (Eq. 5).  Sanity only (no value in
    the paper pins it): with whole outlier channels (x50) in the data, Fig. 1's per-group normalised MXFP4 error of
    the block that held the largest outlier falls under the constructed rotation."""
    x = wl.bf16_bits_to_f32(wl.make_activations("pin-loss", 256, 256, (wl.OutlierSpec(8, 50.0),))).astype(np.float64)
    w = wl.bf16_bits_to_f32(wl.make_weights("pin-loss", 48, 256, 0.02)).astype(np.float64)
    out = C.greedy_rotation(x, wl.make_orthogonal_steps("pin-loss", 64))
    R1 = out["R"][None]
    xr = rotation.rotate(x, R1).astype(np.float64)
    wr = rotation.rotate(w, R1).astype(np.float64)
    ref = x @ w.T
    assert np.linalg.norm(xr @ wr.T - ref) <= 1e-5 * np.linalg.norm(ref)
    b = out["block"]

    def block_error(v):
        blk = np.ascontiguousarray(v[:, 32 * b:32 * b + 32].astype(np.float32))
        c, s = mxfp4.quantize(blk)
        return pipeline.per_group_normalised_error(blk, c, s)

    assert block_error(xr) < 0.9 * block_error(x)
