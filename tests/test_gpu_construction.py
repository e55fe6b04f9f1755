"""GPU parity of the greedy construction of the shared rotation block (Sec. 4.2, steps (1)-(3)) against the CPU
oracle: the same block, the same number of kept steps, the same peaks and the same matrix, bit for bit (both sides
work in fp64 in the same operation order, so the argmax / argmin decisions cannot differ); then the constructed
block on the online path.  The construction itself is this build's reading of the paper's sketch (parity unpinned
beyond the oracle's own pins)."""
import numpy as np
import pytest

import workloads as wl
from oracle import construction, mxfp4, rotation
from helpers import rotation_error_ratio, to_dev, to_dev_bf16, untile_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


CASES = [
    # T, K, steps, outliers
    (300, 512, 24, (wl.OutlierSpec(3, 1000.0, 4), wl.OutlierSpec(6, 20.0))),   # massive + normal outliers, ragged T
    (64, 32, 5, (wl.OutlierSpec(2, 50.0),)),                                    # a single block, one workgroup of rows
    (1, 4096, 3, (wl.OutlierSpec(4, 50.0),)),                                   # one token
    (2048, 14336, 128, (wl.OutlierSpec(4, 1000.0, 8), wl.OutlierSpec(32, 20.0))),   # the 8B down_proj input, 128 steps
    (777, 1184, 0, (wl.OutlierSpec(4, 50.0),)),                                 # no step: the identity
]


@pytest.mark.parametrize("T,K,steps,outliers", CASES)
def test_construct_rotation_matches_oracle(env, T, K, steps, outliers):
    torch, duqpp = env
    name = f"gpu-cons-{T}-{K}"
    xb = wl.make_activations(name, T, K, outliers)
    q = wl.make_orthogonal_steps(name, steps)
    print(f"[construct] T={T} K={K} steps={steps}", flush=True)
    R, block, kept, peaks = duqpp.construct_rotation(to_dev_bf16(xb, torch), to_dev(q, torch), return_peaks=True)
    torch.cuda.synchronize()
    ref = construction.greedy_rotation(wl.bf16_bits_to_f32(xb), q)
    assert block == ref["block"] and kept == ref["steps"]
    np.testing.assert_array_equal(peaks.cpu().numpy(), ref["peaks"])
    np.testing.assert_array_equal(R.cpu().numpy()[0], ref["R"])
    Rd = R.cpu().numpy()[0].astype(np.float64)
    assert np.max(np.abs(Rd.T @ Rd - np.eye(32))) < 1e-6
    assert ref["peaks"][kept] <= ref["peaks"][0]


def test_constructed_block_on_the_online_path(env):
    """The constructed matrix goes in as the one shared block (n_rblocks = 1): rotation within tolerance of the
    oracle's, codes and scales bit-exact on the device's own rotated values, and the peak of the block it was built
    from falls as the construction reported."""
    torch, duqpp = env
    T, K = 512, 2048
    xb = wl.make_activations("gpu-cons-path", T, K, (wl.OutlierSpec(3, 1000.0, 6), wl.OutlierSpec(8, 20.0)))
    q = wl.make_orthogonal_steps("gpu-cons-path", 64)
    x = to_dev_bf16(xb, torch)
    R, block, kept, peaks = duqpp.construct_rotation(x, to_dev(q, torch), return_peaks=True)
    codes, scales, yrot = duqpp.rotate_quantize(x, R, return_rotated=True)
    ct, st = duqpp.rotate_quantize_tiled(x, R)
    torch.cuda.synchronize()
    xf = wl.bf16_bits_to_f32(xb)
    yr = yrot.cpu().numpy()
    assert rotation_error_ratio(yr, rotation.rotate(xf, R.cpu().numpy()), xf) <= 1e-5
    c_ref, s_ref = mxfp4.quantize(yr)
    np.testing.assert_array_equal(codes.cpu().numpy(), c_ref)
    np.testing.assert_array_equal(scales.cpu().numpy(), s_ref)
    c_t, s_t, _, _ = untile_np(ct.cpu().numpy(), st.cpu().numpy(), T, K)
    np.testing.assert_array_equal(c_t, c_ref)
    pk = peaks.cpu().numpy()
    assert kept >= 1 and pk[kept] < 0.5 * pk[0]
    got = float(np.max(np.abs(yr[:, 32 * block:32 * block + 32])))
    assert abs(got - pk[kept]) <= 1e-5 * pk[0]                  # fp32 online rotation against the fp64 search state


def test_construct_rotation_rejections(env):
    torch, duqpp = env
    x = to_dev_bf16(wl.make_activations("gpu-cons-rej", 8, 64, ()), torch)
    q = to_dev(wl.make_orthogonal_steps("gpu-cons-rej", 2), torch)
    small = torch.empty(256, dtype=torch.uint8, device=x.device)
    with pytest.raises(duqpp.DuqppError):
        duqpp.construct_rotation(x, q, workspace=small)
    with pytest.raises(ValueError):
        duqpp.construct_rotation(x, q[:, :30])
