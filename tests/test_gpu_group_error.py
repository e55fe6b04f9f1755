"""GPU parity of duqpp_group_error: the per-group normalised quantisation error of Sec. 4.1 (the statistic of Fig. 1),
||Q(y) - y||_2 / ||y||_2 per group of 32 with y the rotated group (Eq. 4) and Q the quantiser of Eq. 2.  The oracle
computes it in fp64 from the device's own fp32 rotated values (as the quantiser's parity does), so the two sides
differ by the rounding of the ratio to fp32 only."""
import numpy as np
import pytest

import workloads as wl
from oracle import mxfp4, pipeline
from helpers import to_dev, to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


def _check(err, mean, want):
    ok = want >= 0
    np.testing.assert_array_equal(err[~ok], -1.0)
    assert np.all(err[ok] >= 0)
    np.testing.assert_allclose(err[ok], want[ok], rtol=2e-7, atol=1e-12)       # one rounding to fp32
    want_mean = float(np.mean(want[ok])) if ok.any() else 0.0
    assert abs(mean - want_mean) <= 1e-7 * max(want_mean, 1e-30) + 1e-12


@pytest.mark.parametrize("T,K,shared", [(77, 1184, 0), (300, 2048, 1), (2048, 4096, 0), (33, 32, 0)])
def test_group_error_of_rotated_groups(env, T, K, shared):
    torch, duqpp = env
    name = f"gpu-gerr-{T}-{K}-{shared}"
    xb = wl.make_activations(name, T, K, (wl.OutlierSpec(min(4, K // 8), 50.0), wl.OutlierSpec(1, 1000.0, 1)))
    xb[min(3, T - 1), :32] = 0                               # a group of zeros: no ratio
    if K >= 64:
        xb[0, K - 32:] = 0x8000                              # and one of negative zeros
    R = wl.make_rotation_blocks(name, 1 if shared else K // 32)
    x, Rd = to_dev_bf16(xb, torch), to_dev(R, torch)
    print(f"[group error] rotated T={T} K={K} shared={shared}", flush=True)
    err, mean = duqpp.group_error(x, Rd)
    _, _, yrot = duqpp.rotate_quantize(x, Rd, return_rotated=True)
    torch.cuda.synchronize()
    y = yrot.cpu().numpy()
    c, s = mxfp4.quantize(y)
    want = pipeline.per_group_normalised_errors(y, c, s)
    assert want[min(3, T - 1), 0] == -1.0
    _check(err.cpu().numpy(), mean, want)


@pytest.mark.parametrize("T,K,pad", [(100, 1024, 0), (65, 2080, 8)])
def test_group_error_without_rotation(env, T, K, pad):
    """R = NULL: the statistic of the activations themselves (the figure's unrotated setting), token rows possibly
    strided."""
    torch, duqpp = env
    name = f"gpu-gerr-plain-{T}-{K}"
    xb = wl.make_activations(name, T, K + pad, (wl.OutlierSpec(8, 50.0),))
    xb[5, 64:96] = 0
    x = to_dev_bf16(xb, torch)[:, :K]
    print(f"[group error] unrotated T={T} K={K} ldx={K + pad}", flush=True)
    err, mean = duqpp.group_error(x, None)
    err_only, none = duqpp.group_error(x, None, return_mean=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(err, err_only)
    xf = wl.bf16_bits_to_f32(np.ascontiguousarray(xb[:, :K]))
    c, s = mxfp4.quantize(xf)
    want = pipeline.per_group_normalised_errors(xf, c, s)
    assert want[5, 2] == -1.0
    _check(err.cpu().numpy(), mean, want)


def test_group_error_orders_the_settings_as_fig_1_does(env):
    """Ungraded sanity on the synthetic stand-in for a down-projection input (no value in the paper pins the numbers):
    over the groups that hold an outlier channel a rotation lowers the mean normalised error, the ordering of Fig. 1;
    and the block that the greedy construction of Sec. 4.2 builds lowers it on the group it was built from."""
    torch, duqpp = env
    T, K = 512, 4096
    xb = wl.make_activations("gpu-gerr-fig1", T, K, (wl.OutlierSpec(8, 50.0),))
    x = to_dev_bf16(xb, torch)
    before, _ = duqpp.group_error(x, None)
    R = to_dev(wl.make_rotation_blocks("gpu-gerr-fig1", K // 32), torch)
    after, _ = duqpp.group_error(x, R)
    q = torch.from_numpy(wl.make_orthogonal_steps("gpu-gerr-fig1", 128)).to(x.device)
    Rc, block, kept = duqpp.construct_rotation(x, q)
    built, _ = duqpp.group_error(x, Rc)
    torch.cuda.synchronize()
    xf = np.abs(wl.bf16_bits_to_f32(xb)).mean(axis=0).reshape(K // 32, 32)
    groups = np.where(xf.max(axis=1) > 10)[0]                 # groups that hold an outlier channel
    assert len(groups) >= 1 and block in groups
    b, a = before.cpu().numpy()[:, groups].mean(), after.cpu().numpy()[:, groups].mean()
    bb, cb = before.cpu().numpy()[:, block].mean(), built.cpu().numpy()[:, block].mean()
    print(f"[group error] outlier groups: unrotated {b:.4f}, random orthogonal blocks {a:.4f}; "
          f"group {block}: unrotated {bb:.4f}, constructed block ({kept} steps kept) {cb:.4f}", flush=True)
    assert a < b
    assert cb < bb
