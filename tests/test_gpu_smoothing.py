"""GPU parity of the smoothed form of Eq. 5: the smoothing diagonal merged into the rotation blocks on the
device, and the unchanged rotate+quantise / GEMM kernels run on the merged blocks, against the oracle's
definition (x / lambda, then rotate; w * lambda, then rotate)."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear, mxfp4, pipeline, rotation, smoothing
from helpers import (assert_codes_differ_only_at_boundaries, rel_fro, rotation_error_ratio, to_dev, to_dev_bf16,
                     untile_np)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


@pytest.mark.parametrize("K,shared", [(4096, False), (1184, False), (2048, True), (32, True)])
def test_fold_kernel_matches_the_oracle(env, K, shared):
    torch, duqpp = env
    R = wl.make_rotation_blocks(f"gpu-fold-{K}", 1 if shared else K // 32)
    lam = wl.make_smoothing_scales(f"gpu-fold-{K}", K)
    Ra, Rw = duqpp.fold_smoothing(to_dev(R, torch), to_dev(lam, torch))
    torch.cuda.synchronize()
    Ra_ref, Rw_ref = smoothing.fold_into_rotation(R, lam)
    # one correctly rounded fp32 operation on the device, fp64 then one rounding in the oracle: the same value
    # except where the fp64 quotient sits within 2^-29 of a rounding boundary
    for got, ref in ((Ra.cpu().numpy(), Ra_ref), (Rw.cpu().numpy(), Rw_ref)):
        assert got.shape == ref.shape
        ulp = np.spacing(np.abs(ref))
        assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= ulp)
        assert np.mean(got != ref) < 1e-6
    np.testing.assert_array_equal(Rw.cpu().numpy(), Rw_ref)      # a product of two fp32 is exact in fp64


@pytest.mark.parametrize("T,N,K", [(70, 96, 1184), (16, 300, 4096), (300, 200, 2048)])
def test_smoothed_path_against_the_definition(env, T, N, K):
    torch, duqpp = env
    xb = wl.make_activations(f"gpu-smooth-{T}", T, K, (wl.OutlierSpec(8, 50.0), wl.OutlierSpec(2, 1000.0, 2)))
    wb = wl.make_weights(f"gpu-smooth-{T}", N, K, 0.02)
    R = wl.make_rotation_blocks(f"gpu-smooth-{T}", K // 32)
    xf, wf = wl.bf16_bits_to_f32(xb), wl.bf16_bits_to_f32(wb)
    lam = smoothing.smoothing_scales(xf, wf, 0.5).astype(np.float32)      # calibrated on the same synthetic data
    x, w = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch)
    Ra, Rw = duqpp.fold_smoothing(to_dev(R, torch), to_dev(lam, torch))
    print(f"[smoothing] T={T} N={N} K={K}", flush=True)

    # activations: rotated values against (x / lambda) . R in fp64, codes bit-exact on the device's own values
    ac, asc, yrot = duqpp.rotate_quantize(x, Ra, return_rotated=True)
    torch.cuda.synchronize()
    xs = xf.astype(np.float64) / lam.astype(np.float64)[None, :]
    assert rotation_error_ratio(yrot.cpu().numpy(), rotation.rotate(xs, R), xs) <= 1e-5
    c_ref, s_ref = mxfp4.quantize(yrot.cpu().numpy())
    np.testing.assert_array_equal(ac.cpu().numpy(), c_ref)
    np.testing.assert_array_equal(asc.cpu().numpy(), s_ref)
    # end to end (each side in its own precision): codes differ only at rounding boundaries
    c_def, s_def, y_def = pipeline.rotate_quantize(xb, R, lam=lam)
    assert_codes_differ_only_at_boundaries(ac.cpu().numpy(), asc.cpu().numpy(), c_def, s_def, y_def, xs)

    # weights, tiled, and the product
    bct, bst = duqpp.quantize_weights_tiled(w, Rw)
    act, ast = duqpp.rotate_quantize_tiled(x, Ra)
    y = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K)
    torch.cuda.synchronize()
    a_c, a_s, _, _ = untile_np(act.cpu().numpy(), ast.cpu().numpy(), T, K)
    np.testing.assert_array_equal(a_c, ac.cpu().numpy())
    b_c, b_s, _, _ = untile_np(bct.cpu().numpy(), bst.cpu().numpy(), N, K)
    cw_def, sw_def, yw_def = pipeline.quantize_weights(wb, R, lam=lam)
    assert_codes_differ_only_at_boundaries(b_c, b_s, cw_def, sw_def, yw_def,
                                           wf.astype(np.float64) * lam.astype(np.float64)[None, :])
    assert rel_fro(y.cpu().numpy(), linear.mxfp4_gemm(a_c, a_s, b_c, b_s)) <= 1e-5
    # ungraded sanity: smoothing + rotation + W4A4 still approximates X W^T
    exact = xf.astype(np.float64) @ wf.astype(np.float64).T
    e = rel_fro(y.cpu().numpy(), exact)
    print(f"[smoothing] W4A4 vs exact product, relative error {e:.3f}", flush=True)
    assert e < 0.5
