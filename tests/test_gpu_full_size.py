"""GPU parity at the headline size (LLaMA-3-8B down_proj prefill: T=2048, K=14336, N=4096) in the
launch configuration the bench times.  Rotate+quantise is checked in full; the GEMM on sampled output
rows and columns the oracle computes one by one."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear, mxfp4, rotation
from helpers import bf16_dev_to_bits, rel_fro, rotation_error_ratio, to_dev, to_dev_bf16, untile_np

pytestmark = pytest.mark.gpu


def test_headline_config_full_size():
    import torch

    import paper_2604_17789_amd as duqpp
    cfg = wl.CONFIGS["c2_8b_down_prefill"]
    T, K, N = cfg["T"], cfg["K"], cfg["N"]
    print(f"[full] generating T={T} K={K} N={N}", flush=True)
    xb = wl.make_activations("c2", T, K, cfg["outliers"])
    wb = wl.make_weights("c2", N, K, cfg["w_std"])
    R = wl.make_rotation_blocks("c2", K // 32)
    x, w, Rd = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch), to_dev(R, torch)
    print("[full] device: quantize_weights, rotate_quantize, gemm (bf16 and fp32), rotq_gemm", flush=True)
    bc, bs = duqpp.quantize_weights(w, Rd)
    ac, asc, yrot = duqpp.rotate_quantize(x, Rd, return_rotated=True)
    y16 = duqpp.mxfp4_gemm(ac, asc, bc, bs, out_dtype=1)
    y32 = duqpp.mxfp4_gemm(ac, asc, bc, bs, out_dtype=0)
    yf = duqpp.rotq_gemm(x, Rd, bc, bs, out_dtype=1)
    torch.cuda.synchronize()
    ac_h, as_h, yrot_h = ac.cpu().numpy(), asc.cpu().numpy(), yrot.cpu().numpy()

    print("[full] oracle: rotation", flush=True)
    xf = wl.bf16_bits_to_f32(xb)
    assert rotation_error_ratio(yrot_h, rotation.rotate(xf, R), xf) <= 1e-5
    print("[full] oracle: quantiser on the device's rotated values", flush=True)
    c_ref, s_ref = mxfp4.quantize(yrot_h)
    np.testing.assert_array_equal(as_h, s_ref)
    np.testing.assert_array_equal(ac_h, c_ref)
    del c_ref, s_ref, yrot_h

    print("[full] oracle: sampled GEMM rows and columns", flush=True)
    rng = np.random.default_rng(2048)
    rows = np.sort(rng.choice(T, 64, replace=False))
    cols = np.sort(rng.choice(N, 64, replace=False))
    bc_h, bs_h = bc.cpu().numpy(), bs.cpu().numpy()
    y32_h = y32.cpu().numpy()
    ref_rows = linear.mxfp4_gemm(ac_h[rows], as_h[rows], bc_h, bs_h)
    ref_cols = linear.mxfp4_gemm(ac_h, as_h, bc_h[cols], bs_h[cols])
    assert rel_fro(y32_h[rows], ref_rows) <= 1e-5
    assert rel_fro(y32_h[:, cols], ref_cols) <= 1e-5
    y16_h = bf16_dev_to_bits(y16)
    np.testing.assert_array_equal(y16_h, linear.round_to_bf16_bits(y32_h))
    assert torch.equal(y16, yf)

    # the tiled path, exactly as the bench launches it: same codes in tiled positions, same product
    print("[full] device: tiled path", flush=True)
    bct, bst = duqpp.quantize_weights_tiled(w, Rd)
    act, ast = duqpp.rotate_quantize_tiled(x, Rd)
    y16_t = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=1)
    y32_t = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=0)
    yf_t = duqpp.rotq_gemm_tiled(x, Rd, bct, bst, N, out_dtype=1)
    torch.cuda.synchronize()
    a_c, a_s, pc, ps = untile_np(act.cpu().numpy(), ast.cpu().numpy(), T, K)
    np.testing.assert_array_equal(a_c, ac_h)
    np.testing.assert_array_equal(a_s, as_h)
    assert np.all(pc == 0) and np.all(ps == 127)
    b_c, b_s, _, _ = untile_np(bct.cpu().numpy(), bst.cpu().numpy(), N, K)
    np.testing.assert_array_equal(b_c, bc_h)
    np.testing.assert_array_equal(b_s, bs_h)
    y32_th = y32_t.cpu().numpy()
    assert rel_fro(y32_th[rows], ref_rows) <= 1e-5
    assert rel_fro(y32_th[:, cols], ref_cols) <= 1e-5
    np.testing.assert_array_equal(bf16_dev_to_bits(y16_t), linear.round_to_bf16_bits(y32_th))
    assert torch.equal(y16_t, yf_t)
