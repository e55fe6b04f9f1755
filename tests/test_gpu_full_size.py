"""GPU parity at the headline size (LLaMA-3-8B down_proj prefill: T=2048, K=14336, N=4096) in the
launch configuration the bench times.  Rotate+quantise is checked in full; the GEMM on sampled output
rows and columns the oracle computes one by one."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear, mxfp4, rotation
from helpers import (assert_codes_differ_only_at_boundaries, bf16_dev_to_bits, per_element_gemm_bound, rel_fro,
                     rotation_error_ratio, to_dev, to_dev_bf16, untile_np)

ELEM_TOL = 1e-5      # per sampled output: |y - ref| <= ELEM_TOL * sum_k |a| |b| (fp32 accumulation of exact products)

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
    y_ref = rotation.rotate(xf, R)
    assert rotation_error_ratio(yrot_h, y_ref, xf) <= 1e-5
    print("[full] oracle: quantiser on the device's rotated values", flush=True)
    c_ref, s_ref = mxfp4.quantize(yrot_h)
    np.testing.assert_array_equal(as_h, s_ref)
    np.testing.assert_array_equal(ac_h, c_ref)
    del c_ref, s_ref, yrot_h
    print("[full] oracle: quantiser on its own rotated values (differences only at rounding boundaries)", flush=True)
    c_own, s_own = mxfp4.quantize(y_ref)
    n_c, n_s = assert_codes_differ_only_at_boundaries(ac_h, as_h, c_own, s_own, y_ref, xf)
    print(f"[full] {n_c} of {T * K} codes and {n_s} of {T * K // 32} scales differ end to end", flush=True)
    del c_own, s_own, y_ref

    print("[full] oracle: sampled GEMM rows and columns", flush=True)
    rng = np.random.default_rng(2048)
    rows = np.sort(rng.choice(T, 64, replace=False))
    cols = np.sort(rng.choice(N, 64, replace=False))
    bc_h, bs_h = bc.cpu().numpy(), bs.cpu().numpy()
    y32_h = y32.cpu().numpy()
    ref_rows = linear.mxfp4_gemm(ac_h[rows], as_h[rows], bc_h, bs_h)
    ref_cols = linear.mxfp4_gemm(ac_h, as_h, bc_h[cols], bs_h[cols])
    bound_rows = ELEM_TOL * per_element_gemm_bound(ac_h[rows], as_h[rows], bc_h, bs_h, mxfp4.dequantize)
    bound_cols = ELEM_TOL * per_element_gemm_bound(ac_h, as_h, bc_h[cols], bs_h[cols], mxfp4.dequantize)
    assert rel_fro(y32_h[rows], ref_rows) <= 1e-5
    assert rel_fro(y32_h[:, cols], ref_cols) <= 1e-5
    assert np.all(np.abs(y32_h[rows] - ref_rows) <= bound_rows)
    assert np.all(np.abs(y32_h[:, cols] - ref_cols) <= bound_cols)
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
    assert np.all(np.abs(y32_th[rows] - ref_rows) <= bound_rows)
    assert np.all(np.abs(y32_th[:, cols] - ref_cols) <= bound_cols)
    np.testing.assert_array_equal(bf16_dev_to_bits(y16_t), linear.round_to_bf16_bits(y32_th))
    assert torch.equal(y16_t, yf_t)


def _tiled_path_sampled(name, T, K, N, outliers, w_std, out_dtype, n_rows=48, n_cols=48):
    """The tiled path exactly as the bench launches it, at full size: rotate+quantise checked through the
    quantiser on sampled rows (rotation against fp64, codes bit-exact on the device's own rotated values via
    the row-major call, which must agree with the tiled call), the product on sampled rows and columns."""
    import torch

    import paper_2604_17789_amd as duqpp
    print(f"[full] {name}: generating T={T} K={K} N={N}", flush=True)
    xb = wl.make_activations(name, T, K, outliers)
    wb = wl.make_weights(name, N, K, w_std)
    R = wl.make_rotation_blocks(name, K // 32)
    x, w, Rd = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch), to_dev(R, torch)
    del wb
    print(f"[full] {name}: device", flush=True)
    bct, bst = duqpp.quantize_weights_tiled(w, Rd)
    act, ast = duqpp.rotate_quantize_tiled(x, Rd)
    y = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=out_dtype)
    # the fp32 result of the same kernel at the same shape: graded at 1e-5; a bf16 result must be its rounding
    y32 = y if out_dtype == 0 else duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=0)
    assert duqpp.gemm_kernel_for(T, N, K, 0) == duqpp.gemm_kernel_for(T, N, K, out_dtype)
    torch.cuda.synchronize()
    rng = np.random.default_rng(T + N)
    rows = np.sort(rng.choice(T, n_rows, replace=False))
    cols = np.sort(rng.choice(N, n_cols, replace=False))

    # rotate+quantise on the sampled token rows: the row-major call on just those rows gives the same codes
    # as the tiled call on all rows (rows are independent), plus the rotated values the quantiser saw
    xs = x[torch.from_numpy(rows).to(x.device)].contiguous()
    c_rm, s_rm, yrot = duqpp.rotate_quantize(xs, Rd, return_rotated=True)
    torch.cuda.synchronize()
    a_c, a_s, pc, ps = untile_np(act.cpu().numpy(), ast.cpu().numpy(), T, K)
    assert np.all(pc == 0) and np.all(ps == 127)
    np.testing.assert_array_equal(a_c[rows], c_rm.cpu().numpy())
    np.testing.assert_array_equal(a_s[rows], s_rm.cpu().numpy())
    xf = wl.bf16_bits_to_f32(xb[rows])
    y_own = rotation.rotate(xf, R)
    assert rotation_error_ratio(yrot.cpu().numpy(), y_own, xf) <= 1e-5
    c_ref, s_ref = mxfp4.quantize(yrot.cpu().numpy())
    np.testing.assert_array_equal(c_rm.cpu().numpy(), c_ref)
    np.testing.assert_array_equal(s_rm.cpu().numpy(), s_ref)
    c_own, s_own = mxfp4.quantize(y_own)                   # end to end: differences only at rounding boundaries
    assert_codes_differ_only_at_boundaries(a_c[rows], a_s[rows], c_own, s_own, y_own, xf)

    print(f"[full] {name}: oracle on sampled rows and columns", flush=True)
    b_c, b_s, _, _ = untile_np(bct.cpu().numpy(), bst.cpu().numpy(), N, K)
    ri, ci = torch.from_numpy(rows).to(y32.device), torch.from_numpy(cols).to(y32.device)
    y_rows, y_cols = y32[ri].cpu().numpy(), y32[:, ci].cpu().numpy()
    ref_rows = linear.mxfp4_gemm(a_c[rows], a_s[rows], b_c, b_s)
    ref_cols = linear.mxfp4_gemm(a_c, a_s, b_c[cols], b_s[cols])
    assert rel_fro(y_rows, ref_rows) <= 1e-5
    assert rel_fro(y_cols, ref_cols) <= 1e-5
    assert np.all(np.abs(y_rows - ref_rows) <= ELEM_TOL * per_element_gemm_bound(a_c[rows], a_s[rows], b_c, b_s, mxfp4.dequantize))
    assert np.all(np.abs(y_cols - ref_cols) <= ELEM_TOL * per_element_gemm_bound(a_c, a_s, b_c[cols], b_s[cols], mxfp4.dequantize))
    if out_dtype != 0:
        np.testing.assert_array_equal(bf16_dev_to_bits(y[ri]), linear.round_to_bf16_bits(y_rows))
        np.testing.assert_array_equal(bf16_dev_to_bits(y[:, ci].contiguous()), linear.round_to_bf16_bits(y_cols))
        # the whole result, on the device: every bf16 entry is the round-to-nearest-even of the fp32 entry
        u = y32.view(torch.int32)
        rne = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).to(torch.int16)
        assert torch.equal(rne, y.view(torch.int16))


def test_70b_down_proj_full_size():
    """LLaMA-3-70B down_proj prefill (T=4096, K=28672, N=8192, fp32 out): 512 tiles of 256 x 256, two per
    persistent workgroup, 224 K steps each."""
    import paper_2604_17789_amd as duqpp
    cfg = wl.CONFIGS["c4_70b_down_prefill"]
    assert duqpp.gemm_kernel_for(cfg["T"], cfg["N"], cfg["K"], duqpp.F32) == duqpp.KERNEL_LARGE
    _tiled_path_sampled("c4", cfg["T"], cfg["K"], cfg["N"], cfg["outliers"], cfg["w_std"], 0, n_rows=32, n_cols=32)


def test_layer_set_gate_proj_full_size():
    """gate_proj of the 8B layer set at T=8192 (K=4096, N=14336, bf16 out): 1792 tiles of 256 x 256, seven per
    persistent workgroup, the transfer pipeline crossing every tile boundary."""
    import paper_2604_17789_amd as duqpp
    assert duqpp.gemm_kernel_for(8192, 14336, 4096, duqpp.BF16) == duqpp.KERNEL_LARGE
    _tiled_path_sampled("c5-gate", 8192, 4096, 14336, (), 0.02, 1)


def test_layer_set_down_proj_full_size():
    """down_proj of the 8B layer set at T=8192 (K=14336, N=4096, bf16 out, outlier channels x100 on its input):
    the rotate+quantise launch with the most token tiles per wave, 512 tiles of 256 x 256 for the product."""
    _tiled_path_sampled("c5-down", 8192, 14336, 4096, (wl.OutlierSpec(8, 100.0),), 0.02, 1, n_rows=32, n_cols=32)


def test_layer_set_kv_proj_full_size():
    """k / v projection of the layer set (K=4096, N=1024, bf16 out): one 128 x 256 tile per CU."""
    import paper_2604_17789_amd as duqpp
    assert duqpp.gemm_kernel_for(8192, 1024, 4096, duqpp.BF16) == duqpp.KERNEL_MID
    _tiled_path_sampled("c5-k", 8192, 4096, 1024, (), 0.02, 1, n_rows=32, n_cols=32)
