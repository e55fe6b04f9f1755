"""GPU parity where byte offsets and element indices pass 2^31 and 2^32: 2.2 M tokens of K = 4096 (an 18 GB
activation tensor, 4.5 GB of codes, a 4.5 GB / 9 GB result), checked on runs of rows that straddle every such
boundary of every array, and on the ragged last row tile."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear, mxfp4, rotation
from helpers import bf16_dev_to_bits, rel_fro, rotation_error_ratio, to_dev, to_dev_bf16, untile_np

pytestmark = pytest.mark.gpu

T, K, N = 2_200_007, 4096, 1024
# first rows at which: x passes 2^31 and 2^32 bytes (8 KiB per row) = 2^31 elements; the fp32 result passes 2^32
# bytes; codes (2 KiB per row, either layout) and the bf16 result pass 2^32 bytes, the result 2^31 elements
BOUNDARIES = (0, 262_144, 524_288, 1_048_576, 2_097_152, T)


def _sampled_rows():
    rows = set()
    for b in BOUNDARIES:
        rows.update(range(max(b - 20, 0), min(b + 20, T)))
    return np.array(sorted(rows), dtype=np.int64)


def test_rows_beyond_4_gib():
    import torch

    import paper_2604_17789_amd as duqpp
    dev = torch.device("cuda:0")
    free, _ = torch.cuda.mem_get_info()
    if free < 80 * 2 ** 30:
        pytest.skip("needs 80 GiB of free device memory")
    print(f"[offsets] generating T={T} K={K} N={N}", flush=True)
    gen = torch.Generator(device=dev)
    gen.manual_seed(0x260417789)
    x = torch.empty((T, K), dtype=torch.bfloat16, device=dev)
    step = 1 << 18
    for r0 in range(0, T, step):                           # N(0,1) in pieces, eight channels x50 (Sec. 4.1's normal outliers)
        r1 = min(r0 + step, T)
        piece = torch.randn((r1 - r0, K), generator=gen, device=dev, dtype=torch.float32)
        piece[:, 37::512] *= 50.0
        x[r0:r1] = piece.to(torch.bfloat16)
    del piece
    R = wl.make_rotation_blocks("offsets", K // 32)
    wb = wl.make_weights("offsets", N, K, 0.02)
    Rd, w = to_dev(R, torch), to_dev_bf16(wb, torch)
    rows = _sampled_rows()
    rows_d = torch.from_numpy(rows).to(dev)

    print("[offsets] device: rotate+quantise, both layouts", flush=True)
    c_rm, s_rm = duqpp.rotate_quantize(x, Rd)
    act, ast = duqpp.rotate_quantize_tiled(x, Rd)
    xs = x[rows_d].contiguous()
    cs, ss, yrot = duqpp.rotate_quantize(xs, Rd, return_rotated=True)
    torch.cuda.synchronize()
    # rows are independent: the call on the sampled rows alone must give the big call's rows
    assert torch.equal(c_rm[rows_d], cs) and torch.equal(s_rm[rows_d], ss)
    cs_h, ss_h, yrot_h = cs.cpu().numpy(), ss.cpu().numpy(), yrot.cpu().numpy()
    xf = xs.float().cpu().numpy()
    assert rotation_error_ratio(yrot_h, rotation.rotate(xf, R), xf) <= 1e-5
    c_ref, s_ref = mxfp4.quantize(yrot_h)
    np.testing.assert_array_equal(cs_h, c_ref)
    np.testing.assert_array_equal(ss_h, s_ref)

    print("[offsets] tiled layout: device conversion in full, index map restated on the sampled row tiles", flush=True)
    c_un, s_un = duqpp.untile_operand(act, ast, T, K)
    assert torch.equal(c_un, c_rm) and torch.equal(s_un, s_rm)
    del c_un, s_un
    GP = (K // 32 + 7) // 8 * 8
    for rt in sorted({int(r) // 32 for r in rows}):
        n_rows = min(32, T - 32 * rt)
        ct = act[rt * GP * 512:(rt + 1) * GP * 512].cpu().numpy()
        st = ast[rt * GP * 32:(rt + 1) * GP * 32].cpu().numpy()
        tc, ts, pc, ps = untile_np(ct, st, n_rows, K)
        np.testing.assert_array_equal(tc, c_rm[32 * rt:32 * rt + n_rows].cpu().numpy())
        np.testing.assert_array_equal(ts, s_rm[32 * rt:32 * rt + n_rows].cpu().numpy())
        assert np.all(pc == 0) and np.all(ps == 127)
    ct2, st2 = duqpp.tile_operand(c_rm, s_rm)
    assert torch.equal(ct2, act) and torch.equal(st2, ast)
    del ct2, st2

    print("[offsets] device: products", flush=True)
    bct, bst = duqpp.quantize_weights_tiled(w, Rd)
    bc, bs = duqpp.untile_operand(bct, bst, N, K)
    y32 = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=duqpp.F32)
    y32_mid = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=duqpp.F32, kernel=duqpp.KERNEL_MID)
    y16 = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=duqpp.BF16)
    torch.cuda.synchronize()
    ref = linear.mxfp4_gemm(cs_h, ss_h, bc.cpu().numpy(), bs.cpu().numpy())
    y32_s = y32[rows_d].cpu().numpy()
    assert rel_fro(y32_s, ref) <= 1e-5
    assert rel_fro(y32_mid[rows_d].cpu().numpy(), ref) <= 1e-5
    del y32_mid
    np.testing.assert_array_equal(bf16_dev_to_bits(y16[rows_d]), linear.round_to_bf16_bits(y32_s))
    # the entry points that take row-major operands or bf16 activations run the same kernels behind a conversion
    y_rm = duqpp.mxfp4_gemm(c_rm, s_rm, bc, bs, out_dtype=duqpp.F32)
    torch.cuda.synchronize()
    assert torch.equal(y_rm, y32)
    del y_rm, y32
    y_f = duqpp.rotq_gemm_tiled(x, Rd, bct, bst, N, out_dtype=duqpp.BF16)
    torch.cuda.synchronize()
    assert torch.equal(y_f, y16)
    del y_f, y16, x, c_rm, s_rm, act, ast
    torch.cuda.empty_cache()
