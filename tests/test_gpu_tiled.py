"""GPU parity of the tiled fast path: tile/untile permutations, rotate+quantise with tiled output, and
the tiled MXFP4 GEMM, all against the CPU oracle (through numpy restatements of the layout's index map)."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear, mxfp4, pipeline, rotation
from helpers import (assert_codes_differ_only_at_boundaries, bf16_dev_to_bits, rel_fro, rotation_error_ratio, tile_np,
                     to_dev, to_dev_bf16, untile_np)

pytestmark = pytest.mark.gpu
GEMM_TOL = 1e-5


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


def _random_mx(rng, rows, K, lo=118, hi=136):
    codes = rng.integers(0, 256, size=(rows, K // 2)).astype(np.uint8)
    scales = rng.integers(lo, hi + 1, size=(rows, K // 32)).astype(np.uint8)
    return codes, scales


def test_numpy_layout_helpers_are_inverse():
    rng = np.random.default_rng(0)
    c, s = _random_mx(rng, 45, 32 * 11)
    ct, st = tile_np(c, s)
    c2, s2, pc, ps = untile_np(ct, st, 45, 32 * 11)
    np.testing.assert_array_equal(c, c2)
    np.testing.assert_array_equal(s, s2)
    assert np.all(pc == 0) and np.all(ps == 127)
    # spot-check the documented offsets
    RT, GP = 2, 16
    for (row, j, b) in [(0, 0, 0), (33, 10, 7), (44, 5, 15), (31, 3, 2)]:
        rt, r = divmod(row, 32)
        assert ct[((rt * GP + j) * 32 + r) * 16 + b] == c[row, j * 16 + b]
        assert st[(((rt * (GP // 8) + j // 8) * 2 + (j % 8) // 4) * 32 + r) * 4 + j % 4] == s[row, j]


@pytest.mark.parametrize("rows,K", [(64, 4096), (45, 352), (1, 32), (300, 1184)])
def test_tile_and_untile_kernels(env, rows, K):
    torch, duqpp = env
    rng = np.random.default_rng(rows + K)
    c, s = _random_mx(rng, rows, K, 0, 254)
    ct, st = duqpp.tile_operand(to_dev(c, torch), to_dev(s, torch))
    torch.cuda.synchronize()
    ct_ref, st_ref = tile_np(c, s)
    np.testing.assert_array_equal(ct.cpu().numpy(), ct_ref)
    np.testing.assert_array_equal(st.cpu().numpy(), st_ref)
    c2, s2 = duqpp.untile_operand(ct, st, rows, K)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(c2.cpu().numpy(), c)
    np.testing.assert_array_equal(s2.cpu().numpy(), s)


RQ_SHAPES = [(64, 4096), (1, 4096), (16, 14336), (77, 1184), (33, 32), (300, 2048), (256, 14336)]


@pytest.mark.parametrize("T,K", RQ_SHAPES)
def test_rotate_quantize_tiled(env, T, K):
    """Tiled output = the row-major result (already held to the oracle) in its tiled positions, with
    code 0 / scale 127 in the padding; checked against the oracle directly as well."""
    torch, duqpp = env
    xb = wl.make_activations(f"gpu-rqt-{T}-{K}", T, K, (wl.OutlierSpec(min(8, K // 4), 50.0), wl.OutlierSpec(1, 1000.0, 1)))
    R = wl.make_rotation_blocks(f"gpu-rqt-{T}-{K}", K // 32)
    x, Rd = to_dev_bf16(xb, torch), to_dev(R, torch)
    print(f"[rotq tiled] T={T} K={K}", flush=True)
    ct, st = duqpp.rotate_quantize_tiled(x, Rd)
    c_rm, s_rm, yrot = duqpp.rotate_quantize(x, Rd, return_rotated=True)
    torch.cuda.synchronize()
    codes, scales, pc, ps = untile_np(ct.cpu().numpy(), st.cpu().numpy(), T, K)
    assert np.all(pc == 0) and np.all(ps == 127)
    np.testing.assert_array_equal(codes, c_rm.cpu().numpy())
    np.testing.assert_array_equal(scales, s_rm.cpu().numpy())
    c_ref, s_ref = mxfp4.quantize(yrot.cpu().numpy())
    np.testing.assert_array_equal(codes, c_ref)
    np.testing.assert_array_equal(scales, s_ref)
    xf = wl.bf16_bits_to_f32(xb)
    assert rotation_error_ratio(yrot.cpu().numpy(), rotation.rotate(xf, R), xf) <= 1e-5


def _rotq_edge_shapes():
    """Seeded draws: token counts either side of the 32-token tile edges and of the launch plan's changes of
    shape, group counts that are odd, not multiples of 8 (padded groups) or of 16 (a workgroup's column chunk)."""
    rng = np.random.default_rng(4172026)
    tokens = [1, 2, 31, 32, 33, 63, 64, 65, 127, 129, 255, 257, 300, 511, 513, 1000]
    groups = [1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 33, 37, 63, 65, 100, 129]
    return [(int(rng.choice(tokens)), 32 * int(rng.choice(groups)), int(rng.integers(0, 2))) for _ in range(20)]


@pytest.mark.parametrize("T,K,shared", _rotq_edge_shapes())
def test_rotate_quantize_shapes_at_tile_edges(env, T, K, shared):
    """Both layouts from the same rotated values: codes and scales bit-exact against the oracle's quantiser on the
    values the row-major call reports, the tiled call's bytes in their tiled positions with the documented padding,
    the rotation within tolerance."""
    torch, duqpp = env
    name = f"gpu-rq-edge-{T}-{K}-{shared}"
    xb = wl.make_activations(name, T, K, (wl.OutlierSpec(min(4, K // 8), 50.0), wl.OutlierSpec(1, 1000.0, 1)))
    R = wl.make_rotation_blocks(name, 1 if shared else K // 32)
    x, Rd = to_dev_bf16(xb, torch), to_dev(R, torch)
    print(f"[rotq] tile edges T={T} K={K} shared={shared}", flush=True)
    ct, st = duqpp.rotate_quantize_tiled(x, Rd)
    c_rm, s_rm, yrot = duqpp.rotate_quantize(x, Rd, return_rotated=True)
    torch.cuda.synchronize()
    codes, scales, pc, ps = untile_np(ct.cpu().numpy(), st.cpu().numpy(), T, K)
    assert np.all(pc == 0) and np.all(ps == 127)
    c_ref, s_ref = mxfp4.quantize(yrot.cpu().numpy())
    np.testing.assert_array_equal(c_rm.cpu().numpy(), c_ref)
    np.testing.assert_array_equal(s_rm.cpu().numpy(), s_ref)
    np.testing.assert_array_equal(codes, c_ref)
    np.testing.assert_array_equal(scales, s_ref)
    xf = wl.bf16_bits_to_f32(xb)
    assert rotation_error_ratio(yrot.cpu().numpy(), rotation.rotate(xf, R), xf) <= 1e-5


@pytest.mark.parametrize("T,K,pad", [(77, 1184, 8), (300, 2048, 4096), (2100, 4096, 64)])
def test_rotate_quantize_tiled_strided_input(env, T, K, pad):
    """Token rows `ldx` = K + pad elements apart (a slice of a wider tensor): the same bytes as from dense rows,
    for the tiled call and for the fused call built on it."""
    torch, duqpp = env
    xb = wl.make_activations(f"gpu-rqt-strided-{T}-{K}", T, K + pad, (wl.OutlierSpec(8, 50.0),))
    R = wl.make_rotation_blocks(f"gpu-rqt-strided-{T}-{K}", K // 32)
    wide, Rd = to_dev_bf16(xb, torch), to_dev(R, torch)
    x = wide[:, :K]
    assert x.stride(0) == K + pad
    print(f"[rotq tiled] strided input T={T} K={K} ldx={K + pad}", flush=True)
    ct, st = duqpp.rotate_quantize_tiled(x, Rd)
    ct_d, st_d = duqpp.rotate_quantize_tiled(x.contiguous(), Rd)
    torch.cuda.synchronize()
    assert torch.equal(ct, ct_d) and torch.equal(st, st_d)
    N = 136
    wb = wl.make_weights(f"gpu-rqt-strided-{T}-{K}", N, K, 0.02)
    bct, bst = duqpp.quantize_weights_tiled(to_dev_bf16(wb, torch), Rd)
    y = duqpp.rotq_gemm_tiled(x, Rd, bct, bst, N)
    y_d = duqpp.mxfp4_gemm_tiled(ct_d, st_d, bct, bst, T, N, K)
    torch.cuda.synchronize()
    assert torch.equal(y, y_d)


def test_rotate_quantize_tiled_shared_block(env):
    """One rotation block shared by every group (the deployed variant of Sec. 4.2): same result as the
    row-major kernel, which is held to the oracle, and as K/32 copies of the block."""
    torch, duqpp = env
    T, K = 200, 2048
    xb = wl.make_activations("gpu-rqt-shared", T, K, (wl.OutlierSpec(8, 50.0),))
    R1 = wl.make_rotation_blocks("gpu-rqt-shared", 1)
    x = to_dev_bf16(xb, torch)
    ct, st = duqpp.rotate_quantize_tiled(x, to_dev(R1, torch))
    c_rm, s_rm = duqpp.rotate_quantize(x, to_dev(R1, torch))
    ct2, st2 = duqpp.rotate_quantize_tiled(x, to_dev(np.repeat(R1, K // 32, axis=0), torch))
    torch.cuda.synchronize()
    codes, scales, _, _ = untile_np(ct.cpu().numpy(), st.cpu().numpy(), T, K)
    np.testing.assert_array_equal(codes, c_rm.cpu().numpy())
    np.testing.assert_array_equal(scales, s_rm.cpu().numpy())
    assert torch.equal(ct, ct2) and torch.equal(st, st2)
    c_ref, s_ref, y_ref = pipeline.rotate_quantize(xb, R1)   # each side rotates in its own precision
    assert_codes_differ_only_at_boundaries(codes, scales, c_ref, s_ref, y_ref, wl.bf16_bits_to_f32(xb))


# Shapes with several token tiles per wave and more workgroups than CUs: short rows (an XCD's workgroups take
# consecutive column chunks), long rows (an XCD owns column chunks), a ragged last token tile, groups that need padding.
# The last five make the launch plan pick 5, 6 and 7 waves per workgroup, with and without a spare wave in the last column chunk,
# and 2 waves per workgroup.
# The three after those have rows of a power-of-two length and enough tokens for the four-wave plan: 4 tiles per wave (two-stage
# ring), then 9 with a ragged last tile and 8 (three-stage ring), the last with a shared block.
RQ_LARGE_SHAPES = [(2048, 4096, 0), (4100, 2336, 0), (1000, 14368, 0), (2048, 14336, 0), (2048, 4096, 1), (1000, 14368, 1),
                   (1000, 4160, 0), (1000, 4928, 1), (1000, 5408, 0), (1000, 6176, 0), (1000, 1280, 0),
                   (4100, 4096, 0), (8192, 2048, 0), (4096, 4096, 1)]


@pytest.mark.parametrize("T,K,shared", RQ_LARGE_SHAPES)
def test_rotate_quantize_tiled_large(env, T, K, shared):
    """Codes and scales bit-exact against the oracle's quantiser on the rotated values the row-major call reports
    (the two calls rotate with the same arithmetic: their codes must be identical), padding as documented, and the
    rotation itself within tolerance of the oracle."""
    torch, duqpp = env
    xb = wl.make_activations(f"gpu-rqtl-{T}-{K}", T, K, (wl.OutlierSpec(min(8, K // 4), 50.0), wl.OutlierSpec(2, 1000.0, 4)))
    R = wl.make_rotation_blocks(f"gpu-rqtl-{T}-{K}", 1 if shared else K // 32)
    x, Rd = to_dev_bf16(xb, torch), to_dev(R, torch)
    print(f"[rotq tiled, large] T={T} K={K} shared={shared}", flush=True)
    ct, st = duqpp.rotate_quantize_tiled(x, Rd)
    c_rm, s_rm, yrot = duqpp.rotate_quantize(x, Rd, return_rotated=True)
    torch.cuda.synchronize()
    codes, scales, pc, ps = untile_np(ct.cpu().numpy(), st.cpu().numpy(), T, K)
    assert np.all(pc == 0) and np.all(ps == 127)
    np.testing.assert_array_equal(codes, c_rm.cpu().numpy())
    np.testing.assert_array_equal(scales, s_rm.cpu().numpy())
    yr = yrot.cpu().numpy()
    c_ref, s_ref = mxfp4.quantize(yr)
    np.testing.assert_array_equal(codes, c_ref)
    np.testing.assert_array_equal(scales, s_ref)
    y_ref = rotation.rotate(wl.bf16_bits_to_f32(xb), R)
    assert rotation_error_ratio(yr, y_ref, wl.bf16_bits_to_f32(xb)) <= 1e-5


def test_quantize_weights_tiled(env):
    torch, duqpp = env
    N, K = 200, 1184
    wb = wl.make_weights("gpu-qwt", N, K, 0.02)
    R = wl.make_rotation_blocks("gpu-qwt", K // 32)
    ct, st = duqpp.quantize_weights_tiled(to_dev_bf16(wb, torch), to_dev(R, torch))
    c_rm, s_rm = duqpp.quantize_weights(to_dev_bf16(wb, torch), to_dev(R, torch))
    torch.cuda.synchronize()
    codes, scales, pc, ps = untile_np(ct.cpu().numpy(), st.cpu().numpy(), N, K)
    assert np.all(pc == 0) and np.all(ps == 127)
    np.testing.assert_array_equal(codes, c_rm.cpu().numpy())
    np.testing.assert_array_equal(scales, s_rm.cpu().numpy())


def _gemm_tiled(env, ac, asc, bc, bsc, out_dtype=0):
    torch, duqpp = env
    T, K = ac.shape[0], ac.shape[1] * 2
    N = bc.shape[0]
    act, ast = tile_np(ac, asc)
    bct, bst = tile_np(bc, bsc)
    y = duqpp.mxfp4_gemm_tiled(to_dev(act, torch), to_dev(ast, torch), to_dev(bct, torch), to_dev(bst, torch),
                               T, N, K, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return y


GEMM_SHAPES = [
    (64, 96, 512),
    (77, 130, 1184),      # ragged in T, N; 37 groups padded to 40
    (1, 257, 4096),       # decode
    (16, 300, 2048),
    (24, 200, 1184),      # one ragged row tile, ragged K steps over the decode kernel's eight waves
    (32, 96, 32),         # decode kernel, a single group
    (33, 200, 1184),      # decode kernel with two activation row tiles, the second almost empty
    (64, 4100, 288),      # two full activation row tiles, 129 weight row tiles (each cut in two)
    (50, 8200, 544),      # two activation row tiles, 257 weight row tiles (whole tiles per workgroup)
    (96, 300, 1184),      # decode kernel in two passes; the second pass has one real row tile
    (128, 4100, 288),     # decode kernel in two passes of two full row tiles
    (100, 8200, 544),     # two passes, whole weight row tiles per workgroup, ragged last token tile
    (130, 70, 32),        # a single group (one K step of mostly padding)
    (200, 264, 2304),
    (129, 513, 1312),
    (256, 512, 256),      # exactly one K step
    (384, 768, 512),      # two K steps, several workgroups
    (300, 1000, 768),     # three K steps
    # more output tiles than CUs: workgroups walk several tiles with the transfer pipeline running on
    (1100, 8300, 544),    # 9 x 33 = 297 tiles, three K steps, ragged edges
    (2100, 4200, 32),     # 17 x 17 = 289 tiles of a single K step each
    (3000, 5000, 288),    # 24 x 20 = 480 tiles, two K steps (the second mostly padding)
    (700, 40000, 256),    # 6 x 157 = 942 tiles: up to four tiles per workgroup, one K step
    # the 16-row weight-streaming kernel (up to 16 tokens, fewer than 256 weight row tiles)
    (16, 40, 256),        # one K step: seven of the eight waves have none; second row tile with 8 real rows
    (9, 17, 32),          # a single group; tokens and channels both short of 16
    (13, 300, 14368),     # 57 K steps over eight waves: 8, 8, ..., 1 steps (even and odd runs of the two-set loop)
    (16, 8160, 64),       # 255 row tiles, the most this kernel takes
    (1, 4100, 14336),     # the LLaMA-3-8B down_proj decode shape, ragged in N
    (16, 8192, 64),       # 256 row tiles: back on the 32-row kernel
    (48, 28672, 288),     # 33-64 tokens against so many channels that the 64 x 128 tiles are chosen over weight streaming
]


@pytest.mark.parametrize("T,N,K", GEMM_SHAPES)
def test_gemm_tiled_random_codes(env, T, N, K):
    rng = np.random.default_rng(T * 1000003 + N * 1009 + K)
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    print(f"[gemm tiled] random codes T={T} N={N} K={K}", flush=True)
    y = _gemm_tiled(env, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    assert rel_fro(y, ref) <= GEMM_TOL


def test_gemm_tiled_exact_integer_case(env):
    rng = np.random.default_rng(78)
    T, N, K = 160, 320, 14336
    ac = rng.integers(0, 256, size=(T, K // 2)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    asc = np.full((T, K // 32), 125, dtype=np.uint8)
    bsc = np.full((N, K // 32), 131, dtype=np.uint8)
    y = _gemm_tiled(env, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    np.testing.assert_array_equal(y, ref.astype(np.float32))


def test_gemm_tiled_scale_bytes_pair_with_their_own_group(env):
    T, N, K = 70, 300, 1024
    G = K // 32
    rng = np.random.default_rng(6)
    ac = np.zeros((T, K // 2), dtype=np.uint8)
    bc = np.zeros((N, K // 2), dtype=np.uint8)
    pos = rng.integers(0, 32, size=G)
    for j in range(G):
        k = 32 * j + int(pos[j])
        ac[:, k // 2] = 0x02 << (4 * (k & 1))
        bc[:, k // 2] = 0x02 << (4 * (k & 1))
    asc = (110 + (np.arange(T)[:, None] * 7 + np.arange(G)[None, :] * 3) % 9).astype(np.uint8)
    bsc = (120 + (np.arange(N)[:, None] * 5 + np.arange(G)[None, :]) % 8).astype(np.uint8)
    y = _gemm_tiled(env, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    np.testing.assert_array_equal(y, ref.astype(np.float32))   # sums of at most 32 powers of two within 2^17: exact


def _edge_shapes():
    """Seeded draws of T and N from the values either side of every tile edge of the four kernels (32, 64, 128,
    256 and their multiples), K from 1 to 80 groups."""
    rng = np.random.default_rng(20260417)
    edges = [1, 2, 31, 32, 33, 63, 64, 65, 95, 97, 127, 128, 129, 191, 193, 255, 256, 257, 300, 383, 385, 511, 512,
             513, 640, 767, 769]
    shapes = []
    for _ in range(28):
        shapes.append((int(rng.choice(edges)), int(rng.choice(edges)), 32 * int(rng.integers(1, 81))))
    return shapes


@pytest.mark.parametrize("T,N,K", _edge_shapes())
def test_gemm_tiled_shapes_at_tile_edges(env, T, N, K):
    """Whatever kernel the library picks for the shape: the product against the oracle, and the bf16 result as
    the rounding of the fp32 one."""
    rng = np.random.default_rng(T * 7919 + N * 104729 + K)
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    print(f"[gemm tiled] tile edges T={T} N={N} K={K}", flush=True)
    y32 = _gemm_tiled(env, ac, asc, bc, bsc, 0).cpu().numpy()
    assert rel_fro(y32, linear.mxfp4_gemm(ac, asc, bc, bsc)) <= GEMM_TOL
    np.testing.assert_array_equal(bf16_dev_to_bits(_gemm_tiled(env, ac, asc, bc, bsc, 1)), linear.round_to_bf16_bits(y32))


@pytest.mark.parametrize("T", [1, 7, 16])
def test_gemm_tiled_16_row_kernel_exact_cases(env, T):
    """Up to 16 tokens against fewer than 256 weight row tiles: the 16-row kernel.  Equal scales make every partial
    sum exact (bit-identical to the oracle in any order); then one non-zero element per group with scales that differ
    from group to group and row to row, where a scale byte taken from the wrong group, row or operand shows."""
    rng = np.random.default_rng(160 + T)
    N, K = 330, 14336
    ac = rng.integers(0, 256, size=(T, K // 2)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    asc = np.full((T, K // 32), 125, dtype=np.uint8)
    bsc = np.full((N, K // 32), 131, dtype=np.uint8)
    y = _gemm_tiled(env, ac, asc, bc, bsc).cpu().numpy()
    np.testing.assert_array_equal(y, linear.mxfp4_gemm(ac, asc, bc, bsc).astype(np.float32))
    K = 1024
    G = K // 32
    ac = np.zeros((T, K // 2), dtype=np.uint8)
    bc = np.zeros((N, K // 2), dtype=np.uint8)
    pos = rng.integers(0, 32, size=G)
    for j in range(G):
        k = 32 * j + int(pos[j])
        ac[:, k // 2] = 0x02 << (4 * (k & 1))
        bc[:, k // 2] = 0x02 << (4 * (k & 1))
    asc = (110 + (np.arange(T)[:, None] * 7 + np.arange(G)[None, :] * 3) % 9).astype(np.uint8)
    bsc = (120 + (np.arange(N)[:, None] * 5 + np.arange(G)[None, :]) % 8).astype(np.uint8)
    y = _gemm_tiled(env, ac, asc, bc, bsc).cpu().numpy()
    np.testing.assert_array_equal(y, linear.mxfp4_gemm(ac, asc, bc, bsc).astype(np.float32))
    y16 = bf16_dev_to_bits(_gemm_tiled(env, ac, asc, bc, bsc, 1))
    np.testing.assert_array_equal(y16, linear.round_to_bf16_bits(y))


@pytest.mark.parametrize("T,N,K", [(70, 200, 1024), (1100, 8300, 544), (2100, 4200, 32)])
def test_gemm_tiled_bf16_output(env, T, N, K):
    rng = np.random.default_rng(14)
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    y32 = _gemm_tiled(env, ac, asc, bc, bsc, 0).cpu().numpy()
    y16 = bf16_dev_to_bits(_gemm_tiled(env, ac, asc, bc, bsc, 1))
    np.testing.assert_array_equal(y16, linear.round_to_bf16_bits(y32))
    # against the oracle: one bf16 rounding (2^-9 relative, taken as 2^-8) on top of the fp32 accumulation
    # error, which is relative to the size of the terms, not of a sum that cancels
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    val = wl.bf16_bits_to_f32(y16).astype(np.float64)
    assert np.all(np.abs(val - ref) <= 2.0 ** -8 * np.abs(ref) + GEMM_TOL * np.max(np.abs(ref)))
    if T * N <= 70 * 200:                                  # small case: no cancelling sums, so within one bf16 step
        ref16 = linear.round_to_bf16_bits(ref.astype(np.float32))
        assert np.max(np.abs(y16.astype(np.int32) - ref16.astype(np.int32))) <= 1


@pytest.mark.parametrize("T,N,K", [(1, 512, 4096), (16, 4096, 1184), (100, 200, 1024), (64, 4096, 4096)])
def test_whole_tiled_path_and_fused_call(env, T, N, K):
    torch, duqpp = env
    xb = wl.make_activations(f"tiled-{T}", T, K, (wl.OutlierSpec(8, 50.0),))
    wb = wl.make_weights(f"tiled-{T}", N, K, 0.02)
    R = wl.make_rotation_blocks(f"tiled-{T}", K // 32)
    x, w, Rd = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch), to_dev(R, torch)
    bct, bst = duqpp.quantize_weights_tiled(w, Rd)
    act, ast = duqpp.rotate_quantize_tiled(x, Rd)
    for dt in (0, 1):
        y = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=dt)
        yf = duqpp.rotq_gemm_tiled(x, Rd, bct, bst, N, out_dtype=dt)
        torch.cuda.synchronize()
        assert torch.equal(y, yf)
    ac, asc, _, _ = untile_np(act.cpu().numpy(), ast.cpu().numpy(), T, K)
    bc, bsc, _, _ = untile_np(bct.cpu().numpy(), bst.cpu().numpy(), N, K)
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    y32 = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K).cpu().numpy()
    assert rel_fro(y32, ref) <= GEMM_TOL
    # and the row-major entry points give the same product from the same codes
    y_rm = duqpp.mxfp4_gemm(to_dev(ac, torch), to_dev(asc, torch), to_dev(bc, torch), to_dev(bsc, torch)).cpu().numpy()
    assert rel_fro(y_rm, ref) <= GEMM_TOL


@pytest.mark.parametrize("name", ["c3_decode_gateup_T1", "c3_decode_gateup_T4", "c3_decode_gateup_T16",
                                  "c3_decode_down_T1", "c3_decode_down_T4", "c3_decode_down_T16"])
def test_decode_configs(env, name):
    """LLaMA-3-8B decode shapes: weights resident as tiled MXFP4, activations rotated + quantised per call."""
    torch, duqpp = env
    cfg = wl.CONFIGS[name]
    T, K, N = cfg["T"], cfg["K"], cfg["N"]
    xb = wl.make_activations(name, T, K, cfg["outliers"])
    wb = wl.make_weights(name, N, K, cfg["w_std"])
    R = wl.make_rotation_blocks(name, K // 32)
    x, w, Rd = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch), to_dev(R, torch)
    print(f"[decode] {name} T={T} K={K} N={N}", flush=True)
    bct, bst = duqpp.quantize_weights_tiled(w, Rd)
    act, ast = duqpp.rotate_quantize_tiled(x, Rd)
    y = duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K)
    yf = duqpp.rotq_gemm_tiled(x, Rd, bct, bst, N)
    torch.cuda.synchronize()
    assert torch.equal(y, yf)
    ac, asc, _, _ = untile_np(act.cpu().numpy(), ast.cpu().numpy(), T, K)
    bc, bsc, _, _ = untile_np(bct.cpu().numpy(), bst.cpu().numpy(), N, K)
    c_ref, s_ref, y_ref = pipeline.rotate_quantize(xb, R)  # activation codes: own rotations may differ at rounding boundaries
    assert_codes_differ_only_at_boundaries(ac, asc, c_ref, s_ref, y_ref, wl.bf16_bits_to_f32(xb))
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    assert rel_fro(y.cpu().numpy(), ref) <= GEMM_TOL


def test_graph_replay_matches_eager_launches(env):
    """The bench times a captured graph of the two kernels: every replay must give what eager launches give,
    also after the inputs behind the captured pointers have changed (prefill and decode kernels)."""
    torch, duqpp = env
    for (T, N, K) in [(300, 520, 1184), (16, 300, 2048)]:
        R = to_dev(wl.make_rotation_blocks("graph", K // 32), torch)
        w = to_dev_bf16(wl.make_weights("graph", N, K, 0.02), torch)
        bct, bst = duqpp.quantize_weights_tiled(w, R)
        x = to_dev_bf16(wl.make_activations("graph-0", T, K, (wl.OutlierSpec(4, 50.0),)), torch)
        cb, sb = duqpp.tiled_bytes(T, K)
        act = torch.empty(cb, dtype=torch.uint8, device=x.device)
        ast = torch.empty(sb, dtype=torch.uint8, device=x.device)
        y = torch.empty((T, N), dtype=torch.float32, device=x.device)

        def run():
            duqpp.rotate_quantize_tiled(x, R, out=(act, ast))
            duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out=y)

        run()                                              # first call outside the capture (function attributes)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                run()
        torch.cuda.synchronize()
        for rep in range(3):
            x.copy_(to_dev_bf16(wl.make_activations(f"graph-{rep + 1}", T, K, (wl.OutlierSpec(4, 50.0),)), torch))
            y.zero_()
            g.replay()
            torch.cuda.synchronize()
            y_graph, a_graph = y.clone(), act.clone()
            y.zero_()
            run()
            torch.cuda.synchronize()
            assert torch.equal(a_graph, act) and torch.equal(y_graph, y), (T, N, K, rep)
            assert float(y.abs().max()) > 0


def test_two_stream_graph_matches_eager_launches(env):
    """The bench's second launch form: all rotate+quantise launches on one stream, all GEMMs on another, tied by
    events (a GEMM after the codes it reads, a rotate+quantise after the GEMM that last read its output buffers), so
    that consecutive batches overlap at their edges.  Every replay must give what eager launches give, with the
    program's own eager work and synchronisations between the replays.  The check runs in a process of its own
    (tests/two_stream_graph_check.py), as the bench's measurement does."""
    import os
    import subprocess
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    p = subprocess.run([sys.executable, os.path.join(here, "two_stream_graph_check.py")], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 0 and "two-stream graph: OK" in p.stdout, p.stdout[-2000:]


def test_fused_tiled_call_checks_both_stages_before_launching(env):
    """A bad argument of the second stage (the product) must be refused before the first stage (rotate+quantise) has
    been enqueued: the workspace, which rotate+quantise would overwrite, keeps its contents."""
    torch, duqpp = env
    T, K, N = 40, 256, 64
    x = to_dev_bf16(wl.make_activations("fused-args", T, K), torch)
    R = to_dev(wl.make_rotation_blocks("fused-args", K // 32), torch)
    bct, bst = duqpp.quantize_weights_tiled(to_dev_bf16(wl.make_weights("fused-args", N, K, 0.02), torch), R)
    cb, sb = duqpp.tiled_bytes(T, K)
    ws = torch.full((((cb + 255) // 256 + (sb + 255) // 256) * 256,), 0x5A, dtype=torch.uint8, device=x.device)
    y = torch.full((T, N), 7.0, dtype=torch.float32, device=x.device)
    L = duqpp.lib
    def call(out_dtype=0, ldy=N, yptr=None):
        return L.duqpp_rotq_gemm_tiled(x.data_ptr(), K, R.data_ptr(), K // 32, bct.data_ptr(), bst.data_ptr(), T, N, K,
                                       y.data_ptr() if yptr is None else yptr, out_dtype, ldy, ws.data_ptr(), ws.numel(), None)
    assert call(out_dtype=9) == -4
    assert call(ldy=N - 1) == -2
    assert call(yptr=y.data_ptr() + 2) == -3
    torch.cuda.synchronize()
    assert bool((ws == 0x5A).all()) and bool((y == 7.0).all())
    assert call() == 0
    torch.cuda.synchronize()
    assert not bool((ws == 0x5A).all()) and torch.equal(y, duqpp.rotq_gemm_tiled(x, R, bct, bst, N))
