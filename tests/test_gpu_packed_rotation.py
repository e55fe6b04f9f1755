"""GPU tests of the packed rotation blocks (duqpp_pack_rotation): the packed bytes against a numpy restatement of
the exact three-way bf16 split and of the operand's lane order, and the *_packed entry points bit for bit against
their fp32-block counterparts (which the other GPU tests hold to the oracle)."""
import numpy as np
import pytest

import workloads as wl
from helpers import to_dev, to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


def _bf16_trunc(v32):
    """fp32 array -> (the fp32 value of its top 16 bits, those 16 bits)."""
    u = v32.view(np.uint32) & np.uint32(0xFFFF0000)
    return u.view(np.float32), (u >> np.uint32(16)).astype(np.uint16)


def _split3(R):
    hi, hb = _bf16_trunc(R)
    r1 = (R - hi).astype(np.float32)                      # exact: the low 16 bits of the significand
    mid, mb = _bf16_trunc(r1)
    r2 = (r1 - mid).astype(np.float32)
    lo, lb = _bf16_trunc(r2)
    return (hi, mid, lo), (hb, mb, lb)


@pytest.mark.parametrize("n", [1, 3, 448])
def test_packed_bytes_are_the_exact_split_in_operand_order(env, n):
    torch, duqpp = env
    R = wl.make_rotation_blocks(f"gpu-pack-{n}", n)
    if n == 3:                                             # entries that exercise the split: tiny, huge, negative, exact bf16
        R[1] = np.ldexp(R[1], -60)
        R[2, 0, :8] = [1.0, -1.0, 0.0, 3.0e38, -1.0e-30, 0.33333334, 1.0 + 2.0 ** -23, -(1.0 + 2.0 ** -16)]
    vals, bits = _split3(R)
    # the three pieces are bf16 values that add up to the entry exactly (fp64 holds the sum exactly).  This holds while
    # the third piece is a normal number, i.e. for entries of magnitude 2^-110 and more (and for zero); below that the
    # split drops less than 2^-133, far outside anything a rotation block holds.
    assert np.all((np.abs(R) >= 2.0 ** -110) | (R == 0))
    np.testing.assert_array_equal(vals[0].astype(np.float64) + vals[1].astype(np.float64) + vals[2].astype(np.float64),
                                  R.astype(np.float64))
    packed = duqpp.pack_rotation(to_dev(R, torch))
    torch.cuda.synchronize()
    got = packed.cpu().numpy().view(np.uint16).reshape(n, 3, 2, 64, 8)       # [block][piece][k-step s][lane][i]
    for piece, b in ((0, bits[2]), (1, bits[1]), (2, bits[0])):              # low, middle, high
        # lane c + 32 h, element i of k-step s  <-  R[16 s + 8 h + i][c]
        want = b.reshape(n, 2, 2, 8, 32).transpose(0, 1, 2, 4, 3).reshape(n, 2, 64, 8)   # [block][s][h][i][c] -> [s][h*32 + c][i]
        np.testing.assert_array_equal(got[:, piece], want)


SHAPES = [(64, 4096, 0), (1, 4096, 0), (16, 14336, 0), (77, 1184, 0), (33, 32, 0), (300, 2048, 1), (2048, 14336, 0),
          (1000, 14368, 1), (2048, 4096, 0), (4100, 4096, 0), (8192, 2048, 1)]   # the last two: three-stage ring


@pytest.mark.parametrize("T,K,shared", SHAPES)
def test_rotate_quantize_tiled_packed_matches_the_unpacked_call(env, T, K, shared):
    torch, duqpp = env
    name = f"gpu-packed-{T}-{K}-{shared}"
    xb = wl.make_activations(name, T, K, (wl.OutlierSpec(min(8, K // 4), 50.0), wl.OutlierSpec(1, 1000.0, 1)))
    R = to_dev(wl.make_rotation_blocks(name, 1 if shared else K // 32), torch)
    x = to_dev_bf16(xb, torch)
    print(f"[packed R] T={T} K={K} shared={shared}", flush=True)
    Rp = duqpp.pack_rotation(R)
    ct, st = duqpp.rotate_quantize_tiled(x, R)
    cp, sp = duqpp.rotate_quantize_tiled_packed(x, Rp)
    torch.cuda.synchronize()
    assert torch.equal(ct, cp) and torch.equal(st, sp)


@pytest.mark.parametrize("T,N,K,dt", [(16, 300, 4096, 0), (300, 264, 2048, 1), (2048, 512, 14336, 1)])
def test_rotq_gemm_tiled_packed_matches_the_unpacked_call(env, T, N, K, dt):
    torch, duqpp = env
    name = f"gpu-packed-fused-{T}"
    xb = wl.make_activations(name, T, K, (wl.OutlierSpec(8, 50.0),))
    R = to_dev(wl.make_rotation_blocks(name, K // 32), torch)
    x, w = to_dev_bf16(xb, torch), to_dev_bf16(wl.make_weights(name, N, K, 0.02), torch)
    bct, bst = duqpp.quantize_weights_tiled(w, R)
    y = duqpp.rotq_gemm_tiled(x, R, bct, bst, N, out_dtype=dt)
    yp = duqpp.rotq_gemm_tiled_packed(x, duqpp.pack_rotation(R), bct, bst, N, out_dtype=dt)
    torch.cuda.synchronize()
    assert torch.equal(y, yp) and float(y.float().abs().max()) > 0


def test_packed_calls_check_their_arguments(env):
    torch, duqpp = env
    x = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda:0")
    Rp = duqpp.pack_rotation(to_dev(wl.make_rotation_blocks("gpu-packed-args", 2), torch))
    cb, sb = duqpp.tiled_bytes(8, 64)
    c = torch.empty(cb, dtype=torch.uint8, device=x.device)
    s = torch.empty(sb, dtype=torch.uint8, device=x.device)
    L = duqpp.lib
    assert L.duqpp_rotate_quantize_tiled_packed(x.data_ptr(), 8, 64, 64, None, 2, c.data_ptr(), s.data_ptr(), None) == -1
    assert L.duqpp_rotate_quantize_tiled_packed(x.data_ptr(), 8, 64, 64, Rp.data_ptr(), 3, c.data_ptr(), s.data_ptr(), None) == -2
    assert L.duqpp_rotate_quantize_tiled_packed(x.data_ptr(), 8, 64, 64, Rp.data_ptr() + 4, 2, c.data_ptr(), s.data_ptr(), None) == -3
    assert L.duqpp_pack_rotation(None, 2, Rp.data_ptr(), None) == -1
    assert L.duqpp_pack_rotation(Rp.data_ptr(), 0, Rp.data_ptr(), None) == -2
    assert L.duqpp_packed_rotation_bytes(0) == 0 and L.duqpp_packed_rotation_bytes(448) == 448 * 6144
