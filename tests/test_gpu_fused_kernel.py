"""GPU parity of the one-kernel form of the online path (duqpp_rotq_gemm_fused_decode; shaped for up to 32 tokens,
more run as tiles of 32): the
activation codes and scales it forms in its prologue must be the bytes duqpp_rotate_quantize_tiled writes (which the
other GPU tests hold to the oracle), and its product must match the oracle's product of those codes."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear, mxfp4
from helpers import bf16_dev_to_bits, per_element_gemm_bound, rel_fro, to_dev, to_dev_bf16, untile_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


# (T, N, K, one shared rotation block)
SHAPES = [
    (1, 14336, 4096, 0), (4, 14336, 4096, 0), (16, 14336, 4096, 0),      # LLaMA-3-8B gate/up decode
    (1, 4096, 14336, 0), (16, 4096, 14336, 0),                           # down decode
    (24, 200, 1184, 0),       # ragged tokens and channels, 37 groups padded to 40, waves with uneven runs of K steps
    (32, 96, 32, 0),          # a single group: seven of the eight waves have no step
    (7, 300, 2048, 1),        # the shared block of Sec. 4.2
    (20, 8200, 544, 0),       # 257 weight row tiles
    (100, 200, 1184, 0),      # four token tiles, the last with four tokens
    (300, 264, 2048, 1),      # ten token tiles, shared block
]


@pytest.mark.parametrize("T,N,K,shared", SHAPES)
def test_one_kernel_form_against_the_two_launches_and_the_oracle(env, T, N, K, shared):
    torch, duqpp = env
    name = f"gpu-fused-{T}-{N}-{K}"
    xb = wl.make_activations(name, T, K, (wl.OutlierSpec(min(8, K // 4), 50.0), wl.OutlierSpec(1, 1000.0, 1)))
    R = to_dev(wl.make_rotation_blocks(name, 1 if shared else K // 32), torch)
    x, w = to_dev_bf16(xb, torch), to_dev_bf16(wl.make_weights(name, N, K, 0.02), torch)
    bct, bst = duqpp.quantize_weights_tiled(w, R)
    Rp = duqpp.pack_rotation(R)
    print(f"[one kernel] T={T} N={N} K={K} shared={shared}", flush=True)
    y, ct, st = duqpp.rotq_gemm_fused_decode(x, Rp, bct, bst, N, return_operand=True)
    y16 = duqpp.rotq_gemm_fused_decode(x, Rp, bct, bst, N, out_dtype=duqpp.BF16)
    ct_ref, st_ref = duqpp.rotate_quantize_tiled(x, R)
    y_two = duqpp.rotq_gemm_tiled(x, R, bct, bst, N)
    torch.cuda.synchronize()
    # the same codes as the separate path, padding included
    assert torch.equal(ct, ct_ref) and torch.equal(st, st_ref)
    ac, asc, _, _ = untile_np(ct.cpu().numpy(), st.cpu().numpy(), T, K)
    bc, bsc, _, _ = untile_np(bct.cpu().numpy(), bst.cpu().numpy(), N, K)
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    yh = y.cpu().numpy()
    assert rel_fro(yh, ref) <= 1e-5
    assert np.all(np.abs(yh - ref) <= 1e-5 * per_element_gemm_bound(ac, asc, bc, bsc, mxfp4.dequantize))
    np.testing.assert_array_equal(bf16_dev_to_bits(y16), linear.round_to_bf16_bits(yh))
    assert rel_fro(yh, y_two.cpu().numpy()) <= 1e-6            # same codes, another order of the fp32 additions
    if N >= 8192 and 16 < T <= 32:
        # here the two-launch path runs the weight-streaming kernel with whole row tiles, whose K split and reduction
        # this kernel shares: the same additions in the same order
        assert torch.equal(y, y_two)


def test_one_kernel_form_checks_its_arguments(env):
    torch, duqpp = env
    x = torch.zeros((33, 64), dtype=torch.bfloat16, device="cuda:0")
    R = to_dev(wl.make_rotation_blocks("gpu-fused-args", 2), torch)
    Rp = duqpp.pack_rotation(R)
    bct, bst = duqpp.quantize_weights_tiled(torch.zeros((40, 64), dtype=torch.bfloat16, device="cuda:0"), R)
    y = torch.full((33, 40), 7.0, dtype=torch.float32, device="cuda:0")
    L = duqpp.lib
    args = lambda T, dt=0, rp=Rp.data_ptr(), nb=2: (x.data_ptr(), 64, rp, nb, bct.data_ptr(), bst.data_ptr(), T, 40, 64, y.data_ptr(), dt, 40, None, None, None)
    assert L.duqpp_rotq_gemm_fused_decode(*args(8, 0, Rp.data_ptr(), 3)) == -2    # three blocks for two groups
    assert L.duqpp_rotq_gemm_fused_decode(*args(0)) == -2
    assert L.duqpp_rotq_gemm_fused_decode(*args(8, 3)) == -4
    assert L.duqpp_rotq_gemm_fused_decode(*args(8, 0, None)) == -1
    assert L.duqpp_rotq_gemm_fused_decode(*args(8, 0, Rp.data_ptr() + 8)) == -3
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
