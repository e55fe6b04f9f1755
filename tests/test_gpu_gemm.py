"""GPU parity: duqpp_mxfp4_gemm and duqpp_rotq_gemm against the CPU oracle, through the C ABI.
Bar: relative Frobenius error <= 1e-5 on the same codes (fp32 output); bit-exact when every partial
sum is exactly representable; bf16 output = round-to-nearest-even of the kernel's own fp32 result."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear, mxfp4, pipeline
from helpers import bf16_dev_to_bits, rel_fro, to_dev, to_dev_bf16

pytestmark = pytest.mark.gpu
GEMM_TOL = 1e-5


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


_WS = None    # workspace argument of the row-major call: None = scratch allocated (re-tile + fast kernel), False = direct kernel


@pytest.fixture(params=["scratch", "direct"], autouse=True)
def gemm_path(request):
    """Every test of this module runs on both code paths behind duqpp_mxfp4_gemm."""
    global _WS
    _WS = None if request.param == "scratch" else False
    yield request.param


def _random_mx(rng, rows, K, lo=118, hi=136):
    codes = rng.integers(0, 256, size=(rows, K // 2)).astype(np.uint8)
    scales = rng.integers(lo, hi + 1, size=(rows, K // 32)).astype(np.uint8)
    return codes, scales


def _gemm(env, ac, asc, bc, bsc, out_dtype=0):
    torch, duqpp = env
    y = duqpp.mxfp4_gemm(to_dev(ac, torch), to_dev(asc, torch), to_dev(bc, torch), to_dev(bsc, torch), out_dtype=out_dtype,
                         workspace=_WS)
    torch.cuda.synchronize()
    return y


SHAPES = [
    (64, 96, 512),
    (77, 130, 1184),      # ragged in T, N and an odd number of groups (scale rows not word aligned)
    (1, 257, 4096),       # decode
    (16, 300, 2048),
    (130, 70, 32),        # a single group
    (200, 264, 2304),     # K = 9 * 256: exact multiple of the K step
    (129, 129, 1312),     # 41 groups: ragged K tail, scale rows not word aligned
]


@pytest.mark.parametrize("T,N,K", SHAPES)
def test_random_codes(env, T, N, K):
    rng = np.random.default_rng(T * 1000003 + N * 1009 + K)
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    print(f"[gemm] random codes T={T} N={N} K={K}", flush=True)
    y = _gemm(env, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    assert rel_fro(y, ref) <= GEMM_TOL


def test_exact_integer_case_is_bit_exact(env):
    """Equal scales per operand: all products are multiples of 1/4 (times one power of two) and every
    partial sum stays below 2^24 quarter-units, so any summation order gives the same fp32 result."""
    rng = np.random.default_rng(77)
    T, N, K = 96, 160, 14336
    ac = rng.integers(0, 256, size=(T, K // 2)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    asc = np.full((T, K // 32), 125, dtype=np.uint8)
    bsc = np.full((N, K // 32), 131, dtype=np.uint8)
    y = _gemm(env, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    np.testing.assert_array_equal(y, ref.astype(np.float32))
    assert np.all(ref == ref.astype(np.float32))


def test_scale_bytes_pair_with_their_own_group(env):
    """One nonzero element per group with a distinct power-of-two scale per group and row: any mix-up
    of scale bytes between groups, rows or operands changes the (exactly representable) result."""
    T, N, K = 40, 48, 512
    G = K // 32
    rng = np.random.default_rng(5)
    ac = np.zeros((T, K // 2), dtype=np.uint8)
    bc = np.zeros((N, K // 2), dtype=np.uint8)
    pos_a = rng.integers(0, 32, size=G)
    for j in range(G):
        k = 32 * j + int(pos_a[j])
        ac[:, k // 2] = 0x02 << (4 * (k & 1))       # 1.0 at element k
        bc[:, k // 2] = 0x02 << (4 * (k & 1))
    asc = (127 + (np.arange(T)[:, None] % 3) + np.zeros((1, G), dtype=int)).astype(np.uint8)
    asc = (asc + (np.arange(G)[None, :] % 2)).astype(np.uint8)
    bsc = (120 + (np.arange(N)[:, None] % 5) - 0 * np.arange(G)[None, :]).astype(np.uint8)
    bsc = (bsc + np.arange(G)[None, :] % 4).astype(np.uint8)
    y = _gemm(env, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    np.testing.assert_array_equal(y, ref.astype(np.float32))


def test_bf16_output(env):
    rng = np.random.default_rng(12)
    T, N, K = 70, 200, 1024
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    y32 = _gemm(env, ac, asc, bc, bsc, 0).cpu().numpy()
    y16 = bf16_dev_to_bits(_gemm(env, ac, asc, bc, bsc, 1))
    np.testing.assert_array_equal(y16, linear.round_to_bf16_bits(y32))          # RNE of its own fp32 result
    ref16 = linear.round_to_bf16_bits(linear.mxfp4_gemm(ac, asc, bc, bsc).astype(np.float32))
    assert np.max(np.abs(y16.astype(np.int32) - ref16.astype(np.int32))) <= 1     # within one bf16 ulp of the oracle


def test_strided_output(env):
    torch, duqpp = env
    rng = np.random.default_rng(13)
    T, N, K = 33, 100, 256
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    big = torch.full((T, 128), -7.0, dtype=torch.float32, device="cuda:0")
    duqpp.mxfp4_gemm(to_dev(ac, torch), to_dev(asc, torch), to_dev(bc, torch), to_dev(bsc, torch), out=big[:, :N], workspace=_WS)
    torch.cuda.synchronize()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    assert rel_fro(big[:, :N].cpu().numpy(), ref) <= GEMM_TOL
    assert torch.all(big[:, N:] == -7.0)


def test_whole_path_on_the_reference_config(env):
    """T=64, K=4096, N=4096 (q_proj shape): weights prepared on the device, activations rotated and
    quantised on the device, product against the oracle on the same codes; the fused call must give
    exactly what the two separate calls give."""
    torch, duqpp = env
    cfg = wl.CONFIGS["c1_qproj_T64"]
    T, K, N = cfg["T"], cfg["K"], cfg["N"]
    xb = wl.make_activations("c1", T, K, cfg["outliers"])
    wb = wl.make_weights("c1", N, K, cfg["w_std"])
    R = wl.make_rotation_blocks("c1", K // 32)
    x, w, Rd = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch), to_dev(R, torch)
    bc, bs = duqpp.quantize_weights(w, Rd)
    ac, asc = duqpp.rotate_quantize(x, Rd)
    y = duqpp.mxfp4_gemm(ac, asc, bc, bs, workspace=_WS)
    yf = duqpp.rotq_gemm(x, Rd, bc, bs)
    torch.cuda.synchronize()
    ref = linear.mxfp4_gemm(ac.cpu().numpy(), asc.cpu().numpy(), bc.cpu().numpy(), bs.cpu().numpy())
    assert rel_fro(y.cpu().numpy(), ref) <= GEMM_TOL
    # the fused call is the fast separate call (same kernel, same order of additions): bit-identical
    assert torch.equal(duqpp.mxfp4_gemm(ac, asc, bc, bs), yf)
    assert rel_fro(yf.cpu().numpy(), ref) <= GEMM_TOL
    # ungraded sanity: the W4A4 result approximates the unquantised product
    exact = wl.bf16_bits_to_f32(xb).astype(np.float64) @ wl.bf16_bits_to_f32(wb).astype(np.float64).T
    e = rel_fro(y.cpu().numpy(), exact)
    print(f"[gemm] W4A4 vs exact product, relative error {e:.3f}", flush=True)
    assert e < 0.5


@pytest.mark.parametrize("T,N,K", [(1, 512, 4096), (4, 300, 14336), (16, 4096, 1184), (100, 200, 1024)])
def test_fused_call_equals_separate_calls(env, T, N, K):
    torch, duqpp = env
    xb = wl.make_activations(f"fused-{T}", T, K, (wl.OutlierSpec(8, 50.0),))
    wb = wl.make_weights(f"fused-{T}", N, K, 0.02)
    R = wl.make_rotation_blocks(f"fused-{T}", K // 32)
    x, w, Rd = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch), to_dev(R, torch)
    bc, bs = duqpp.quantize_weights(w, Rd)
    ac, asc = duqpp.rotate_quantize(x, Rd)
    for dt in (0, 1):
        y = duqpp.mxfp4_gemm(ac, asc, bc, bs, out_dtype=dt)
        yf = duqpp.rotq_gemm(x, Rd, bc, bs, out_dtype=dt)
        torch.cuda.synchronize()
        assert torch.equal(y, yf)                           # same kernel, same order of additions
    ref = linear.mxfp4_gemm(ac.cpu().numpy(), asc.cpu().numpy(), bc.cpu().numpy(), bs.cpu().numpy())
    assert rel_fro(duqpp.mxfp4_gemm(ac, asc, bc, bs, workspace=_WS).cpu().numpy(), ref) <= GEMM_TOL
