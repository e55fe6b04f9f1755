"""GPU parity of every tiled MXFP4 GEMM kernel at shapes the library would not pick it for: each kernel is run by
name through duqpp_mxfp4_gemm_tiled_on and compared with the CPU oracle's product (Eq. 5 on given codes)."""
import numpy as np
import pytest

import workloads as wl
from oracle import linear
from helpers import bf16_dev_to_bits, rel_fro, tile_np, to_dev

pytestmark = pytest.mark.gpu
GEMM_TOL = 1e-5
DECODE, SMALL, MID, LARGE = 1, 2, 3, 4
NAMES = {DECODE: "decode", SMALL: "64x128", MID: "128x256", LARGE: "256x256"}


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


def _run(env, kernel, ac, asc, bc, bsc, out_dtype=0, out=None):
    torch, duqpp = env
    T, K, N = ac.shape[0], ac.shape[1] * 2, bc.shape[0]
    act, ast = tile_np(ac, asc)
    bct, bst = tile_np(bc, bsc)
    y = duqpp.mxfp4_gemm_tiled(to_dev(act, torch), to_dev(ast, torch), to_dev(bct, torch), to_dev(bst, torch),
                               T, N, K, out_dtype=out_dtype, kernel=kernel, out=out)
    torch.cuda.synchronize()
    return y


# shapes chosen per kernel: one tile, ragged edges in T, N and in the padded groups, one and several K steps,
# more tiles than CUs (several tiles per persistent workgroup)
SHAPES = [
    (LARGE, 256, 256, 128),       # one tile, one pair of K steps
    (LARGE, 256, 256, 32),        # a single group: seven of the eight padded groups are padding
    (LARGE, 300, 523, 1056),      # ragged in T and N, 33 groups padded to 40
    (LARGE, 31, 70, 2336),        # far smaller than a tile
    (LARGE, 513, 1030, 288),
    (LARGE, 4200, 4200, 32),      # 17 x 17 = 289 tiles: two tiles for some workgroups, transfers running on
    (LARGE, 1100, 8300, 544),
    (MID, 31, 70, 2336),
    (MID, 64, 96, 512),
    (SMALL, 2100, 4200, 32),      # 33 x 33 = 1089 tiles
    (SMALL, 300, 523, 1056),
    (DECODE, 128, 300, 1184),
    (DECODE, 100, 8200, 544),
]


@pytest.mark.parametrize("kernel,T,N,K", SHAPES)
def test_named_kernel_random_codes(env, kernel, T, N, K):
    rng = np.random.default_rng(kernel * 7919 + T * 1000003 + N * 1009 + K)
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    print(f"[gemm kernel {NAMES[kernel]}] random codes T={T} N={N} K={K}", flush=True)
    y = _run(env, kernel, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    assert rel_fro(y, ref) <= GEMM_TOL


@pytest.mark.parametrize("kernel", [SMALL, MID, LARGE])
def test_named_kernel_exact_integer_case(env, kernel):
    """Equal scales: every partial sum is a multiple of a quarter unit below 2^24, so any summation order gives the
    oracle's value bit for bit."""
    rng = np.random.default_rng(78 + kernel)
    T, N, K = 290, 330, 14336
    ac = rng.integers(0, 256, size=(T, K // 2)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    asc = np.full((T, K // 32), 125, dtype=np.uint8)
    bsc = np.full((N, K // 32), 131, dtype=np.uint8)
    print(f"[gemm kernel {NAMES[kernel]}] exact integer case", flush=True)
    y = _run(env, kernel, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    np.testing.assert_array_equal(y, ref.astype(np.float32))


@pytest.mark.parametrize("kernel", [SMALL, MID, LARGE])
def test_named_kernel_scale_bytes_pair_with_their_own_group(env, kernel):
    """One non-zero element per group and scales that differ from group to group and row to row: a scale byte
    applied to the wrong group, row or operand changes the (exact) result."""
    T, N, K = 270, 300, 1024
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
    y = _run(env, kernel, ac, asc, bc, bsc).cpu().numpy()
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    np.testing.assert_array_equal(y, ref.astype(np.float32))   # sums of at most 32 powers of two within 2^17: exact


@pytest.mark.parametrize("kernel,T,N,K", [(LARGE, 300, 520, 1056), (LARGE, 2100, 4200, 64), (LARGE, 70, 200, 1024),
                                          (MID, 300, 523, 1056), (SMALL, 300, 523, 1056)])
def test_named_kernel_bf16_output(env, kernel, T, N, K):
    """bf16 output = round-to-nearest-even of the same kernel's fp32 output, bit for bit; and within one bf16
    rounding of the oracle where sums do not cancel."""
    rng = np.random.default_rng(14 + kernel)
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    print(f"[gemm kernel {NAMES[kernel]}] bf16 output T={T} N={N} K={K}", flush=True)
    y32 = _run(env, kernel, ac, asc, bc, bsc, 0).cpu().numpy()
    y16 = bf16_dev_to_bits(_run(env, kernel, ac, asc, bc, bsc, 1))
    np.testing.assert_array_equal(y16, linear.round_to_bf16_bits(y32))
    ref = linear.mxfp4_gemm(ac, asc, bc, bsc)
    val = wl.bf16_bits_to_f32(y16).astype(np.float64)
    assert np.all(np.abs(val - ref) <= 2.0 ** -8 * np.abs(ref) + GEMM_TOL * np.max(np.abs(ref)))


def test_named_kernel_rejections(env):
    """A kernel that cannot run a call says so instead of running something else."""
    torch, duqpp = env
    rng = np.random.default_rng(3)
    ac, asc = _random_mx(rng, 200, 64)
    bc, bsc = _random_mx(rng, 70, 64)
    with pytest.raises(duqpp.DuqppError):
        _run(env, DECODE, ac, asc, bc, bsc)                # 200 tokens > 128
    with pytest.raises(duqpp.DuqppError):
        _run(env, LARGE, ac, asc, bc, bsc, 1)              # bf16 output with N = 70 not a multiple of 8
    with pytest.raises(duqpp.DuqppError):
        _run(env, 9, ac, asc, bc, bsc)
    y = _run(env, LARGE, ac, asc, bc, bsc, 0).cpu().numpy()   # fp32 output is fine
    assert rel_fro(y, linear.mxfp4_gemm(ac, asc, bc, bsc)) <= GEMM_TOL


@pytest.mark.parametrize("kernel,T,N,K", [(DECODE, 100, 328, 544), (SMALL, 300, 520, 288), (MID, 300, 520, 288),
                                          (LARGE, 300, 520, 288)])
@pytest.mark.parametrize("out_dtype", [0, 1])
@pytest.mark.parametrize("pad", [8, 3])
def test_named_kernel_strided_output(env, kernel, T, N, K, out_dtype, pad):
    """Rows of the result `ldy` = N + pad elements apart: the same values as into a dense result, and nothing
    written between the rows.  pad = 3 leaves bf16 rows off the 16-byte grid: the 256 x 256 kernel refuses that
    call, the others store element by element."""
    torch, duqpp = env
    rng = np.random.default_rng(kernel * 31 + out_dtype * 7 + pad)
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    print(f"[gemm kernel {NAMES[kernel]}] strided output T={T} N={N} K={K} dtype={out_dtype} ldy=N+{pad}", flush=True)
    dense = _run(env, kernel, ac, asc, bc, bsc, out_dtype)
    sentinel = -77.0
    big = torch.full((T, N + pad), sentinel, dtype=dense.dtype, device=dense.device)
    if kernel == LARGE and out_dtype == 1 and pad % 8:
        with pytest.raises(duqpp.DuqppError):
            _run(env, kernel, ac, asc, bc, bsc, out_dtype, out=big[:, :N])
        return
    _run(env, kernel, ac, asc, bc, bsc, out_dtype, out=big[:, :N])
    assert torch.equal(big[:, :N], dense)
    assert torch.all(big[:, N:] == sentinel)
    assert rel_fro(dense.float().cpu().numpy(), linear.mxfp4_gemm(ac, asc, bc, bsc)) <= (GEMM_TOL if out_dtype == 0 else 2.0 ** -8)
