"""GPU parity: duqpp_rotate_quantize / duqpp_quantize_weights / duqpp_quantize_f32_dbg against the
CPU oracle, through the C ABI.  Bars: rotated values within 1e-5 of the block norm; scales and codes
bit-exact when the oracle quantises the device's own fp32 rotated values."""
import numpy as np
import pytest

import workloads as wl
from oracle import mxfp4, pipeline, rotation
from helpers import assert_codes_differ_only_at_boundaries, rotation_error_ratio, to_dev, to_dev_bf16

pytestmark = pytest.mark.gpu
ROT_TOL = 1e-5


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


def _check_rotq(env, xb, R, label):
    torch, duqpp = env
    x = to_dev_bf16(xb, torch)
    Rd = to_dev(R, torch)
    print(f"[rotq] {label} rows={xb.shape[0]} K={xb.shape[1]} n_rblocks={R.shape[0]}", flush=True)
    codes, scales, yrot = duqpp.rotate_quantize(x, Rd, return_rotated=True)
    torch.cuda.synchronize()
    codes, scales, yrot = codes.cpu().numpy(), scales.cpu().numpy(), yrot.cpu().numpy()
    xf = wl.bf16_bits_to_f32(xb)
    ratio = rotation_error_ratio(yrot, rotation.rotate(xf, R), xf)
    assert ratio <= ROT_TOL, ratio
    c_ref, s_ref = mxfp4.quantize(yrot)
    np.testing.assert_array_equal(scales, s_ref)
    np.testing.assert_array_equal(codes, c_ref)
    # the debug dump must not change the result
    c2, s2 = duqpp.rotate_quantize(x, Rd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(c2.cpu().numpy(), codes)
    np.testing.assert_array_equal(s2.cpu().numpy(), scales)
    return codes, scales, yrot


SHAPES = [
    (64, 4096),      # the q_proj reference case: several tiles, 8 column chunks
    (1, 4096),       # decode
    (16, 14336),     # decode, down_proj input
    (77, 1184),      # ragged token tail, odd number of groups (37), partial column chunk
    (33, 32),        # a single group
    (300, 2048),     # several token tiles per workgroup
]


@pytest.mark.parametrize("T,K", SHAPES)
def test_random_rotation(env, T, K):
    xb = wl.make_activations(f"gpu-rq-{T}-{K}", T, K, (wl.OutlierSpec(min(8, K // 4), 50.0),))
    R = wl.make_rotation_blocks(f"gpu-rq-{T}-{K}", K // 32)
    _check_rotq(env, xb, R, "random R")


def test_massive_outliers(env):
    T, K = 256, 14336
    xb = wl.make_activations("gpu-rq-massive", T, K, (wl.OutlierSpec(4, 1000.0, 8), wl.OutlierSpec(32, 20.0)))
    R = wl.make_rotation_blocks("gpu-rq-massive", K // 32)
    _check_rotq(env, xb, R, "massive outliers")


def test_identity_rotation_is_the_plain_quantiser(env):
    T, K = 70, 1024
    xb = wl.make_activations("gpu-rq-id", T, K, (wl.OutlierSpec(8, 50.0),))
    codes, scales, yrot = _check_rotq(env, xb, wl.identity_blocks(K // 32), "identity")
    xf = wl.bf16_bits_to_f32(xb)
    np.testing.assert_array_equal(yrot, xf)                       # exact: 1.0 splits into (1, 0, 0)
    c0, s0 = mxfp4.quantize(xf)
    np.testing.assert_array_equal(codes, c0)
    np.testing.assert_array_equal(scales, s0)


def test_signed_permutation_is_exact(env):
    rng = np.random.default_rng(9)
    T, K = 40, 256
    G = K // 32
    P = np.zeros((G, 32, 32), dtype=np.float32)
    for j in range(G):
        P[j, np.arange(32), rng.permutation(32)] = rng.choice([-1.0, 1.0], 32)
    xb = wl.make_activations("gpu-rq-perm", T, K, (wl.OutlierSpec(2, 50.0),))
    codes, scales, yrot = _check_rotq(env, xb, P, "signed permutation")
    c_ref, s_ref, y_ref = pipeline.rotate_quantize(xb, P)
    np.testing.assert_array_equal(yrot, y_ref)
    np.testing.assert_array_equal(codes, c_ref)
    np.testing.assert_array_equal(scales, s_ref)


def test_hadamard_and_shared_block(env):
    T, K = 64, 2048
    xb = wl.make_activations("gpu-rq-had", T, K, (wl.OutlierSpec(8, 50.0),))
    _check_rotq(env, xb, wl.hadamard_blocks(K // 32), "hadamard")
    R1 = wl.make_rotation_blocks("gpu-rq-shared", 1)
    c1, s1, y1 = _check_rotq(env, xb, R1, "one shared block")
    c2, s2, y2 = _check_rotq(env, xb, np.repeat(R1, K // 32, axis=0), "same block repeated")
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(s1, s2)
    np.testing.assert_array_equal(y1, y2)


def test_strided_input_rows(env):
    torch, duqpp = env
    T, K, ld = 50, 512, 640
    xb = wl.make_activations("gpu-rq-ld", T, ld)
    R = wl.make_rotation_blocks("gpu-rq-ld", K // 32)
    xfull = to_dev_bf16(xb, torch)
    codes, scales = duqpp.rotate_quantize(xfull[:, :K], to_dev(R, torch))
    c_ref, s_ref = duqpp.rotate_quantize(xfull[:, :K].contiguous(), to_dev(R, torch))
    torch.cuda.synchronize()
    assert torch.equal(codes, c_ref) and torch.equal(scales, s_ref)


@pytest.mark.parametrize("T,K,spec", [
    (128, 4096, (wl.OutlierSpec(8, 50.0),)),
    (2048, 4096, (wl.OutlierSpec(8, 50.0), wl.OutlierSpec(4, 1000.0, 8))),
])
def test_end_to_end_codes_differ_only_at_rounding_boundaries(env, T, K, spec):
    """Device rotation vs oracle rotation, each quantised by its own side: not bit-exact by construction (the fp32
    sums differ in the last bits), but at most 1e-5 of the codes and scales may differ, and each difference must sit
    where the rotation tolerance allows one: the oracle's value within 1e-5 * ||x_block||_2 of a rounding boundary
    of Eq. 2, or its group maximum that close to a power of two."""
    torch, duqpp = env
    xb = wl.make_activations(f"gpu-rq-e2e-{T}", T, K, spec)
    R = wl.make_rotation_blocks(f"gpu-rq-e2e-{T}", K // 32)
    codes, scales = duqpp.rotate_quantize(to_dev_bf16(xb, torch), to_dev(R, torch))
    torch.cuda.synchronize()
    c_ref, s_ref, y_ref = pipeline.rotate_quantize(xb, R)
    n_c, n_s = assert_codes_differ_only_at_boundaries(codes.cpu().numpy(), scales.cpu().numpy(), c_ref, s_ref, y_ref,
                                                      wl.bf16_bits_to_f32(xb))
    print(f"[rotq] end-to-end T={T}: {n_c} of {T * K} codes and {n_s} of {T * K // 32} scales differ", flush=True)


def test_quantize_weights(env):
    torch, duqpp = env
    N, K = 200, 1184
    wb = wl.make_weights("gpu-qw", N, K, 0.02)
    R = wl.make_rotation_blocks("gpu-qw", K // 32)
    codes, scales = duqpp.quantize_weights(to_dev_bf16(wb, torch), to_dev(R, torch))
    c2, s2, yrot = duqpp.rotate_quantize(to_dev_bf16(wb, torch), to_dev(R, torch), return_rotated=True)
    torch.cuda.synchronize()
    assert torch.equal(codes, c2) and torch.equal(scales, s2)     # same transform as for a token
    c_ref, s_ref = mxfp4.quantize(yrot.cpu().numpy())
    np.testing.assert_array_equal(codes.cpu().numpy(), c_ref)
    np.testing.assert_array_equal(scales.cpu().numpy(), s_ref)
    wf = wl.bf16_bits_to_f32(wb)
    assert rotation_error_ratio(yrot.cpu().numpy(), rotation.rotate(wf, R), wf) <= ROT_TOL


# ---------------------------------------------------------------- the quantiser stage alone
def _dbg_check(env, y):
    torch, duqpp = env
    codes, scales = duqpp.quantize_f32_dbg(to_dev(y, torch))
    torch.cuda.synchronize()
    c_ref, s_ref = mxfp4.quantize(y)
    np.testing.assert_array_equal(scales.cpu().numpy(), s_ref)
    np.testing.assert_array_equal(codes.cpu().numpy(), c_ref)


def test_quantiser_stage_every_bf16_pattern(env):
    bits = np.arange(0, 1 << 16, dtype=np.uint32)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]                    # NaN/Inf are outside the contract
    v = (bits << 16).view(np.float32)
    rng = np.random.default_rng(0)
    for trial in range(3):
        p = rng.permutation(v)
        p = np.concatenate([p, np.zeros((-len(p)) % 64, dtype=np.float32)]).reshape(-1, 64)
        _dbg_check(env, np.ascontiguousarray(p))
    # sorted: neighbours share a scale, so the whole E2M1 range of each binade is exercised
    s = np.sort(v)
    s = np.concatenate([s, np.zeros((-len(s)) % 64, dtype=np.float32)]).reshape(-1, 64)
    _dbg_check(env, np.ascontiguousarray(s))


def test_quantiser_stage_random_fp32_patterns(env):
    rng = np.random.default_rng(1)
    n = 1 << 22
    bits = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    bits[((bits >> 23) & 0xFF) == 0xFF] &= np.uint32(0x807FFFFF)  # turn NaN/Inf into subnormals
    y = bits.view(np.float32).reshape(-1, 128)
    _dbg_check(env, y)
    # same mantissas squeezed into a few binades so that values in a group compete for one scale
    e = rng.integers(120, 134, size=n, dtype=np.uint64).astype(np.uint32)
    y2 = ((bits & np.uint32(0x807FFFFF)) | (e << np.uint32(23))).view(np.float32).reshape(-1, 128)
    _dbg_check(env, y2)
    # subnormal and near-minimum groups (scale clamp at 2^-127)
    e3 = rng.integers(0, 4, size=n, dtype=np.uint64).astype(np.uint32)
    y3 = ((bits & np.uint32(0x807FFFFF)) | (e3 << np.uint32(23))).view(np.float32).reshape(-1, 128)
    _dbg_check(env, y3)
    # top of the fp32 range
    e4 = rng.integers(250, 255, size=n // 8, dtype=np.uint64).astype(np.uint32)
    y4 = ((bits[: n // 8] & np.uint32(0x807FFFFF)) | (e4 << np.uint32(23))).view(np.float32).reshape(-1, 128)
    _dbg_check(env, y4)


def test_quantiser_stage_every_value_near_every_threshold(env):
    """All fp32 values within 512 ulp of each rounding boundary, at many scales, next to a 4.0."""
    ths = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 7.0, 8.0], dtype=np.float32)
    rows = []
    for th in ths:
        base = int(th.view(np.uint32))
        pats = np.arange(base - 512, base + 512, dtype=np.uint32).view(np.float32)
        for sgn in (1.0, -1.0):
            g = np.zeros((len(pats), 32), dtype=np.float32)
            g[:, 0] = 4.0
            g[:, 7] = sgn * pats
            rows.append(g)
    base = np.concatenate(rows)
    for e in (-125, -60, -3, 0, 1, 17, 100, 120):
        _dbg_check(env, np.ldexp(base.astype(np.float64), e).astype(np.float32))
    z = np.zeros((64, 64), dtype=np.float32)
    z[::2] = -0.0
    _dbg_check(env, z)


def test_groups_are_independent_on_the_device(env):
    """Sec. 4.2: every group of 32 has its own scale, so changing one block of the input changes the codes and the
    scale of that group only (for the tokens changed) -- checked on the device's output byte for byte."""
    torch, duqpp = env
    T, K = 96, 2048
    G = K // 32
    xb = wl.make_activations("gpu-rq-indep", T, K, (wl.OutlierSpec(8, 50.0),))
    R = to_dev(wl.make_rotation_blocks("gpu-rq-indep", G), torch)
    c0, s0 = duqpp.rotate_quantize(to_dev_bf16(xb, torch), R)
    xb2 = xb.copy()
    j, toks = 37, np.array([0, 31, 32, 95])
    xb2[toks[:, None], 32 * j + np.arange(32)[None, :]] = wl.f32_to_bf16_bits(
        1000.0 * wl.bf16_bits_to_f32(xb[toks[:, None], 32 * j + np.arange(32)[None, :]]) + 3.0)
    c1, s1 = duqpp.rotate_quantize(to_dev_bf16(xb2, torch), R)
    torch.cuda.synchronize()
    c0, s0, c1, s1 = (t.cpu().numpy() for t in (c0, s0, c1, s1))
    same_c = (c0.reshape(T, G, 16) == c1.reshape(T, G, 16)).all(axis=-1)
    same_s = s0 == s1
    touched = np.zeros((T, G), dtype=bool)
    touched[toks, j] = True
    assert same_c[~touched].all() and same_s[~touched].all()
    assert not same_s[touched].any()                     # a thousandfold input moves every touched group's scale


def test_representable_inputs_survive_the_device_quantiser(env):
    """dequant(quant(x)) = x for values that are E2M1 values times a power of two with the group's largest magnitude
    4 or 6 (so that the scale is that power of two), and quantising the decoded values again gives the same bytes."""
    torch, duqpp = env
    rng = np.random.default_rng(11)
    mags = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    rows, K = 256, 256
    v = mags[rng.integers(0, 8, size=(rows, K))] * rng.choice([-1.0, 1.0], size=(rows, K))
    v.reshape(rows, K // 32, 32)[:, :, 5] = rng.choice([4.0, 6.0, -4.0, -6.0], size=(rows, K // 32))
    e = rng.integers(-100, 100, size=(rows, K // 32))
    y = np.ldexp(v, np.repeat(e, 32, axis=1)).astype(np.float32)
    codes, scales = duqpp.quantize_f32_dbg(to_dev(y, torch))
    torch.cuda.synchronize()
    codes, scales = codes.cpu().numpy(), scales.cpu().numpy()
    np.testing.assert_array_equal(scales, (e + 127).astype(np.uint8))
    back = mxfp4.dequantize(codes, scales)
    np.testing.assert_array_equal(back, y.astype(np.float64))
    c2, s2 = duqpp.quantize_f32_dbg(to_dev(back.astype(np.float32), torch))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(c2.cpu().numpy(), codes)
    np.testing.assert_array_equal(s2.cpu().numpy(), scales)
