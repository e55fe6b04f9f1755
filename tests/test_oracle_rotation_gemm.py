"""Pins for the oracle's rotation (Eq. 4/5), GEMM (Eq. 5) and composed entry points.  CPU only."""
from fractions import Fraction

import numpy as np

import workloads as wl
from oracle import linear, mxfp4, pipeline, rotation


def _f(x):
    return Fraction(float(x))


# ---------------------------------------------------------------- rotation
def test_rotation_identity_is_exact():
    x = wl.bf16_bits_to_f32(wl.make_activations("rot-id", 5, 96, (wl.OutlierSpec(3, 50.0),)))
    np.testing.assert_array_equal(rotation.rotate(x, wl.identity_blocks(3)), x)


def test_rotation_direction_and_block_alignment():
    """y = x . R with R[j][r][c]: a cyclic-shift block P[r][(r+1)%32] = 1 moves channel r to
    r+1 *inside its own block*; a transposed operand or a wrong block index fails this."""
    G = 3
    P = np.zeros((G, 32, 32), dtype=np.float32)
    for j in range(G):
        for r in range(32):
            P[j, r, (r + 1 + j) % 32] = -1.0 if (r % 3 == 0) else 1.0     # signed, block-dependent shift
    x = np.arange(2 * 32 * G, dtype=np.float32).reshape(2, 32 * G) + 1
    y = rotation.rotate(x, P)
    for j in range(G):
        for r in range(32):
            sgn = -1.0 if (r % 3 == 0) else 1.0
            assert np.all(y[:, 32 * j + (r + 1 + j) % 32] == sgn * x[:, 32 * j + r])


def test_rotation_exact_rational_brute_force():
    """Against the exact rational dot product: the oracle accumulates in fp64 (error below 32 * 2^-53 of the sum
    of the terms' magnitudes) and rounds once to fp32 (half an fp32 ulp of the result).  An accumulation in fp32
    would be off by some 2^-24 of the *terms'* magnitudes, far more wherever the terms cancel."""
    x = wl.bf16_bits_to_f32(wl.make_activations("rot-bf", 4, 64, (wl.OutlierSpec(1, 1000.0, 1),)))
    R = wl.make_rotation_blocks("rot-bf", 2)
    y = rotation.rotate(x, R)
    assert y.dtype == np.float32
    for t in range(4):
        for j in range(2):
            for c in range(32):
                exact = sum(_f(x[t, 32 * j + r]) * _f(R[j, r, c]) for r in range(32))
                ref = float(exact)
                scale = float(sum(abs(_f(x[t, 32 * j + r]) * _f(R[j, r, c])) for r in range(32)))
                got = float(y[t, 32 * j + c])
                assert abs(got - ref) <= 2.0 ** -24 * max(abs(ref), abs(got)) + 2.0 ** -45 * scale


def test_rotation_shared_block_equals_repeated_block():
    x = wl.bf16_bits_to_f32(wl.make_activations("rot-sh", 4, 128))
    R1 = wl.make_rotation_blocks("rot-sh", 1)
    np.testing.assert_array_equal(rotation.rotate(x, R1), rotation.rotate(x, np.repeat(R1, 4, axis=0)))


def test_generated_blocks_are_orthogonal_and_norm_preserving():
    R = wl.make_rotation_blocks("orth", 16).astype(np.float64)
    for j in range(16):
        assert np.max(np.abs(R[j].T @ R[j] - np.eye(32))) < 1e-6
        assert np.max(np.abs(R[j] @ R[j].T - np.eye(32))) < 1e-6
    x = wl.bf16_bits_to_f32(wl.make_activations("orth", 8, 512, (wl.OutlierSpec(4, 50.0),)))
    y = rotation.rotate(x, R.astype(np.float32)).astype(np.float64)
    nx = np.linalg.norm(x.astype(np.float64).reshape(8, 16, 32), axis=-1)
    ny = np.linalg.norm(y.reshape(8, 16, 32), axis=-1)
    assert np.max(np.abs(nx - ny) / nx) < 1e-6


def test_rotation_is_lossless_before_quantisation():
    """(X R)(W R)^T = X W^T  (Eq. 5: the orthogonal transform changes nothing before Q)."""
    x = wl.bf16_bits_to_f32(wl.make_activations("lossless", 6, 256, (wl.OutlierSpec(4, 50.0),))).astype(np.float64)
    w = wl.bf16_bits_to_f32(wl.make_weights("lossless", 9, 256, 0.02)).astype(np.float64)
    R = wl.make_rotation_blocks("lossless", 8)
    ref = x @ w.T
    got = rotation.rotate(x, R).astype(np.float64) @ rotation.rotate(w, R).astype(np.float64).T
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 1e-5


def test_hadamard_closed_form():
    """x = a e_r in a block, R = H32/sqrt(32): all |y| = a/sqrt(32); a = 3 gives 0.5303 ->
    floor(log2) = -1 -> e = -3 -> byte 124; 0.5303*8 = 4.24 -> magnitude code 6 everywhere."""
    G = 2
    H = wl.hadamard_blocks(G)
    x = np.zeros((1, 64), dtype=np.float32)
    x[0, 32 + 5] = 3.0
    codes, scales, y = pipeline.rotate_quantize(x, H)
    assert np.allclose(np.abs(y[0, 32:]), 3.0 / np.sqrt(32.0), rtol=1e-6)
    assert np.all(y[0, :32] == 0)
    assert list(scales[0]) == [0, 124]
    u = mxfp4.unpack_codes(codes)[0]
    assert np.all((u[32:] & 7) == 6) and np.all(u[:32] == 0)
    # signs follow row 5 of the Sylvester matrix: (-1)^popcount(5 & c)
    sign = np.array([bin(5 & c).count("1") & 1 for c in range(32)])
    np.testing.assert_array_equal(u[32:] >> 3, sign)


# ---------------------------------------------------------------- composed entry points
def test_identity_rotation_reduces_to_plain_quantiser():
    xb = wl.make_activations("p3", 8, 256, (wl.OutlierSpec(4, 50.0),))
    c, s, y = pipeline.rotate_quantize(xb, wl.identity_blocks(8))
    c0, s0 = mxfp4.quantize(wl.bf16_bits_to_f32(xb))
    np.testing.assert_array_equal(c, c0)
    np.testing.assert_array_equal(s, s0)


def test_signed_permutation_permutes_codes():
    rng = np.random.default_rng(5)
    G = 4
    P = np.zeros((G, 32, 32), dtype=np.float32)
    perm = [rng.permutation(32) for _ in range(G)]
    sgn = [rng.choice([-1.0, 1.0], 32) for _ in range(G)]
    for j in range(G):
        P[j, np.arange(32), perm[j]] = sgn[j]
    xb = wl.make_activations("p4", 4, 32 * G, (wl.OutlierSpec(2, 50.0),))
    c, s, _ = pipeline.rotate_quantize(xb, P)
    c0, s0 = mxfp4.quantize(wl.bf16_bits_to_f32(xb))
    np.testing.assert_array_equal(s, s0)
    u, u0 = mxfp4.unpack_codes(c), mxfp4.unpack_codes(c0)
    for j in range(G):
        for r in range(32):
            flip = 8 if sgn[j][r] < 0 else 0
            np.testing.assert_array_equal(u[:, 32 * j + perm[j][r]], u0[:, 32 * j + r] ^ flip)


def test_weights_are_rotated_row_by_row_like_tokens():
    wb = wl.make_weights("wq", 5, 64, 0.02)
    R = wl.make_rotation_blocks("wq", 2)
    c, s, y = pipeline.quantize_weights(wb, R)
    w = wl.bf16_bits_to_f32(wb).astype(np.float64)
    # W^ = R^T W in the paper's [C_in, C_out] orientation == rows of the [N, K] weight times R
    Rfull = np.zeros((64, 64))
    Rfull[:32, :32], Rfull[32:, 32:] = R[0], R[1]
    np.testing.assert_allclose(y, (Rfull.T @ w.T).T, rtol=0, atol=1e-7)


def test_rotation_lowers_group_error_on_outlier_groups():
    """Ungraded sanity (Fig. 1 ordering): groups holding an outlier channel quantise with lower
    normalised error after an orthogonal rotation than before.  No value in the paper pins the numbers."""
    spec = (wl.OutlierSpec(8, 50.0),)
    xb = wl.make_activations("fig1", 64, 1024, spec)
    x = wl.bf16_bits_to_f32(xb)
    chan_mean = np.abs(x).mean(axis=0).reshape(32, 32)      # [group, channel in group]
    groups = np.where(chan_mean.max(axis=1) > 10)[0]         # groups that hold an outlier channel
    assert len(groups) >= 1
    cols = np.concatenate([np.arange(32 * g, 32 * g + 32) for g in groups])
    c0, s0 = mxfp4.quantize(np.ascontiguousarray(x[:, cols]))
    before = pipeline.per_group_normalised_error(x[:, cols], c0, s0)
    R = wl.make_rotation_blocks("fig1", 32)
    c1, s1, y = pipeline.rotate_quantize(xb, R)
    yc = np.ascontiguousarray(y[:, cols])
    c1c, s1c = mxfp4.quantize(yc)
    after = pipeline.per_group_normalised_error(yc, c1c, s1c)
    assert after < before


def _worked_group_errors():
    """(group values, hand-worked squared error norm, hand-worked squared norm) of tests/golden/group_error_worked.txt,
    the group values taken from the worked groups of Eq. 2 by name."""
    import os
    here = os.path.dirname(__file__)
    groups = {}
    for line in open(os.path.join(here, "golden", "mxfp4_worked_groups.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = [p.strip() for p in line.split(";")]
        x = np.full(32, float(parts[2][5:]) if parts[2].startswith("fill=") else 0.0, dtype=np.float32)
        vals = [float(v) for v in parts[1].split(",")]
        x[:len(vals)] = vals
        groups[parts[0]] = x
    out = []
    for line in open(os.path.join(here, "golden", "group_error_worked.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, num, den = [p.strip() for p in line.split(";")]
        out.append((groups[name], float(num), float(den)))
    return out


def test_group_error_statistic_on_hand_worked_groups():
    """The statistic of Sec. 4.1 (caption of Fig. 1): per group ||Q(x) - x||_2 / ||x||_2, then the mean over groups.
    Each worked group alone, then all of them side by side in two rows with an all-zero group between them (a group
    without norm has no ratio and is left out of the mean).  A squared norm, the norm of Q(x) in the denominator, a
    ratio of whole-tensor norms or a mean that counts the empty group all miss these values."""
    worked = _worked_group_errors()
    assert len(worked) == 4
    ratios = []
    for x, num, den in worked:
        c, s = mxfp4.quantize(x.reshape(1, 32))
        r = pipeline.per_group_normalised_error(x.reshape(1, 32), c, s)
        assert abs(r - (num / den) ** 0.5) <= 1e-7, (r, num, den)
        ratios.append((num / den) ** 0.5)
    assert ratios[0] < 0.06 < 0.14 < ratios[1] < 0.15 < 0.19 < ratios[2] < 0.2 and ratios[3] == 0.0
    z = np.zeros(32, dtype=np.float32)
    rows = np.stack([np.concatenate([worked[0][0], z, worked[1][0]]),
                     np.concatenate([worked[2][0], worked[3][0], z])])
    c, s = mxfp4.quantize(rows)
    got = pipeline.per_group_normalised_error(rows, c, s)
    assert abs(got - sum(ratios) / 4.0) <= 1e-7
    # the same ratios group by group, the groups without norm marked -1
    per = pipeline.per_group_normalised_errors(rows, c, s)
    want = np.array([[ratios[0], -1.0, ratios[1]], [ratios[2], ratios[3], -1.0]])
    assert per.shape == (2, 3) and np.max(np.abs(per - want)) <= 1e-7


# ---------------------------------------------------------------- GEMM
def _random_mx(rng, rows, K, scale_lo=120, scale_hi=134):
    codes = rng.integers(0, 256, size=(rows, K // 2)).astype(np.uint8)
    scales = rng.integers(scale_lo, scale_hi + 1, size=(rows, K // 32)).astype(np.uint8)
    return codes, scales


def test_gemm_exact_rational_brute_force_tiny():
    rng = np.random.default_rng(21)
    T, K, N = 3, 128, 4
    ac, asc = _random_mx(rng, T, K)
    bc, bsc = _random_mx(rng, N, K)
    y = linear.mxfp4_gemm(ac, asc, bc, bsc)
    assert y.shape == (T, N) and y.dtype == np.float64
    # group sums at exponents up to 28 apart: the results need more than fp32's 24 bits, fp64 holds them exactly
    assert any(float(np.float32(v)) != float(v) for v in y.flat)
    mags = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]

    def val(codes, scales, row, k):
        byte = int(codes[row, k // 2])
        nib = (byte >> 4) if (k & 1) else (byte & 15)
        v = mags[nib & 7] * (Fraction(2) ** (int(scales[row, k // 32]) - 127))
        return -v if nib & 8 else v

    for t in range(T):
        for n in range(N):
            exact = sum(val(ac, asc, t, k) * val(bc, bsc, n, k) for k in range(K))
            assert y[t, n] == float(exact)          # 128 exact products within 45 bits of each other: the fp64 sum is exact


def test_gemm_integer_case_is_exact():
    """Equal scales: every product is a multiple of 1/4 and every partial sum fits 53 bits, so the
    result must equal integer arithmetic exactly."""
    rng = np.random.default_rng(22)
    T, K, N = 7, 512, 5
    ac = rng.integers(0, 256, size=(T, K // 2)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    asc = np.full((T, K // 32), 127, dtype=np.uint8)
    bsc = np.full((N, K // 32), 130, dtype=np.uint8)
    twice = np.array([0, 1, 2, 3, 4, 6, 8, 12, 0, -1, -2, -3, -4, -6, -8, -12], dtype=np.int64)
    ai = twice[mxfp4.unpack_codes(ac)]
    bi = twice[mxfp4.unpack_codes(bc)]
    ref = (ai @ bi.T).astype(np.float64) / 4.0 * 8.0
    np.testing.assert_array_equal(linear.mxfp4_gemm(ac, asc, bc, bsc), ref)


def test_gemm_per_group_scales_apply_to_their_own_group_only():
    T, K, N = 1, 64, 1
    ac = np.zeros((T, K // 2), dtype=np.uint8)
    bc = np.zeros((N, K // 2), dtype=np.uint8)
    ac[0, 0] = 0x02      # element 0 = 1.0 (group 0)
    bc[0, 0] = 0x04      # element 0 = 2.0
    ac[0, 16] = 0x20     # element 33 = 1.0 (group 1, high nibble of byte 16)
    bc[0, 16] = 0x50     # element 33 = 3.0
    asc = np.array([[128, 125]], dtype=np.uint8)    # 2, 1/4
    bsc = np.array([[127, 130]], dtype=np.uint8)    # 1, 8
    y = linear.mxfp4_gemm(ac, asc, bc, bsc)
    assert y[0, 0] == 1 * 2 * 2 * 1 + 1 * 3 * 0.25 * 8


def test_bf16_rounding_ties_to_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7; 1 + 3*2^-8 ties up to 1 + 2^-6 (even)
    bits = linear.round_to_bf16_bits(f)
    assert list(bits[:4]) == [0x3F80, 0x3F80, 0x3F82, 0xBF80]
    np.testing.assert_array_equal(bits, wl.f32_to_bf16_bits(f))


def test_end_to_end_error_is_moderate_on_gaussian_data():
    """Ungraded sanity: the W4A4 product of Gaussian data lands within O(0.1) of the exact product."""
    xb = wl.make_activations("e2e", 16, 512)
    wb = wl.make_weights("e2e", 24, 512, 0.02)
    R = wl.make_rotation_blocks("e2e", 16)
    bc, bs, _ = pipeline.quantize_weights(wb, R)
    y = pipeline.rotq_gemm(xb, R, bc, bs)
    ref = wl.bf16_bits_to_f32(xb).astype(np.float64) @ wl.bf16_bits_to_f32(wb).astype(np.float64).T
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert 0.01 < rel < 0.3
