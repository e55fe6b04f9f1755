"""Shared helpers for the GPU parity tests (data movement and error statistics only)."""
import numpy as np


def to_dev_bf16(bits_u16, torch, dev="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).view(torch.bfloat16).to(dev)


def to_dev(a, torch, dev="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def bf16_dev_to_bits(t):
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def rotation_error_ratio(y_gpu, y_ref, x_f32):
    """max over groups of  max_c |y_gpu - y_ref| / ||x_block||_2  (the block norm bounds every
    rotated entry because the block is orthogonal); groups with zero norm must match exactly."""
    rows, K = y_ref.shape
    G = K // 32
    err = np.abs(y_gpu.astype(np.float64) - y_ref.astype(np.float64)).reshape(rows, G, 32).max(axis=-1)
    nrm = np.linalg.norm(x_f32.astype(np.float64).reshape(rows, G, 32), axis=-1)
    assert np.all(err[nrm == 0] == 0)
    ok = nrm > 0
    return float(np.max(err[ok] / nrm[ok])) if np.any(ok) else 0.0


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


E2M1_BOUNDARIES = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])     # rounding boundaries of Eq. 2 in units of the scale


def assert_codes_differ_only_at_boundaries(codes, scales, c_ref, s_ref, y_ref, x_f32, tol=1e-5, max_fraction=1e-5):
    """Device codes / scales (each side rotated in its own precision) against the oracle's, both row-major.
    The device's rotated values lie within tol * ||x_block||_2 of the oracle's y_ref, so a differing scale needs the
    oracle's group maximum within that distance of a power of two (and differs by one), and a differing code in a
    group with equal scales needs the oracle's |y| / s within tol * ||x_block||_2 / s of a rounding boundary of Eq. 2
    (and is the neighbouring code; its sign may differ only if |y| itself is that small).  At most max_fraction of the
    codes and of the scales may differ at all.  Returns (differing codes, differing scales)."""
    rows, G = s_ref.shape
    u = np.stack([codes & 0xF, codes >> 4], axis=-1).reshape(rows, G, 32)
    u_ref = np.stack([c_ref & 0xF, c_ref >> 4], axis=-1).reshape(rows, G, 32)
    y = np.abs(np.asarray(y_ref, dtype=np.float64)).reshape(rows, G, 32)
    slack = tol * np.linalg.norm(np.asarray(x_f32, dtype=np.float64).reshape(rows, G, 32), axis=-1)     # [rows, G]
    ds = scales != s_ref
    for t, j in zip(*np.nonzero(ds)):
        assert abs(int(scales[t, j]) - int(s_ref[t, j])) == 1, (t, j, scales[t, j], s_ref[t, j])
        amax = y[t, j].max()
        edge = 2.0 ** (max(int(scales[t, j]), int(s_ref[t, j])) - 127 + 2)      # the power of two between the two scales
        assert abs(amax - edge) <= slack[t, j], (t, j, amax, edge, slack[t, j])
    dc = (u != u_ref) & ~ds[:, :, None]
    for t, j, i in zip(*np.nonzero(dc)):
        s = 2.0 ** (int(s_ref[t, j]) - 127)
        v = y[t, j, i] / s
        a, b = int(u[t, j, i]), int(u_ref[t, j, i])
        if (a ^ b) & 8:
            assert y[t, j, i] <= slack[t, j], (t, j, i, "sign", y[t, j, i], slack[t, j])
        assert abs((a & 7) - (b & 7)) <= 1, (t, j, i, a, b)
        if (a & 7) != (b & 7):
            assert np.min(np.abs(E2M1_BOUNDARIES - v)) <= slack[t, j] / s, (t, j, i, v, slack[t, j] / s)
    n_c, n_s = int(dc.sum()), int(ds.sum())
    assert n_c <= max(1, int(max_fraction * u.size)) and n_s <= max(1, int(max_fraction * ds.size)), (n_c, n_s)
    return n_c, n_s


def per_element_gemm_bound(a_codes, a_scales, b_codes, b_scales, dequantize):
    """sum_k |a[t, k]| |b[n, k]|: what an fp32 accumulation error of a product sum is relative to."""
    return np.abs(dequantize(a_codes, a_scales)) @ np.abs(dequantize(b_codes, b_scales)).T


# ---- the tiled operand layout, restated in numpy (index arithmetic only) ----
def tiled_shape(rows, K):
    G = K // 32
    return (rows + 31) // 32, (G + 7) // 8 * 8


def tile_np(codes, scales):
    """Row-major [rows, K/2] + [rows, G] -> flat tiled codes [RT][GP][32][16] and scales [RT][GP/8][2][32][4]."""
    rows, G = scales.shape
    RT, GP = tiled_shape(rows, G * 32)
    c = np.zeros((RT * 32, GP, 16), dtype=np.uint8)
    s = np.full((RT * 32, GP), 127, dtype=np.uint8)
    c[:rows, :G] = codes.reshape(rows, G, 16)
    s[:rows, :G] = scales
    ct = c.reshape(RT, 32, GP, 16).transpose(0, 2, 1, 3)                      # [rt][j][r][16]
    st = s.reshape(RT, 32, GP // 8, 2, 4).transpose(0, 2, 3, 1, 4)            # [rt][q][g][r][b]
    return np.ascontiguousarray(ct).reshape(-1), np.ascontiguousarray(st).reshape(-1)


def untile_np(codes_t, scales_t, rows, K):
    """Inverse of tile_np; also returns the padding so that tests can check it."""
    G = K // 32
    RT, GP = tiled_shape(rows, K)
    c = codes_t.reshape(RT, GP, 32, 16).transpose(0, 2, 1, 3).reshape(RT * 32, GP, 16)
    s = scales_t.reshape(RT, GP // 8, 2, 32, 4).transpose(0, 3, 1, 2, 4).reshape(RT * 32, GP)
    codes = np.ascontiguousarray(c[:rows, :G]).reshape(rows, G * 16)
    scales = np.ascontiguousarray(s[:rows, :G])
    pad_codes = np.concatenate([c[rows:].reshape(-1), c[:rows, G:].reshape(-1)])
    pad_scales = np.concatenate([s[rows:].reshape(-1), s[:rows, G:].reshape(-1)])
    return codes, scales, pad_codes, pad_scales
