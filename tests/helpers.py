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
