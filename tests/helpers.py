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
