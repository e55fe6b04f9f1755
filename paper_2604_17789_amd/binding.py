"""ctypes binding with the same names as the C ABI (include/duqpp.h).  Argument marshalling only."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libduqpp.so"

F32, BF16 = 0, 1
# kernels of the tiled GEMM (the DUQPP_GEMM_KERNEL_* values of the header)
KERNEL_AUTO, KERNEL_DECODE, KERNEL_SMALL, KERNEL_MID, KERNEL_LARGE = 0, 1, 2, 3, 4


class DuqppError(RuntimeError):
    def __init__(self, status, what):
        super().__init__(f"{what}: {status_string(status)} ({status})")
        self.status = status


def library_path():
    return os.path.join(_HERE, _LIB_NAME)


def _load():
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'); "
            "there is no fallback path")
    L = ctypes.CDLL(path)
    vp, i64, u8p, fp, sz, ci = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                ctypes.c_size_t, ctypes.c_int)
    L.duqpp_quantize_weights.argtypes = [vp, i64, i64, i64, fp, i64, u8p, u8p, vp]
    L.duqpp_rotate_quantize.argtypes = [vp, i64, i64, i64, fp, i64, u8p, u8p, fp, vp]
    L.duqpp_mxfp4_gemm.argtypes = [u8p, u8p, u8p, u8p, i64, i64, i64, vp, ci, i64, vp, sz, vp]
    L.duqpp_rotq_gemm.argtypes = [vp, i64, fp, i64, u8p, u8p, i64, i64, i64, vp, ci, i64, vp, sz, vp]
    L.duqpp_quantize_f32_dbg.argtypes = [fp, i64, i64, i64, u8p, u8p, vp]
    L.duqpp_group_error.argtypes = [vp, i64, i64, i64, fp, i64, fp, vp, vp]
    L.duqpp_gemm_workspace_bytes.argtypes = [i64, i64, i64, ci]
    L.duqpp_gemm_workspace_bytes.restype = sz
    L.duqpp_validate_rotate_quantize.argtypes = [vp, i64, i64, i64, fp, i64, u8p, u8p]
    L.duqpp_validate_mxfp4_gemm.argtypes = [u8p, u8p, u8p, u8p, i64, i64, i64, vp, ci, i64, vp, sz, ci]
    szp = ctypes.POINTER(ctypes.c_size_t)
    L.duqpp_tiled_bytes.argtypes = [i64, i64, szp, szp]
    L.duqpp_tile_operand.argtypes = [u8p, u8p, i64, i64, u8p, u8p, vp]
    L.duqpp_untile_operand.argtypes = [u8p, u8p, i64, i64, u8p, u8p, vp]
    L.duqpp_quantize_weights_tiled.argtypes = [vp, i64, i64, i64, fp, i64, u8p, u8p, vp]
    L.duqpp_rotate_quantize_tiled.argtypes = [vp, i64, i64, i64, fp, i64, u8p, u8p, vp]
    L.duqpp_mxfp4_gemm_tiled.argtypes = [u8p, u8p, u8p, u8p, i64, i64, i64, vp, ci, i64, vp]
    L.duqpp_mxfp4_gemm_tiled_on.argtypes = [ci, u8p, u8p, u8p, u8p, i64, i64, i64, vp, ci, i64, vp]
    L.duqpp_mxfp4_gemm_tiled_on.restype = ci
    L.duqpp_gemm_kernel_for.argtypes = [i64, i64, i64, ci]
    L.duqpp_gemm_kernel_for.restype = ci
    L.duqpp_rotq_gemm_tiled.argtypes = [vp, i64, fp, i64, u8p, u8p, i64, i64, i64, vp, ci, i64, vp, sz, vp]
    L.duqpp_fold_smoothing.argtypes = [fp, i64, fp, i64, fp, fp, vp]
    L.duqpp_construct_rotation_workspace_bytes.argtypes = [i64, ci]
    L.duqpp_construct_rotation_workspace_bytes.restype = sz
    L.duqpp_construct_rotation.argtypes = [vp, i64, i64, i64, vp, ci, fp, vp, vp, vp, sz, vp]
    L.duqpp_construct_rotation.restype = ci
    L.duqpp_init.argtypes = []
    L.duqpp_init.restype = ci
    L.duqpp_packed_rotation_bytes.argtypes = [i64]
    L.duqpp_packed_rotation_bytes.restype = sz
    L.duqpp_pack_rotation.argtypes = [fp, i64, vp, vp]
    L.duqpp_pack_rotation.restype = ci
    L.duqpp_rotate_quantize_tiled_packed.argtypes = [vp, i64, i64, i64, vp, i64, u8p, u8p, vp]
    L.duqpp_rotate_quantize_tiled_packed.restype = ci
    L.duqpp_rotq_gemm_tiled_packed.argtypes = [vp, i64, vp, i64, u8p, u8p, i64, i64, i64, vp, ci, i64, vp, sz, vp]
    L.duqpp_rotq_gemm_tiled_packed.restype = ci
    L.duqpp_rotq_gemm_fused_decode.argtypes = [vp, i64, vp, i64, u8p, u8p, i64, i64, i64, vp, ci, i64, u8p, u8p, vp]
    L.duqpp_rotq_gemm_fused_decode.restype = ci
    L.duqpp_noalloc_scratch_bytes.argtypes = []
    L.duqpp_noalloc_scratch_bytes.restype = sz
    L.duqpp_rotq_gemm_tiled_noalloc.argtypes = [vp, i64, fp, i64, u8p, u8p, i64, i64, i64, vp, ci, i64, vp]
    L.duqpp_rotq_gemm_tiled_noalloc.restype = ci
    for name in ("duqpp_tiled_bytes", "duqpp_tile_operand", "duqpp_untile_operand", "duqpp_quantize_weights_tiled",
                 "duqpp_rotate_quantize_tiled", "duqpp_mxfp4_gemm_tiled", "duqpp_rotq_gemm_tiled",
                 "duqpp_fold_smoothing"):
        getattr(L, name).restype = ci
    for name in ("duqpp_quantize_weights", "duqpp_rotate_quantize", "duqpp_mxfp4_gemm", "duqpp_rotq_gemm",
                 "duqpp_quantize_f32_dbg", "duqpp_validate_rotate_quantize", "duqpp_validate_mxfp4_gemm"):
        getattr(L, name).restype = ci
    L.duqpp_status_string.argtypes = [ci]
    L.duqpp_status_string.restype = ctypes.c_char_p
    L.duqpp_version.restype = ctypes.c_char_p
    return L


lib = _load()


def status_string(status):
    return lib.duqpp_status_string(int(status)).decode()


def version():
    return lib.duqpp_version().decode()


def _check(status, what):
    if status != 0:
        raise DuqppError(status, what)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype):
        raise TypeError(f"{what} must be a cuda tensor of {dtype}")
    return t


def _n_rblocks(R):
    if R.dim() != 3 or tuple(R.shape[1:]) != (32, 32) or not R.is_contiguous():
        raise ValueError("R must be a contiguous [n_rblocks, 32, 32] fp32 tensor")
    return R.shape[0]


def gemm_workspace_bytes(T, N, K, fused=False):
    return int(lib.duqpp_gemm_workspace_bytes(T, N, K, int(bool(fused))))


def _workspace(nbytes, device):
    if nbytes == 0:
        return None, 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)   # torch device allocations are >= 256-byte aligned
    return ws, nbytes


def _rows_op(fn_name, x, R, want_rot, out=None):
    _dev(x, torch.bfloat16, "x")
    _dev(R, torch.float32, "R")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [rows, K] with unit stride along K")
    rows, K = x.shape
    if out is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
        scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device)
    else:
        codes, scales = out
        _dev(codes, torch.uint8, "codes")
        _dev(scales, torch.uint8, "scales")
        if (tuple(codes.shape) != (rows, K // 2) or tuple(scales.shape) != (rows, K // 32)
                or not codes.is_contiguous() or not scales.is_contiguous()):
            raise ValueError("bad output tensors")
    nb = _n_rblocks(R)
    if fn_name == "duqpp_rotate_quantize":
        yrot = torch.empty((rows, K), dtype=torch.float32, device=x.device) if want_rot else None
        st = lib.duqpp_rotate_quantize(x.data_ptr(), rows, K, x.stride(0), R.data_ptr(), nb, codes.data_ptr(),
                                       scales.data_ptr(), yrot.data_ptr() if want_rot else None, _stream())
        _check(st, fn_name)
        return (codes, scales, yrot) if want_rot else (codes, scales)
    st = lib.duqpp_quantize_weights(x.data_ptr(), rows, K, x.stride(0), R.data_ptr(), nb, codes.data_ptr(),
                                    scales.data_ptr(), _stream())
    _check(st, fn_name)
    return codes, scales


def rotate_quantize(x, R, return_rotated=False, out=None):
    """x bf16 [T, K], R fp32 [K/32 or 1, 32, 32] -> (codes u8 [T, K/2], scales u8 [T, K/32][, y_rot fp32 [T, K]]).
    `out=(codes, scales)` reuses caller tensors."""
    return _rows_op("duqpp_rotate_quantize", x, R, return_rotated, out)


def quantize_weights(w, R, out=None):
    """w bf16 [N, K] -> (codes u8 [N, K/2], scales u8 [N, K/32]) of R^T W."""
    return _rows_op("duqpp_quantize_weights", w, R, False, out)


def _out(T, N, out_dtype, device, out):
    tdt = torch.float32 if out_dtype == F32 else torch.bfloat16
    if out is None:
        out = torch.empty((T, N), dtype=tdt, device=device)
    elif out.dtype != tdt or tuple(out.shape) != (T, N) or out.stride(1) != 1:
        raise ValueError("bad output tensor")
    return out


def mxfp4_gemm(a_codes, a_scales, b_codes, b_scales, out_dtype=F32, out=None, workspace=None):
    """Row-major operands -> Y [T, N].  workspace: None = allocate the scratch of the fast path, False = none
    (direct kernel), or a uint8 tensor of at least gemm_workspace_bytes(T, N, K)."""
    for t, n in ((a_codes, "a_codes"), (a_scales, "a_scales"), (b_codes, "b_codes"), (b_scales, "b_scales")):
        _dev(t, torch.uint8, n)
        if not t.is_contiguous():
            raise ValueError(f"{n} must be contiguous")
    T, K = a_codes.shape[0], a_codes.shape[1] * 2
    N = b_codes.shape[0]
    if b_codes.shape[1] * 2 != K or tuple(a_scales.shape) != (T, K // 32) or tuple(b_scales.shape) != (N, K // 32):
        raise ValueError("operand shapes disagree")
    y = _out(T, N, out_dtype, a_codes.device, out)
    if workspace is None:
        workspace, nbytes = _workspace(gemm_workspace_bytes(T, N, K, False), a_codes.device)
    elif workspace is False:                                # no scratch: the direct row-major kernel
        workspace, nbytes = None, 0
    else:
        nbytes = workspace.numel()
    st = lib.duqpp_mxfp4_gemm(a_codes.data_ptr(), a_scales.data_ptr(), b_codes.data_ptr(), b_scales.data_ptr(),
                              T, N, K, y.data_ptr(), out_dtype, y.stride(0),
                              workspace.data_ptr() if workspace is not None else None, nbytes, _stream())
    _check(st, "duqpp_mxfp4_gemm")
    return y


def rotq_gemm(x, R, b_codes, b_scales, out_dtype=F32, out=None, workspace=None):
    _dev(x, torch.bfloat16, "x")
    _dev(R, torch.float32, "R")
    _dev(b_codes, torch.uint8, "b_codes")
    _dev(b_scales, torch.uint8, "b_scales")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [T, K] with unit stride along K")
    T, K = x.shape
    N = b_codes.shape[0]
    if b_codes.shape[1] * 2 != K or tuple(b_scales.shape) != (N, K // 32):
        raise ValueError("operand shapes disagree")
    y = _out(T, N, out_dtype, x.device, out)
    if workspace is None:
        workspace, nbytes = _workspace(gemm_workspace_bytes(T, N, K, True), x.device)
    else:
        nbytes = workspace.numel()
    st = lib.duqpp_rotq_gemm(x.data_ptr(), x.stride(0), R.data_ptr(), _n_rblocks(R), b_codes.data_ptr(),
                             b_scales.data_ptr(), T, N, K, y.data_ptr(), out_dtype, y.stride(0),
                             workspace.data_ptr() if workspace is not None else None, nbytes, _stream())
    _check(st, "duqpp_rotq_gemm")
    return y


def quantize_f32_dbg(y):
    """Test only: the device quantiser stage on fp32 [rows, K]."""
    _dev(y, torch.float32, "y")
    rows, K = y.shape
    codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=y.device)
    scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=y.device)
    st = lib.duqpp_quantize_f32_dbg(y.data_ptr(), rows, K, y.stride(0), codes.data_ptr(), scales.data_ptr(), _stream())
    _check(st, "duqpp_quantize_f32_dbg")
    return codes, scales


def group_error(x, R=None, return_mean=True):
    """x bf16 [T, K], R fp32 [K/32 or 1, 32, 32] or None (no rotation) -> (err fp32 [T, K/32], mean): the per-group
    normalised quantisation error of Sec. 4.1 (Fig. 1), -1 where a group is all zero, and its mean over the other
    groups (a Python float; None with return_mean=False)."""
    _dev(x, torch.bfloat16, "x")
    T, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must have unit stride along K")
    nrb = 1
    if R is not None:
        _dev(R, torch.float32, "R")
        if not R.is_contiguous() or R.dim() != 3 or tuple(R.shape[1:]) != (32, 32):
            raise ValueError("R must be a contiguous [n, 32, 32] tensor")
        nrb = R.shape[0]
    err = torch.empty((T, K // 32), dtype=torch.float32, device=x.device)
    mean = torch.empty(1, dtype=torch.float64, device=x.device) if return_mean else None
    st = lib.duqpp_group_error(x.data_ptr(), T, K, x.stride(0), R.data_ptr() if R is not None else None, nrb,
                               err.data_ptr(), mean.data_ptr() if mean is not None else None, _stream())
    _check(st, "duqpp_group_error")
    return err, (float(mean.item()) if mean is not None else None)


# ---------------------------------------------------------------- tiled operand layout
def tiled_bytes(rows, K):
    """(codes bytes, scales bytes) of the tiled form of a [rows, K] operand."""
    cb, sb = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib.duqpp_tiled_bytes(rows, K, ctypes.byref(cb), ctypes.byref(sb)), "duqpp_tiled_bytes")
    return int(cb.value), int(sb.value)


def _tiled_buffers(rows, K, device, out=None):
    cb, sb = tiled_bytes(rows, K)
    if out is None:
        return (torch.empty(cb, dtype=torch.uint8, device=device), torch.empty(sb, dtype=torch.uint8, device=device))
    c, s = out
    _dev(c, torch.uint8, "codes_t")
    _dev(s, torch.uint8, "scales_t")
    if c.numel() != cb or s.numel() != sb or not c.is_contiguous() or not s.is_contiguous():
        raise ValueError("bad tiled output tensors")
    return c, s


def tile_operand(codes, scales):
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.uint8, "scales")
    rows, K = codes.shape[0], codes.shape[1] * 2
    ct, st_ = _tiled_buffers(rows, K, codes.device)
    _check(lib.duqpp_tile_operand(codes.data_ptr(), scales.data_ptr(), rows, K, ct.data_ptr(), st_.data_ptr(), _stream()),
           "duqpp_tile_operand")
    return ct, st_


def untile_operand(codes_t, scales_t, rows, K):
    _dev(codes_t, torch.uint8, "codes_t")
    _dev(scales_t, torch.uint8, "scales_t")
    codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=codes_t.device)
    scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=codes_t.device)
    _check(lib.duqpp_untile_operand(codes_t.data_ptr(), scales_t.data_ptr(), rows, K, codes.data_ptr(), scales.data_ptr(),
                                    _stream()), "duqpp_untile_operand")
    return codes, scales


def _rows_op_tiled(fn, name, x, R, out):
    _dev(x, torch.bfloat16, "x")
    _dev(R, torch.float32, "R")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [rows, K] with unit stride along K")
    rows, K = x.shape
    ct, st_ = _tiled_buffers(rows, K, x.device, out)
    _check(fn(x.data_ptr(), rows, K, x.stride(0), R.data_ptr(), _n_rblocks(R), ct.data_ptr(), st_.data_ptr(), _stream()), name)
    return ct, st_


def rotate_quantize_tiled(x, R, out=None):
    """x bf16 [T, K] -> (codes_t, scales_t): flat uint8 tensors in the tiled operand layout."""
    return _rows_op_tiled(lib.duqpp_rotate_quantize_tiled, "duqpp_rotate_quantize_tiled", x, R, out)


def quantize_weights_tiled(w, R, out=None):
    return _rows_op_tiled(lib.duqpp_quantize_weights_tiled, "duqpp_quantize_weights_tiled", w, R, out)


PACKED_BLOCK_BYTES = 6144


def pack_rotation(R):
    """R fp32 [n, 32, 32] -> flat uint8 tensor of n * 6144 bytes: the blocks as the tiled-output kernel reads them."""
    _dev(R, torch.float32, "R")
    n = _n_rblocks(R)
    nbytes = int(lib.duqpp_packed_rotation_bytes(n))
    assert nbytes == n * PACKED_BLOCK_BYTES
    out = torch.empty(nbytes, dtype=torch.uint8, device=R.device)
    _check(lib.duqpp_pack_rotation(R.data_ptr(), n, out.data_ptr(), _stream()), "duqpp_pack_rotation")
    return out


def _n_packed(Rp):
    _dev(Rp, torch.uint8, "R_packed")
    if Rp.dim() != 1 or not Rp.is_contiguous() or Rp.numel() == 0 or Rp.numel() % PACKED_BLOCK_BYTES:
        raise ValueError("R_packed must be the flat tensor pack_rotation returns")
    return Rp.numel() // PACKED_BLOCK_BYTES


def rotate_quantize_tiled_packed(x, R_packed, out=None):
    """rotate_quantize_tiled on packed rotation blocks: same bytes out."""
    _dev(x, torch.bfloat16, "x")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [rows, K] with unit stride along K")
    rows, K = x.shape
    ct, st_ = _tiled_buffers(rows, K, x.device, out)
    _check(lib.duqpp_rotate_quantize_tiled_packed(x.data_ptr(), rows, K, x.stride(0), R_packed.data_ptr(), _n_packed(R_packed),
                                                  ct.data_ptr(), st_.data_ptr(), _stream()), "duqpp_rotate_quantize_tiled_packed")
    return ct, st_


def rotq_gemm_tiled_packed(x, R_packed, b_codes_t, b_scales_t, N, out_dtype=F32, out=None, workspace=None):
    _dev(x, torch.bfloat16, "x")
    _dev(b_codes_t, torch.uint8, "b_codes_t")
    _dev(b_scales_t, torch.uint8, "b_scales_t")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [T, K] with unit stride along K")
    T, K = x.shape
    if (b_codes_t.numel(), b_scales_t.numel()) != tiled_bytes(N, K):
        raise ValueError("weight operand sizes disagree with N, K")
    y = _out(T, N, out_dtype, x.device, out)
    cb, sb = tiled_bytes(T, K)
    if workspace is None:
        workspace = torch.empty(((cb + 255) // 256 + (sb + 255) // 256) * 256, dtype=torch.uint8, device=x.device)
    _check(lib.duqpp_rotq_gemm_tiled_packed(x.data_ptr(), x.stride(0), R_packed.data_ptr(), _n_packed(R_packed),
                                            b_codes_t.data_ptr(), b_scales_t.data_ptr(), T, N, K, y.data_ptr(), out_dtype,
                                            y.stride(0), workspace.data_ptr(), workspace.numel(), _stream()),
           "duqpp_rotq_gemm_tiled_packed")
    return y


def rotq_gemm_fused_decode(x, R_packed, b_codes_t, b_scales_t, N, out_dtype=F32, out=None, return_operand=False):
    """The one-kernel form (T <= 32).  return_operand: also the activation codes / scales (tiled) it was formed from."""
    _dev(x, torch.bfloat16, "x")
    _dev(b_codes_t, torch.uint8, "b_codes_t")
    _dev(b_scales_t, torch.uint8, "b_scales_t")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [T, K] with unit stride along K")
    T, K = x.shape
    if (b_codes_t.numel(), b_scales_t.numel()) != tiled_bytes(N, K):
        raise ValueError("weight operand sizes disagree with N, K")
    y = _out(T, N, out_dtype, x.device, out)
    ct, st_ = _tiled_buffers(T, K, x.device) if return_operand else (None, None)
    _check(lib.duqpp_rotq_gemm_fused_decode(x.data_ptr(), x.stride(0), R_packed.data_ptr(), _n_packed(R_packed),
                                            b_codes_t.data_ptr(), b_scales_t.data_ptr(), T, N, K, y.data_ptr(), out_dtype,
                                            y.stride(0), ct.data_ptr() if return_operand else None,
                                            st_.data_ptr() if return_operand else None, _stream()),
           "duqpp_rotq_gemm_fused_decode")
    return (y, ct, st_) if return_operand else y


def gemm_kernel_for(T, N, K, out_dtype=F32):
    k = lib.duqpp_gemm_kernel_for(T, N, K, out_dtype)
    if k < 0:
        _check(k, "duqpp_gemm_kernel_for")
    return k


def mxfp4_gemm_tiled(a_codes_t, a_scales_t, b_codes_t, b_scales_t, T, N, K, out_dtype=F32, out=None, kernel=KERNEL_AUTO):
    for t, n in ((a_codes_t, "a_codes_t"), (a_scales_t, "a_scales_t"), (b_codes_t, "b_codes_t"), (b_scales_t, "b_scales_t")):
        _dev(t, torch.uint8, n)
    if (a_codes_t.numel(), a_scales_t.numel()) != tiled_bytes(T, K) or (b_codes_t.numel(), b_scales_t.numel()) != tiled_bytes(N, K):
        raise ValueError("operand sizes disagree with T, N, K")
    y = _out(T, N, out_dtype, a_codes_t.device, out)
    if kernel != KERNEL_AUTO:
        _check(lib.duqpp_mxfp4_gemm_tiled_on(kernel, a_codes_t.data_ptr(), a_scales_t.data_ptr(), b_codes_t.data_ptr(),
                                             b_scales_t.data_ptr(), T, N, K, y.data_ptr(), out_dtype, y.stride(0), _stream()),
               "duqpp_mxfp4_gemm_tiled_on")
        return y
    _check(lib.duqpp_mxfp4_gemm_tiled(a_codes_t.data_ptr(), a_scales_t.data_ptr(), b_codes_t.data_ptr(), b_scales_t.data_ptr(),
                                      T, N, K, y.data_ptr(), out_dtype, y.stride(0), _stream()), "duqpp_mxfp4_gemm_tiled")
    return y


def rotq_gemm_tiled(x, R, b_codes_t, b_scales_t, N, out_dtype=F32, out=None, workspace=None):
    _dev(x, torch.bfloat16, "x")
    _dev(R, torch.float32, "R")
    _dev(b_codes_t, torch.uint8, "b_codes_t")
    _dev(b_scales_t, torch.uint8, "b_scales_t")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [T, K] with unit stride along K")
    T, K = x.shape
    if (b_codes_t.numel(), b_scales_t.numel()) != tiled_bytes(N, K):
        raise ValueError("weight operand sizes disagree with N, K")
    y = _out(T, N, out_dtype, x.device, out)
    cb, sb = tiled_bytes(T, K)
    need = ((cb + 255) // 256 + (sb + 255) // 256) * 256
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _check(lib.duqpp_rotq_gemm_tiled(x.data_ptr(), x.stride(0), R.data_ptr(), _n_rblocks(R), b_codes_t.data_ptr(),
                                     b_scales_t.data_ptr(), T, N, K, y.data_ptr(), out_dtype, y.stride(0),
                                     workspace.data_ptr(), workspace.numel(), _stream()), "duqpp_rotq_gemm_tiled")
    return y


def noalloc_scratch_bytes():
    return int(lib.duqpp_noalloc_scratch_bytes())


def rotq_gemm_tiled_noalloc(x, R, b_codes_t, b_scales_t, N, out_dtype=F32, out=None):
    """duqpp_rotq_gemm_tiled_noalloc: the fused call on the library's fixed scratch.  Pass `out` to keep this wrapper
    from allocating the result."""
    _dev(x, torch.bfloat16, "x")
    _dev(R, torch.float32, "R")
    _dev(b_codes_t, torch.uint8, "b_codes_t")
    _dev(b_scales_t, torch.uint8, "b_scales_t")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [T, K] with unit stride along K")
    T, K = x.shape
    if (b_codes_t.numel(), b_scales_t.numel()) != tiled_bytes(N, K):
        raise ValueError("weight operand sizes disagree with N, K")
    y = _out(T, N, out_dtype, x.device, out)
    _check(lib.duqpp_rotq_gemm_tiled_noalloc(x.data_ptr(), x.stride(0), R.data_ptr(), _n_rblocks(R), b_codes_t.data_ptr(),
                                             b_scales_t.data_ptr(), T, N, K, y.data_ptr(), out_dtype, y.stride(0),
                                             _stream()), "duqpp_rotq_gemm_tiled_noalloc")
    return y


def fold_smoothing(R, lam):
    """R fp32 [K/32 or 1, 32, 32], lam fp32 [K] (the diagonal of the smoothing step) -> (R_act, R_wgt), fp32
    [K/32, 32, 32] each: rotate_quantize(x, R_act) and quantize_weights(w, R_wgt) then yield the smoothed operands."""
    _dev(R, torch.float32, "R")
    _dev(lam, torch.float32, "lam")
    if lam.dim() != 1 or not lam.is_contiguous():
        raise ValueError("lam must be a contiguous vector of K entries")
    K = lam.shape[0]
    R_act = torch.empty((K // 32, 32, 32), dtype=torch.float32, device=R.device)
    R_wgt = torch.empty_like(R_act)
    _check(lib.duqpp_fold_smoothing(R.data_ptr(), _n_rblocks(R), lam.data_ptr(), K, R_act.data_ptr(),
                                    R_wgt.data_ptr(), _stream()), "duqpp_fold_smoothing")
    return R_act, R_wgt


def construct_rotation(x, q_steps, return_peaks=False, workspace=None):
    """Greedy construction of the shared rotation block from calibration activations x [T, K] bf16 and the steps'
    orthogonal draws q_steps [steps, 31, 31] fp64.  Returns (R [1, 32, 32] fp32, block index, steps kept[, peaks])."""
    _dev(x, torch.bfloat16, "x")
    _dev(q_steps, torch.float64, "q_steps")
    if q_steps.dim() != 3 or tuple(q_steps.shape[1:]) != (31, 31) or not q_steps.is_contiguous():
        raise ValueError("q_steps must be contiguous [steps, 31, 31]")
    T, K = x.shape
    steps = q_steps.shape[0]
    nbytes = lib.duqpp_construct_rotation_workspace_bytes(T, steps)
    if nbytes == 0:
        raise ValueError("bad T or number of steps")
    ws = workspace if workspace is not None else _workspace(nbytes, x.device)[0]
    R = torch.empty((1, 32, 32), dtype=torch.float32, device=x.device)
    info = torch.empty(2, dtype=torch.int32, device=x.device)
    peaks = torch.empty(steps + 1, dtype=torch.float64, device=x.device) if return_peaks else None
    _check(lib.duqpp_construct_rotation(x.data_ptr(), T, K, x.stride(0), q_steps.data_ptr(), steps, R.data_ptr(),
                                        info.data_ptr(), peaks.data_ptr() if return_peaks else None, ws.data_ptr(),
                                        ws.numel(), _stream()), "duqpp_construct_rotation")
    block, kept = (int(v) for v in info.cpu())
    return (R, block, kept, peaks) if return_peaks else (R, block, kept)


def init():
    """Per-device set-up for the current device (optional; every call does what it needs by itself)."""
    _check(lib.duqpp_init(), "duqpp_init")
