"""DuQuant++ online hot path for AMD MI355X: thin Python binding over libduqpp's C ABI.

Every step (block rotation, MXFP4 quantisation, W4A4 GEMM) runs in the library's HIP
kernels; this module only marshals torch device tensors into raw pointers and sizes.
There is no CPU or PyTorch fallback: importing without the built library raises.
"""
from .binding import (  # noqa: F401
    BF16,
    F32,
    KERNEL_AUTO,
    KERNEL_DECODE,
    KERNEL_LARGE,
    KERNEL_MID,
    KERNEL_SMALL,
    gemm_kernel_for,
    DuqppError,
    construct_rotation,
    fold_smoothing,
    gemm_workspace_bytes,
    lib,
    library_path,
    mxfp4_gemm,
    mxfp4_gemm_tiled,
    init,
    pack_rotation,
    rotate_quantize_tiled_packed,
    rotq_gemm_tiled_packed,
    rotq_gemm_fused_decode,
    noalloc_scratch_bytes,
    rotq_gemm_tiled_noalloc,
    quantize_weights_tiled,
    rotate_quantize_tiled,
    rotq_gemm_tiled,
    tile_operand,
    tiled_bytes,
    untile_operand,
    quantize_f32_dbg,
    group_error,
    quantize_weights,
    rotate_quantize,
    rotq_gemm,
    status_string,
    version,
)
