"""Seeded synthetic inputs shared by the tests, the bench and the smoke run.

This package only *draws data* (activations, weights, rotation blocks) with the
shapes and outlier structure of LLaMA-3 linear layers.  It contains none of the
method's arithmetic: no rotation, no MXFP4 encoding, no GEMM.  Both the CPU
oracle and the HIP library receive these buffers as plain inputs.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    LAYER_SET_8B,
    LAYER_SET_CONFIGS,
    OutlierSpec,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    hadamard_blocks,
    identity_blocks,
    make_activations,
    make_orthogonal_steps,
    make_rotation_blocks,
    make_smoothing_scales,
    make_weights,
    stream_seed,
)
