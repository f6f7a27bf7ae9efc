"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package holds no arithmetic of the decoding method itself: only shape tables, random
draws, the weight-blob container format and dtype conversion of the draws.
"""
from .inputs import (  # noqa: F401
    HawkShape,
    CONFIGS,
    BLOB_MAGIC,
    BLOB_HEADER_BYTES,
    blob_layout,
    blob_tensor,
    make_weights,
    make_cond,
    make_uniforms,
    make_spatial_heads,
    make_logit_rows,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
)
