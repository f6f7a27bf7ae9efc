"""MI355X-native hot path of Hawk-style speculative decoding for autoregressive image tokens.

Thin Python binding over libhawk.so (hand-written HIP kernels behind a C ABI, see
include/hawk.h).  PyTorch is used for device memory and the stream only.
"""
from .hawk import (  # noqa: F401
    Hawk,
    HawkConfig,
    HawkError,
    HawkStats,
    lib_path,
    load_library,
    multi_verify,
    multi_verify_static,
    multi_verify_workspace_bytes,
    plan_info,
    sample_rows,
    spatial_heads,
    spec_cache_bytes,
    spec_cache_slot,
    tree_layout,
    SpecCache,
    workspace_bytes,
)
