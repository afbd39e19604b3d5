"""Paged single-query attention for MI355X: thin Python face of libpa.so.

The library itself (csrc/pa.hip, C ABI in include/pa.h) does all the work;
this package only marshals torch tensors into it.
"""
from .binding import (PA_BF16, PA_F16, PA_F32, PA_PARTITION_AUTO, PAError, load_library,
                      pa_copy_blocks, pa_debug_validate, pa_decode, pa_decode_multi, pa_decode_shared,
                      pa_decode_shared_planned, pa_decode_shared_workspace_bytes, pa_decode_static,
                      pa_decode_workspace_bytes, PA_STATIC_SCRATCH_BYTES,
                      pa_reshape_and_cache, pa_shared_plan, pa_stream_read, pa_swap_blocks, pa_version)

__all__ = ["PA_BF16", "PA_F16", "PA_F32", "PA_PARTITION_AUTO", "PAError", "load_library",
           "pa_copy_blocks", "pa_debug_validate", "pa_decode", "pa_decode_multi", "pa_decode_shared",
           "pa_decode_shared_planned", "pa_decode_shared_workspace_bytes", "pa_decode_static",
           "pa_decode_workspace_bytes", "PA_STATIC_SCRATCH_BYTES",
           "pa_reshape_and_cache", "pa_shared_plan", "pa_stream_read", "pa_swap_blocks", "pa_version"]
