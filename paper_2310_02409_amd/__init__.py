"""Dodo hot path on MI355X: thin Python binding of the C-ABI library libdodo.so.

The functions below carry the names of the C entry points declared in
``include/dodo.h`` and only marshal arguments (pointers, sizes, the current
HIP stream); every step of the path runs in the library's HIP kernels.  PyTorch
is used for device memory and streams only.  There is no CPU fallback: if the
library has not been built, importing this package raises.
"""
from .binding import (  # noqa: F401
    BF16, F32, FORCE_LAST, GELU, HEAD_MAJOR, RELU, TANH, TOKEN_MAJOR, DodoError, LIB_PATH,
    dodo_gather_nuggets, dodo_gather_nuggets_layers, dodo_meanpool_nuggets, dodo_nugget_attention, dodo_nugget_attention_workspace_bytes, dodo_nugget_attention_workspace_bytes_grouped, dodo_nugget_count, dodo_probe_copy, dodo_probe_read,
    dodo_nugget_attention_cached, dodo_nugget_attention_indexed, dodo_nugget_attention_noalloc, dodo_nugget_attention_segments, dodo_segment_plan,
    dodo_ste_score_grad, dodo_ste_score_grad_workspace_bytes,
    dodo_score, dodo_score_layers, dodo_score_mlp, dodo_score_mlp_workspace_bytes, dodo_select_threshold, dodo_select_topk,
    dodo_select_topk_workspace_bytes, dodo_status_string, dodo_stream_append, dodo_threshold_from_sample, dodo_threshold_from_sample_workspace_bytes, dodo_version,
    cu_nuggets_from_lengths, lib,
)
