"""MI355X-native hot path of Dynamic Communication Thresholding (DCT).

Thin argument marshalling over the C ABI of libdct (include/dct.h): every step
runs in the HIP kernels; torch only provides device memory and the stream.
"""
from .binding import (  # noqa: F401
    DCT_BF16, DCT_EXACT_K, DCT_F32, DCT_GE_TAU, DCT_SCATTER_ADD, DCT_SCATTER_ASSIGN, DctError, Threshold,
    dct_ef_select_threshold, dct_ef_threshold_compact, dct_rowtopk_bwd, dct_rowtopk_fwd, dct_rowtopk_scatter, dct_scatter, dct_select_threshold, dct_select_threshold_workspace_bytes, dct_select_threshold_workspace_bytes_for,
    dct_status_string, dct_threshold_compact, dct_threshold_compact_workspace_bytes,
    dct_threshold_compact_workspace_init, lib, new_compact_workspace, new_select_workspace, read_count,
    read_threshold, Segment, segment_table, dct_batched_workspace_bytes, new_batched_workspace,
    dct_select_threshold_batched, dct_threshold_compact_batched, dct_rowtopk_fwd_bitmask,
    dct_rowtopk_bwd_bitmask, dct_rowtopk_scatter_bitmask, dct_rowtopk_fwd_idx16, dct_rowtopk_bwd_idx16,
    dct_rowtopk_scatter_idx16, dct_set_wait_limit, dct_threshold_compact_static,
    dct_threshold_compact_static_scratch_bytes,
)
