"""MI355X-native fused linear cross-entropy (forward + backward) behind a C ABI.

The compute lives in libflce.so (hand-written HIP for gfx950); this package is
the argument-marshalling binding with the same names as include/flce.h.
"""
from .binding import (  # noqa: F401
    FLCE_BF16, FLCE_F32, SKIP_DW, SKIP_DX, FlceError,
    flce_chunk_rows, flce_logits_budget_for_workspace, flce_cross_entropy_inplace, flce_cross_entropy_inplace_noalloc,
    CE_NOALLOC_MAX_ROWS, flce_full_logits_bytes, flce_fwd_bwd,
    flce_multihead_fwd_bwd, flce_rmsnorm_fwd_bwd, flce_fwd_bwd_opt, flce_options, flce_workspace_bytes_opt,
    FlceOptions, flce_rmsnorm_workspace_bytes,
    flce_get_logits_budget_bytes, flce_num_chunks, flce_dx_k_ranges,
    flce_set_row_compaction, flce_get_row_compaction, flce_paper_chunk_rows,
    flce_release_workspace, flce_set_logits_budget_bytes, flce_set_workspace,
    flce_workspace_bytes,
    flce_workspace_bytes_max, lib, status_string, flce_timing_enable, flce_timing_collect,
    flce_mfma_ceiling_launch,
    KERNEL_KINDS,
)

flce_status_string = status_string
