"""libgnnagg for AMD MI355X: message-passing Aggregation by feature slices
(arXiv 2104.03058, Algorithm 1) as hand-written HIP kernels behind a C ABI.

This package is only the thin ctypes binding over ``libgnnagg.so``; every step
of the path runs in the library's kernels.  PyTorch supplies device memory and
streams, nothing else.  There is no CPU fallback: without the built library or
without a GPU the calls raise.
"""
from .binding import (  # noqa: F401
    BF16, F32, F_CHUNK_AUTO, MAX, MEAN, NORM_SYM, PLAN_CLASSES, SELF_LOOPS, SUM, SUM_SCALED, WSUM, GnnaggError, RowPlan,
    SourceBlocks, gnnagg_aggregate, gnnagg_aggregate_blocked, gnnagg_aggregate_blocked_workspace_bytes,
    gnnagg_aggregate_noalloc, gnnagg_aggregate_update, gnnagg_aggregate_workspace_bytes, gnnagg_auto_f_chunk,
    gnnagg_auto_source_blocks,
    gnnagg_build_csr, gnnagg_check_csr, gnnagg_combine, gnnagg_copy_probe, gnnagg_gat_attention,
    gnnagg_gat_workspace_bytes, gnnagg_gcn_factors, gnnagg_line_gather_probe, gnnagg_mfma_f64_probe, gnnagg_plan_rows, gnnagg_plan_source_blocks,
    gnnagg_rank_sources, gnnagg_row_pitch, gnnagg_scale_rows, gnnagg_set_workgroup_cap, gnnagg_strerror, gnnagg_tune_blocked, gnnagg_tune_f_chunk,
    pitched_empty, gnnagg_version, library_path, load_library,
)
