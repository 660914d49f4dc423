"""MI355X-native embedding-access hot path of lookahead-cached recommendation-model training
(Bagpipe, arXiv 2202.12429): thin ctypes binding over libbagpipe_hip.so.

The functions carry the names of the C ABI (include/bagpipe.h) and only marshal arguments: every step of
the path runs in the HIP kernels.  torch is used for device memory and streams, nothing else.  There is no
CPU fallback: importing works without the library (so that tools can inspect the package), but any call
raises if libbagpipe_hip.so has not been built (python -m paper_2202_12429_amd.build).
"""
from .binding import (  # noqa: F401
    BF16, F32, SGD, ADAGRAD, ADAGRAD_ROWWISE,
    BagpipeError, Plan, bp_config, library_path, load_library, make_config,
    bp_oracle_plan, bp_oracle_plan_workspace_bytes, bp_oracle_plan_chunk, bp_oracle_plan_chunk_workspace_bytes, PlanState, bp_cache_apply, bp_cache_apply_duplex, bp_cache_apply_duplex_workspace_bytes, bp_cache_stage, bp_cache_apply_staged, bp_cache_apply_handoff,
    bp_pipeline_early_counts, bp_pipeline_create, bp_pipeline_destroy, bp_pipeline_early, bp_pipeline_begin,
    bp_pipeline_acquire, bp_pipeline_release, bp_pipeline_end,
    bp_embbag_fwd,
    bp_embbag_fwd_grouped,
    bp_embbag_bwd_update, bp_embbag_bwd_update_workspace_bytes,
    bp_embbag_bwd_update_grouped, bp_embbag_bwd_update_grouped_workspace_bytes,
    bp_embbag_bwd_ticket_bytes, bwd_tickets, piece_capacity,
    bp_embbag_bwd_update_grouped_static, bp_embbag_bwd_update_grouped_static_bytes,
    bp_embbag_bwd_update_grouped_static_max_bytes,
    bp_error_string, bp_last_error_message, bp_version,
    bp_copy_calibration, bp_gather_calibration, bp_scatter_calibration, bp_profile_enable, bp_profile_select, bp_profile_bracket_overhead, bp_profile_collect, bp_profile_get, profile_totals, profile_spread,
)
