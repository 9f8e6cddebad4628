"""MI355X (gfx950) verifier core for sampled register allocations: thin Python
binding over the C-ABI library built from csrc/ (see include/vl.h)."""
from .binding import (  # noqa: F401
    VlError, RESULT_DTYPE, SUMMARY_DTYPE, LOOP_DTYPE, COUNTS_DTYPE, vl_count_violations_multi, vl_bank_conflicts, load, vl_mir_create, vl_mir_create_lanes, vl_mir_lanes_get, vl_lanes_expand, vl_mir_destroy, vl_liveness, vl_liveness_multi,
    vl_live_destroy, vl_live_get, vl_verify_batch, vl_verify_batch_static, vl_verify_multi, vl_verify_multi_occ_major, vl_summarize_multi, vl_free_bases_multi, make_mask_queries, vl_strerror, vl_last_hip_error, make_jobs, hip_runtime,
    VL_DENSE_POINTS, pad_ld, rows_to_device, view_to_numpy,
)
