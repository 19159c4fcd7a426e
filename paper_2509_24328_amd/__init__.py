"""MI355X-native hot path of Speculative Verification (arxiv 2509.24328).

`binding` exposes the C ABI of include/sv.h one to one (argument marshalling
only); the names below are re-exported from it.
"""
from . import binding  # noqa: F401  (fails loudly when libsv.so is missing)
from .binding import (sv_warp_cutoffs_multi, sv_warp_compact_multi, sv_accept_ratio_warped, sv_accept_ratio_sparse, sv_uniforms, Supports, sv_warp_compact, sv_row_stats_sparse, sv_verify_sample_sparse, sv_warp_cutoffs, sv_row_stats_warped, sv_verify_sample_warped, sv_accept_ratio, sv_profile_accumulate, sv_profile_finalize, sv_quantile_edges,  # noqa: F401
                      SV_BATCH_GREEDY, SV_BF16, SV_F32, SV_PER_SEQUENCE, SvError,  # noqa: F401
                      alloc_workspace, sv_accept_estimate, sv_row_stats, sv_select_length,
                      sv_set_timing_events, sv_strerror, sv_verify_sample, sv_verify_sample_static,
                      sv_verify_sample_chained, sv_verify_sample_warped_chained, sv_estimate_select, sv_repetition_penalty, sv_repetition_penalty_multi,
                      sv_workspace_bytes)
