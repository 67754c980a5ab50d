"""UniPrefill token-sparsification operator for MI355X: Python face of libuniprefill.so."""
from .binding import (  # noqa: F401
    UP_OK, UP_ERR_NULL, UP_ERR_SHAPE, UP_ERR_RANGE, UP_ERR_UNSUPPORTED, UP_ERR_ALIGN, UP_ERR_WORKSPACE,
    UP_ERR_HIP, UP_ERR_SCRATCH, STATIC_SCRATCH_BYTES, uniprefill_fused_static, UP_BF16, UP_F32, EXPORTS, LIB_PATH, UniPrefillError, up_params, make_params, lib, ptr,
    status_string, uniprefill_plan, uniprefill_score, uniprefill_select, uniprefill_compact,
    uniprefill_scatter, uniprefill_fused, uniprefill_fused_phases, uniprefill_select_top_p,
    uniprefill_compact_counted, uniprefill_fused_top_p, uniprefill_compose_index, uniprefill_slot_mapping,
    uniprefill_compact_column, uniprefill_seqused, uniprefill_score_paged, uniprefill_fused_paged, uniprefill_select_top_p_chunked,
    uniprefill_fused_top_p_chunked, uniprefill_keep_mask, uniprefill_fused_lse, uniprefill_score_lse,
    uniprefill_fused_top_p_lse, uniprefill_score_partial, uniprefill_scores_from_partials, uniprefill_plan_chunked, uniprefill_score_chunked, uniprefill_select_chunked, uniprefill_fused_chunked,
    UP_PHASE_PLAN, UP_PHASE_ROW_STATS, UP_PHASE_MERGE_STATS, UP_PHASE_SWEEP_SELECT, UP_PHASE_GATHER,
    UP_PHASE_ALL, UP_PHASE_GATHER_IN_SELECT,
)
