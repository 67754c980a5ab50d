"""fp64 CPU oracle (test infrastructure only; never imported by the product path)."""
from .uniprefill_oracle import *  # noqa: F401,F403
from .uniprefill_oracle import (  # noqa: F401
    SCORE_FLOOR, importance_scores, quantise_scores, phi, packed_keys, forced_mask, kept_count,
    block_kept_counts, plan, select_tokens, compact, scatter, sparsify, block_mass, select_blocks_top_p,
    block_mass_f32, top_p_block_keys, top_p_kept_blocks, chunked_running_sum, TOP_P_CHUNK, select_tokens_top_p, compose_index,
    retained_lengths, keep_mask, kv_slot_mapping, seqused, seqused_per_layer, importance_scores_with_context, importance_scores_from_lse, importance_sums,
    scores_from_partial_sums, sinks_in_chunk, gather_paged_keys,
    select_tokens_with_context, sparsify_with_context, select_tokens_top_p_with_context,
)
