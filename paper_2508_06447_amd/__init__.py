"""MI355X-native pruned prefill layer of SlimInfer: HIP kernels behind a C ABI (libslim.so) and a
thin ctypes binding with the same entry-point names."""
from .binding import (  # noqa: F401
    BF16, F32, FORCE_FIRST, FORCE_LAST, POOL_AVG, POOL_MAX, PRUNE_BEFORE_ATTENTION,
    PRUNE_AFTER_ATTENTION, LIB_PATH, PROBE_LIB_PATH, EXPORTS, PROBE_EXPORTS, load_probe_library, LayerShape, LayerWeights, SlimError, kept_tokens,
    load_library, make_shape, make_weights, n_blocks, pruned_layer_workspace_bytes, slim_compact_tokens,
    slim_linear, slim_linear_bias, slim_prefill_attn, slim_pruned_layer, slim_rmsnorm, slim_rope, slim_score_blocks,
    slim_score_blocks_static,
    slim_score_blocks_pooled, slim_unit_keys, slim_score_blocks_from_unit_keys, slim_kv_swap, slim_decode_attn, slim_gemv, slim_decode_layer,
    slim_rope_table, slim_window_query, slim_window_query_from_rows, slim_linear_rope, slim_score_blocks_from_token_scores,
    slim_linear_pair, slim_row_rstd, slim_rmsnorm_linear, slim_rmsnorm_swiglu_linear, slim_fold_gain,
    slim_select_topk_blocks, slim_swiglu_linear, slim_prefill_model, schedule_keep_counts, probe_mfma, probe_copy,
)
