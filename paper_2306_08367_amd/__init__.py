"""lq on MI355X: fused star-join + model prediction and linear-algebra group-by.

All computation happens in the HIP library ``liblq.so`` (built in-tree by
``paper_2306_08367_amd.build``); this package only marshals torch tensors
into its C interface.  There is no fallback: without the library, importing
``binding`` raises.
"""
from .binding import (  # noqa: F401
    LQ_CHECK_FKS, LQ_REUSE_SIDE_TABLES, LQ_FORCE_GENERIC, LQ_FORCE_TILE, LQError, lib_path, lq_fused_join_predict,
    lq_groupby_workspace_bytes, lq_groupby_bucket_workspace_bytes, lq_last_error, lq_masked_groupby_sum,
    lq_materialized_join_predict, lq_project_dims, lq_stream_copy, lq_version,
    lq_workspace_bytes, lq_tree_table_ld, lq_tree_project_dims, lq_fused_join_tree,
    lq_materialized_join_tree, lq_tree_mask_words, lq_tree_compress_tables, lq_tree_project_dim_rows, lq_tree_fact_mask_bytes, lq_tree_fact_masks, lq_fused_join_tree_masks, LQ_CHECK_KEYS, lq_keymap_bytes, lq_keymap_build, lq_keymap_insert,
    lq_keymap_lookup, lq_compact_matches, lq_project_dim_rows, lq_fusion_advice, lq_groupby_agg,
    lq_keymap64_bytes, lq_keymap64_build, lq_keymap64_insert, lq_keymap64_lookup,
    lq_masked_groupby_sum_static, lq_static_scratch_bytes, lq_group_avg, lq_yardstick_read, lq_yardstick_stream, lq_yardstick_gather, lq_yardstick_matrix,
    lq_group_domain, lq_group_domain_workspace_bytes, lq_order_groups, LQ_KEY_GROUP_COLUMN, LQ_KEY_SUM, LQ_KEY_COUNT,
)
