"""MI355X-native HTTM global-attention layer (arXiv 2511.21317): thin Python binding over the
C-ABI library libhttm.so, whose HIP kernels (gfx950) do all the work."""
from .binding import (  # noqa: F401
    HttmError, Geom, Sizes, WorkspaceLayout, Plan, make_geom, geom_sizes, geom_tables, geom_block_forms,
    workspace_layout, reorder, match_merge, reorder_match_merge, attention, unmerge, layer_forward,
    workspace_views, alloc_workspace, lib, LIB_PATH, VARIANTS,
    reorder_match_merge_filtered, attention_outliers, unmerge_filtered, outlier_stats, global_match,
    attention_log2, attention_log2_static, attention_scratch_bytes, attention_split_plan, FLAG_LOG2_KEYS, LOG2_KEY_SCALE,
)
