"""DFSAttn attention path for MI355X: thin Python binding over libdfsattn.so.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/dfsattn.h; this package only marshals arguments (torch tensors are used as
device memory, the current torch stream as the HIP stream).  There is no fallback:
importing the binding without the built library raises.
"""
from .binding import (  # noqa: F401
    DFS_BF16, DFS_F32, DFS_SELECT_MASS_HEAD, DFS_SELECT_MASS_ROW, DFS_SELECT_TOPK, DfsError, Geom, MaskState, Sizes,
    dfs_block_score, dfs_forward, dfs_geom_sizes, dfs_hilbert_perm, dfs_keep_count, dfs_last_error,
    DFS_WS_BLOCK_SCORE, DFS_WS_FORWARD, DFS_WS_FORWARD_BF16, DFS_WS_HILBERT_PERM, DFS_WS_SELECT_MASK, EXPORTS,
    DFS_ORDER_BLOCK3D, DFS_ORDER_HILBERT2D, DFS_ORDER_HILBERT3D, DFS_ORDER_RASTER, dfs_recall, dfs_schedule, dfs_token_order, dfs_block_score_src, dfs_sparse_attn_fwd_src,
    dfs_permute, dfs_select_mask, dfs_sparse_attn_fwd, dfs_unperm, dfs_workspace_bytes, lib_path, dfs_attn_clock_probe, dfs_block_score_fused, dfs_probe_mfma, dfs_probe_copy, dfs_probe_read, dfs_select_mask_static,
)
