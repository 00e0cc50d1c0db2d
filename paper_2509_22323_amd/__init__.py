"""MI355X-native MM-DiT joint attention (dense / block-sparse) for RAPID^3-style
accelerated DiT sampling.  The compute lives in ``librapid_attn.so`` (hand-written
HIP for gfx950, C ABI declared in ``include/rapid_attn.h``); this package is the
thin binding: argument marshalling only."""
from .binding import (  # noqa: F401
    RapidAttnError,
    library,
    library_path,
    rapid_attn_block_sparse,
    rapid_attn_block_sparse_static,
    STATIC_SCRATCH_BYTES,
    rapid_attn_dense,
    rapid_attn_joint,
    rapid_attn_joint_select,
    rapid_attn_joint_select_workspace_bytes,
    rapid_attn_joint_workspace_bytes,
    rapid_attn_status_string,
    rapid_attn_version,
    rapid_attn_workspace_bytes,
    rapid_cache_reuse,
    rapid_mask_level_tau,
    rapid_mask_select,
    rapid_mask_select_joint,
    rapid_mask_select_joint_workspace_bytes,
    rapid_mask_select_workspace_bytes,
    rapid_cache_store,
    rapid_equivalent_steps,
    rapid_reward,
    STATUS,
)

__all__ = [
    "RapidAttnError", "library", "library_path", "rapid_attn_block_sparse", "rapid_attn_block_sparse_static", "STATIC_SCRATCH_BYTES", "rapid_attn_dense", "rapid_attn_joint", "rapid_attn_joint_select", "rapid_attn_joint_select_workspace_bytes", "rapid_attn_joint_workspace_bytes",
    "rapid_attn_status_string", "rapid_attn_version", "rapid_attn_workspace_bytes", "rapid_cache_reuse", "rapid_mask_level_tau", "rapid_mask_select", "rapid_mask_select_joint", "rapid_mask_select_joint_workspace_bytes", "rapid_mask_select_workspace_bytes",
    "rapid_cache_store", "rapid_equivalent_steps", "rapid_reward", "STATUS",
]
