"""MI355X-native tree verification for draft-then-verify speculative decoding.

The product is libfspad.so (hand-written HIP for gfx950 behind the C ABI of
include/fspad.h); this package is its ctypes binding.
"""
from .binding import (  # noqa: F401
    EXPORTS,
    FSPAD_BF16,
    FSPAD_F32,
    FSPAD_MAX_NODES,
    FspadError,
    PreparedCall,
    fspad_attn_desc,
    fspad_draft_topk,
    fspad_feature_sampler,
    fspad_draft_layer,
    fspad_draft_layer_workspace_bytes,
    fspad_feature_sampler_workspace_bytes,
    fspad_draft_topk_workspace_bytes,
    fspad_kv_commit,
    fspad_pack_weight,
    fspad_packed_weight_bytes,
    fspad_status_string,
    fspad_tree_accept_greedy,
    fspad_tree_accept_greedy_lm_head,
    fspad_tree_accept_lm_head_workspace_bytes,
    fspad_tree_accept_sample,
    fspad_tree_accept_sample_draft,
    fspad_tree_accept_sample_draft_workspace_bytes,
    fspad_tree_accept_sample_lm_head,
    fspad_tree_accept_workspace_bytes,
    fspad_tree_attn,
    fspad_tree_attn_workspace_bytes,
    fspad_tree_build,
    fspad_tree_build_mask,
    fspad_tree_validate,
    library_path,
    make_attn_desc,
)
