"""MI355X-native tree verification for Jakiro-style speculative decoding.

Thin Python binding over the C-ABI library libjakiro_verify.so (hand-written
HIP kernels for gfx950).  Every step of the computation runs in those kernels;
this package only marshals arguments.  There is no CPU fallback: importing the
binding functions without the built library raises.
"""
from .binding import (  # noqa: F401
    JK_BF16, JK_F32, JK_GREEDY, JK_SAMPLE, JK_HEADS_CONTRASTIVE, JK_HEADS_DECOUPLED, JakiroError,
    draft_heads, draft_heads_workspace, prepare_draft_heads, moe_experts, moe_experts_workspace, prepare_moe_experts, linear, TreeState, tree_grow, tree_grow_tail, tree_fill_static, tree_finalize, gather_draft_probs, accept_path, accept_path_greedy_static, accept_path_rows, accept_path_workspace, commit_path, lib,
    library_path, prepare_accept_path, prepare_commit_path, prepare_commit_path_layers, prepare_commit_path_layers_paged,
    prepare_tree_verify_attention_paged, tree_verify_attention_paged, stream_read_probe, prepare_tree_verify_attention, tree_verify_attention, tree_verify_attention_workspace, tree_verify_attention_plan, validate_tree, version, workspace_init, set_tuning, last_device_error,
    JK_DEVERR_BAD_TREE, JK_DEVERR_BAD_TOKEN, JK_DEVERR_BAD_PAGE, JK_DEVERR_MERGE_WAIT, JK_DEVERR_WALK_WAIT, JK_WORKSPACE_HEADER_BYTES,
)
