"""MI355X-native tree-verification step of SpecVLM-style speculative decoding.

The product is ``libspecvlm.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/specvlm.h``); this package is its argument-marshalling Python binding.
PyTorch is used for device memory and streams only.
"""
from .binding import (  # noqa: F401
    AttnDesc,
    SpecvlmError,
    err_flag_names,
    lib,
    load_library,
    specvlm_draft_finalize,
    specvlm_draft_select,
    specvlm_draft_topk,
    specvlm_draft_topk_select,
    specvlm_head_argmax,
    specvlm_head_argmax_workspace_bytes,
    specvlm_kv_compact,
    specvlm_node_argmax,
    specvlm_node_argmax_accept,
    specvlm_tree_accept,
    specvlm_tree_accept_sample,
    specvlm_tree_verify_attn,
    specvlm_tree_verify_attn_num_splits,
    specvlm_tree_verify_attn_static,
    specvlm_tree_verify_attn_vector_alu,
    specvlm_tree_verify_attn_workspace_bytes,
    specvlm_version,
    specvlm_visual_pool,
    specvlm_visual_prune,
)
