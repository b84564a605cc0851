"""MI355X-native tree verification for speculative decoding: thin binding over libhb.so.

Every step runs in the HIP kernels of the C-ABI library; this package only marshals torch
tensors (device memory, streams) into its arguments.  Importing it needs the built library:
``python -m paper_2509_18824_amd.build`` (or ``__graft_entry__.build()``).
"""
from .binding import (
    HbError,
    AttnDesc,
    lib,
    hb_last_error,
    hb_version,
    hb_tree_validate_host,
    hb_tree_verify_attn,
    hb_tree_verify_attn_workspace_bytes,
    hb_tree_verify_attn_num_splits,
    hb_lmhead_argmax,
    hb_lmhead_argmax_workspace_bytes,
    hb_lmhead_argmax_noalloc,
    hb_lmhead_argmax_noalloc_max_rows,
    hb_tree_positions,
    hb_rope_table,
    hb_qkv_rope_project,
    hb_out_project,
    hb_proj_workspace_bytes,
    hb_qkv_rope_project_ws,
    hb_out_project_ws,
    hb_tree_accept,
    hb_tree_accept_sample,
    hb_tree_accept_sample_workspace_bytes,
    hb_kv_compact,
    hb_kv_compact_layers,
    hb_topk_logprob,
    hb_topk_logprob_workspace_bytes,
    hb_draft_tree_candidates,
    hb_tree_grow,
    hb_tree_finalize,
    hb_rmsnorm,
    hb_swiglu_project,
    hb_meta_query_fold_bytes,
    hb_meta_query_fold,
    hb_meta_query_attn_workspace_bytes,
    hb_meta_query_attn,
    HB_F32,
    HB_BF16,
    HB_ATTN_AUTO,
    HB_ATTN_SCALAR,
    HB_ATTN_MFMA,
)

__all__ = [n for n in dir() if n.startswith(("hb_", "HB_", "Hb")) or n in ("AttnDesc", "lib")]
