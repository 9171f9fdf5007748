"""MI355X-native hot path of DREAM's speculative decode step (arXiv 2505.19201).

The product is the C-ABI library `libdream.so` (hand-written HIP for gfx950, declared in
include/dream.h).  This package is the thin Python binding over it: argument marshalling only.
PyTorch is used for device memory and streams, nothing else.  There is no CPU fallback: if the
library is missing or no GPU is present, calls fail loudly.
"""
from .binding import (  # noqa: F401
    BF16, F32, DreamError, AttnDesc, attn_desc, load, library_path,
    dream_init, dream_tree_verify_attn_workspace, dream_tree_verify_attn,
    dream_draft_xattn_workspace, dream_draft_xattn, dream_visual_compress_workspace,
    dream_visual_compress, dream_accept_path_workspace, dream_accept_path,
    dream_accept_path_static, dream_accept_static_init,
    dream_tree_validate_host, dream_last_error, dream_set_kv_splits, dream_set_q_tiles, dream_set_tile_waves, dream_attn_plan_describe, dream_attn_variants, dream_stream_read, dream_kv_commit,
    dream_tree_expand_workspace, dream_tree_expand_level, dream_tree_finalize,
    dream_attention_entropy_workspace, dream_attention_entropy, dream_spec_accept_workspace, dream_spec_accept, dream_project_rows, dream_project_rows_multi,
    alloc_workspace, to_device, EXPORTED_SYMBOLS,
)
