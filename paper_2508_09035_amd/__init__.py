"""MI355X-native causal prefill attention fused with prompt-refinement data
extraction (token importance from the observation window, top-k selection).

All compute runs in the HIP library `libpdd.so` (C ABI in include/pdd.h);
this package only marshals arguments.  There is no CPU fallback: calling any
op without the built library raises.
"""
from .binding import (
    PddError,
    library_path,
    load_library,
    version,
    set_option,
    prefill_attn,
    prefill_attn_chunked,
    prefill_attn_chunked_noalloc,
    token_importance,
    select_topk,
    select_topk_pooled,
    POOL_NONE,
    POOL_MAX,
    POOL_AVG,
    select_sentences,
    SENT_SUM,
    SENT_MEAN,
    pack_mask,
    pack_mask_layout,
    aggregate_scores,
    choose_r_L,
    workspace_bytes,
    AttnDesc,
    make_desc,
    OPT_ATTN_WAVES,
    OPT_IMPORTANCE_KEYS,
    CALL_PREFILL_ATTN,
    CALL_PREFILL_ATTN_CHUNKED,
    CALL_TOKEN_IMPORTANCE,
    CALL_SELECT_TOPK,
)

__all__ = [
    "PddError", "library_path", "load_library", "version", "set_option", "prefill_attn",
    "prefill_attn_chunked", "prefill_attn_chunked_noalloc", "token_importance", "select_topk", "select_topk_pooled", "POOL_NONE", "POOL_MAX", "POOL_AVG", "select_sentences", "SENT_SUM", "SENT_MEAN", "pack_mask", "pack_mask_layout", "aggregate_scores", "choose_r_L", "workspace_bytes", "AttnDesc",
    "make_desc", "OPT_ATTN_WAVES", "OPT_IMPORTANCE_KEYS",
]
