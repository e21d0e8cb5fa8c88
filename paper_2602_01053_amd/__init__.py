"""Flash-LoRA-Attention for MI355X: ctypes binding over the in-tree HIP library."""
from .binding import (  # noqa: F401
    LraAdapters, LraCache, LraError, LraProjection, LraShape, LraTuning, lra_attn_decode, lra_attn_decode_static, lra_attn_prefill,
    lra_append_workspace_bytes, lra_cache_append, lra_set_append_k_splits, lra_probe_mfma_bf16, lra_probe_stream_read, lra_set_append_skinny, lra_set_append_stages, lra_set_append_tile,
    lra_set_decode_split_keys, lra_set_kernel_variant,
    lra_set_prefill_splits, lra_set_profile_mode, lra_set_rope_key_prepass, lra_set_short_prefill, lra_status_string, lra_workspace_bytes,
    load_library, make_cache, make_shape,
)
