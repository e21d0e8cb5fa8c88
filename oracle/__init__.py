"""CPU oracle for Flash-LoRA-Attention.  Test infrastructure only: nothing on
the product path may import this package (see lra_oracle's header)."""
from .lra_oracle import (  # noqa: F401
    gather_paged, materialise_kv, softmax_weights, attend, decode, prefill,
    rope_rotate, project_new_tokens, scatter_paged, scatter_paged_l,
)
