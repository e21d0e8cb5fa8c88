"""Device-side holder for a Workload: copies the tensors to the GPU, builds the C
structs that describe them and calls the library.  Marshalling only."""
from __future__ import annotations

import torch

from . import binding as lra
from .workloads import Workload


class DeviceWorkload:
    """Device copies of a Workload plus the C structs that describe them."""

    def __init__(self, w: Workload, dev, head_major: bool = False, key_rope_theta: float = 0.0, host_lens: bool = True):
        self.w = w
        self.q = w.q.to(dev)
        if w.block_size == 0 and head_major:
            # [Hkv][n][d] storage, viewed as [n][Hkv][d]
            self.k_base = w.k_base.permute(1, 0, 2).contiguous().to(dev).permute(1, 0, 2)
            self.v_base = w.v_base.permute(1, 0, 2).contiguous().to(dev).permute(1, 0, 2)
        else:
            self.k_base = w.k_base.to(dev)
            self.v_base = w.v_base.to(dev)
        self.l = w.l.to(dev)
        self.b_k = w.b_k.to(dev)
        self.b_v = w.b_v.to(dev)
        self.seq_lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
        self.block_table = None if w.block_table is None else w.block_table.to(dev)
        self.query_adapter = w.query_adapter.to(dev)
        self.seq_query_start = w.seq_query_start.to(dev)
        s = w.seq_query_start.tolist()
        self.max_queries_per_seq = max(b - a for a, b in zip(s[:-1], s[1:]))
        self.shape = lra.make_shape(self.q, w.n_kv_heads, w.rank, w.scale, key_rope_theta)
        # (the host copy of the lengths only steers launch planning of batches)
        self.cache = lra.make_cache(self.k_base, self.v_base, self.l, self.seq_lens,
                                    max(w.seq_lens), self.block_table,
                                    seq_lens_host=list(w.seq_lens) if host_lens else None)
        self.out = torch.empty_like(self.q)
        self.workspace = None

    def alloc_workspace(self):
        w = self.w
        nbytes = lra.lra_workspace_bytes(self.shape, self.cache, w.n_queries,
                                         self.max_queries_per_seq, w.n_new if w.kind == "prefill" else 0)
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.q.device)
        return nbytes

    def decode(self, stream=None):
        lra.lra_attn_decode(self.shape, self.cache, self.b_k, self.b_v, self.w.n_adapters, self.q,
                            self.query_adapter, self.seq_query_start, self.max_queries_per_seq,
                            self.out, self.workspace, stream)

    def prefill(self, stream=None):
        lra.lra_attn_prefill(self.shape, self.cache, self.b_k, self.b_v, self.w.n_adapters, self.q,
                             0, int(self.w.query_adapter[0]), self.out, self.workspace, stream)
