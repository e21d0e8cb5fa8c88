"""Seeded synthetic inputs for the Flash-LoRA-Attention path.

This module only draws random numbers, rounds them to a storage dtype and moves
them into the documented memory layouts.  It holds none of the attention
arithmetic: no scores, no softmax, no K/V expansion.  Both the CPU oracle's
tests and the HIP path's tests/bench take their tensors from here, so the two
sides see bit-identical inputs.

What the tensors are (paper Sec. 3.2, BaseLRShared; Alg. 1 inputs):
  k_base, v_base : shared base cache, one copy for every agent,
  l              : shared low-rank ("LR") cache, the activations right after the
                   shared LoRA down-projection A, produced here as X @ A,
  b_k, b_v       : per-agent LoRA up-projections B (Eq. 1-3: r x d_out).

Everything is generated on the CPU with torch.Generator so a run with and
without a GPU sees the same bits.  Large tensors are drawn in fixed row chunks
in a fixed order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import torch

_CHUNK_ROWS = 8192
BASE_SEED = 20260201


@dataclass
class Workload:
    """One call's worth of inputs, in the layouts the C-ABI documents.

    Contiguous (block_size == 0, one sequence):
        k_base, v_base : [n][Hkv][d]   (token-major)
        l              : [n][r]
    Paged (block_size > 0):
        k_base, v_base : [num_blocks][Hkv][block_size][d]
        l              : [num_blocks][block_size][r]
        block_table    : int32 [n_seqs][max_blocks_per_seq]; entry (t, p) is the
                         physical block holding tokens p*bs .. p*bs+bs-1 of
                         sequence t; unused entries are -1.
    Queries are grouped by sequence: the queries of sequence t are
    seq_query_start[t] .. seq_query_start[t+1]-1.
    """
    name: str
    kind: str                       # "decode" | "prefill"
    dtype: torch.dtype
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rank: int
    scale: float
    seq_lens: List[int]
    n_new: int                      # query tokens per agent (1 for decode)
    q: torch.Tensor                 # decode [n_queries][Hq][d]; prefill [n_new][Hq][d]
    k_base: torch.Tensor
    v_base: torch.Tensor
    l: torch.Tensor
    b_k: torch.Tensor               # [n_adapters][r][Hkv*d]
    b_v: torch.Tensor
    query_adapter: torch.Tensor     # int32 [n_queries]
    seq_query_start: torch.Tensor   # int32 [n_seqs+1]
    block_size: int = 0
    block_table: Optional[torch.Tensor] = None
    num_blocks: int = 0
    seed: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def n_seqs(self) -> int:
        return len(self.seq_lens)

    @property
    def n_queries(self) -> int:
        return int(self.query_adapter.numel())

    @property
    def n_adapters(self) -> int:
        return int(self.b_k.shape[0])

    @property
    def max_blocks_per_seq(self) -> int:
        return 0 if self.block_table is None else int(self.block_table.shape[1])

    def query_seq(self) -> torch.Tensor:
        """int32 [n_queries]: sequence index of every query (from the CSR form)."""
        out = torch.empty(self.n_queries, dtype=torch.int32)
        s = self.seq_query_start.tolist()
        for t in range(self.n_seqs):
            out[s[t]:s[t + 1]] = t
        return out

    def algorithmic_bytes(self) -> int:
        """Bytes one call must move at least once: every cached token of K_base,
        V_base and L that some query can see, Q, the output, and the B stacks."""
        es = self.q.element_size()
        toks = sum(self.seq_lens)
        kv = 2 * toks * self.n_kv_heads * self.head_dim * es
        lr = toks * self.rank * es
        b = (self.b_k.numel() + self.b_v.numel()) * es
        qo = 2 * self.q.numel() * es
        return kv + lr + b + qo

    def visible_pairs(self) -> int:
        """(query row, key) pairs that enter a softmax, summed over q heads."""
        s = self.seq_query_start.tolist()
        pairs = 0
        for t, n_t in enumerate(self.seq_lens):
            n_q = s[t + 1] - s[t]
            if self.kind == "decode":
                pairs += n_q * n_t
            else:
                lc = self.n_new
                pairs += n_q * (lc * (n_t - lc) + lc * (lc + 1) // 2)
        return pairs * self.n_q_heads

    def algorithmic_flops(self) -> int:
        """4(d+r) flop per visible pair (score + accumulate, paper App. B cost
        model with the key side added) plus the two rank-r projections per row."""
        d, r = self.head_dim, self.rank
        rows = self.n_queries * self.n_new * self.n_q_heads
        return 4 * (d + r) * self.visible_pairs() + 4 * rows * d * r


def _randn(gen: torch.Generator, *shape: int, std: float = 1.0) -> torch.Tensor:
    t = torch.randn(*shape, generator=gen, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    return t


def _randn_rows(gen: torch.Generator, rows: int, cols_shape, dtype) -> torch.Tensor:
    """[rows, *cols_shape] ~ N(0,1), drawn in fixed row chunks, stored as dtype."""
    out = torch.empty((rows, *cols_shape), dtype=dtype)
    for r0 in range(0, rows, _CHUNK_ROWS):
        r1 = min(rows, r0 + _CHUNK_ROWS)
        out[r0:r1] = _randn(gen, r1 - r0, *cols_shape).to(dtype)
    return out


def _lr_cache_from_hidden(gen: torch.Generator, rows: int, d_model: int,
                          a: torch.Tensor, dtype) -> torch.Tensor:
    """L = X @ A with X [rows][d_model] ~ N(0,1) drawn chunk-wise; fp32 product,
    one rounding to the storage dtype (the LR cache of paper Sec. 3.2)."""
    out = torch.empty((rows, a.shape[1]), dtype=dtype)
    for r0 in range(0, rows, _CHUNK_ROWS):
        r1 = min(rows, r0 + _CHUNK_ROWS)
        x = _randn(gen, r1 - r0, d_model)
        out[r0:r1] = (x @ a).to(dtype)
    return out


def _adapters(gen, n_adapters, rank, d_out, dtype, std=0.02):
    b_k = _randn(gen, n_adapters, rank, d_out, std=std).to(dtype)
    b_v = _randn(gen, n_adapters, rank, d_out, std=std).to(dtype)
    return b_k, b_v


def make_contiguous(name: str, kind: str, *, seed: int, dtype=torch.bfloat16,
                    n_agents: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                    rank: int, n: int, n_new: int = 1, d_model: Optional[int] = None,
                    b_std: float = 0.02, scale: Optional[float] = None) -> Workload:
    """One shared sequence of n cached tokens (the n_new query tokens included),
    n_agents agents (decode) or one agent with n_new tokens (prefill).

    d_model=None draws L ~ N(0,1) directly (tiny config); otherwise L = X @ A
    with A [d_model][r] ~ N(0, variance 1/d_model), which is unit variance too.
    """
    gen = torch.Generator().manual_seed(seed)
    d_out = n_kv_heads * head_dim
    if kind == "decode":
        q = _randn(gen, n_agents, n_q_heads, head_dim).to(dtype)
    else:
        assert n_agents == 1
        q = _randn_rows(gen, n_new, (n_q_heads, head_dim), dtype)
    k_base = _randn_rows(gen, n, (n_kv_heads, head_dim), dtype)
    v_base = _randn_rows(gen, n, (n_kv_heads, head_dim), dtype)
    if d_model is None:
        l = _randn_rows(gen, n, (rank,), dtype)
    else:
        a = _randn(gen, d_model, rank, std=d_model ** -0.5)
        l = _lr_cache_from_hidden(gen, n, d_model, a, dtype)
    b_k, b_v = _adapters(gen, n_agents, rank, d_out, dtype, b_std)
    return Workload(
        name=name, kind=kind, dtype=dtype, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
        head_dim=head_dim, rank=rank,
        scale=float(scale if scale is not None else head_dim ** -0.5),
        seq_lens=[n], n_new=n_new, q=q, k_base=k_base, v_base=v_base, l=l,
        b_k=b_k, b_v=b_v,
        query_adapter=torch.arange(n_agents, dtype=torch.int32),
        seq_query_start=torch.tensor([0, n_agents], dtype=torch.int32),
        seed=seed)


def make_paged(name: str, *, seed: int, dtype=torch.bfloat16, seq_lens: List[int],
               agents_per_seq: int, n_adapters: int, n_q_heads: int, n_kv_heads: int,
               head_dim: int, rank: int, d_model: Optional[int], block_size: int = 16,
               spare_blocks: int = 3, b_std: float = 0.02,
               distinct_adapter_per_query: bool = False,
               poison: bool = True) -> Workload:
    """Ragged batch decode over a paged cache.

    Every sequence's tokens are drawn as in make_contiguous and scattered into
    physical blocks taken from a random permutation of one pool.  Slots that no
    sequence owns (the tail of a last block, spare blocks) are filled with NaN
    when `poison` is set, so a kernel that reads past a sequence's length shows
    up in its output.
    """
    gen = torch.Generator().manual_seed(seed)
    n_seqs = len(seq_lens)
    d_out = n_kv_heads * head_dim
    blocks_per_seq = [(n + block_size - 1) // block_size for n in seq_lens]
    num_blocks = sum(blocks_per_seq) + spare_blocks
    max_blocks = max(blocks_per_seq)
    perm = torch.randperm(num_blocks, generator=gen)
    fill = float("nan") if poison else 0.0
    k_pool = torch.full((num_blocks, n_kv_heads, block_size, head_dim), fill, dtype=dtype)
    v_pool = torch.full((num_blocks, n_kv_heads, block_size, head_dim), fill, dtype=dtype)
    l_pool = torch.full((num_blocks, block_size, rank), fill, dtype=dtype)
    block_table = torch.full((n_seqs, max_blocks), -1, dtype=torch.int32)
    a = None if d_model is None else _randn(gen, d_model, rank, std=d_model ** -0.5)
    nxt = 0
    for t, n in enumerate(seq_lens):
        nb = blocks_per_seq[t]
        phys = perm[nxt:nxt + nb]
        nxt += nb
        block_table[t, :nb] = phys.to(torch.int32)
        k = _randn_rows(gen, n, (n_kv_heads, head_dim), dtype)
        v = _randn_rows(gen, n, (n_kv_heads, head_dim), dtype)
        if a is None:
            lr = _randn_rows(gen, n, (rank,), dtype)
        else:
            lr = _lr_cache_from_hidden(gen, n, d_model, a, dtype)
        full = (n // block_size) * block_size
        if full:
            nbf = full // block_size
            k_pool[phys[:nbf]] = k[:full].view(nbf, block_size, n_kv_heads, head_dim).permute(0, 2, 1, 3)
            v_pool[phys[:nbf]] = v[:full].view(nbf, block_size, n_kv_heads, head_dim).permute(0, 2, 1, 3)
            l_pool[phys[:nbf]] = lr[:full].view(nbf, block_size, rank)
        tail = n - full
        if tail:
            pb = int(phys[nb - 1])
            k_pool[pb, :, :tail] = k[full:].permute(1, 0, 2)
            v_pool[pb, :, :tail] = v[full:].permute(1, 0, 2)
            l_pool[pb, :tail] = lr[full:]
        del k, v, lr
    n_queries = n_seqs * agents_per_seq
    if distinct_adapter_per_query:
        n_adapters = n_queries
        query_adapter = torch.randperm(n_queries, generator=gen).to(torch.int32)
    else:
        query_adapter = (torch.arange(n_queries) % n_adapters).to(torch.int32)
    q = _randn(gen, n_queries, n_q_heads, head_dim).to(dtype)
    b_k, b_v = _adapters(gen, n_adapters, rank, d_out, dtype, b_std)
    return Workload(
        name=name, kind="decode", dtype=dtype, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
        head_dim=head_dim, rank=rank, scale=float(head_dim ** -0.5),
        seq_lens=list(seq_lens), n_new=1, q=q, k_base=k_pool, v_base=v_pool, l=l_pool,
        b_k=b_k, b_v=b_v, query_adapter=query_adapter,
        seq_query_start=(torch.arange(n_seqs + 1) * agents_per_seq).to(torch.int32),
        block_size=block_size, block_table=block_table, num_blocks=num_blocks, seed=seed)


def ragged_lengths(seed: int, n_seqs: int, lo: int, hi: int) -> List[int]:
    """Integer-uniform lengths in [lo, hi], inclusive, not rounded to a block."""
    gen = torch.Generator().manual_seed(seed)
    return torch.randint(lo, hi + 1, (n_seqs,), generator=gen).tolist()


# ---------------------------------------------------------------------------
# The five named configurations.
# ---------------------------------------------------------------------------
def config(index: int, *, shrink: int = 1) -> Workload:
    """Configuration `index` (1-based).  shrink > 1 divides the context lengths
    (and for prefill the new-token count) so a CPU-only run stays small; the
    head layout, rank and distributions are unchanged."""
    seed = BASE_SEED + index
    if index == 1:
        return make_contiguous("cfg1_tiny_decode_fp32", "decode", seed=seed, dtype=torch.float32,
                               n_agents=2, n_q_heads=4, n_kv_heads=4, head_dim=64, rank=8,
                               n=512 // shrink, d_model=None, scale=1.0 / 8.0)
    if index == 2:
        return make_contiguous("cfg2_llama3_8b_decode_a4_n8192_r16", "decode", seed=seed,
                               n_agents=4, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=16,
                               n=8192 // shrink, d_model=4096)
    if index == 3:
        return make_contiguous("cfg3_llama3_8b_prefill_2048_after_16384_r16", "prefill", seed=seed,
                               n_agents=1, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=16,
                               n=18432 // shrink, n_new=2048 // shrink, d_model=4096)
    if index == 4:
        return make_contiguous("cfg4_llama3_8b_decode_a8_n32768_r64", "decode", seed=seed,
                               n_agents=8, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=64,
                               n=32768 // shrink, d_model=4096)
    if index == 5:
        lens = ragged_lengths(seed, 16, 4096 // shrink, 65536 // shrink)
        return make_paged("cfg5_qwen25_7b_ragged_paged_decode_r32", seed=seed, seq_lens=lens,
                          agents_per_seq=4, n_adapters=4, n_q_heads=28, n_kv_heads=4,
                          head_dim=128, rank=32, d_model=3584, block_size=16)
    raise ValueError(f"no configuration {index}")
