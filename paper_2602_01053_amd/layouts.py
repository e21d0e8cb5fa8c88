"""Cache layouts that reduce other LoRA cache-sharing schemes to the one the kernels take.

The library's calls take ONE low-rank cache L [tokens][r] shared by every agent and used
by both the key and the value side (the BaseLRShared scheme of LRAgent Sec. 3.2 with a
shared down-projection).  Two other arrangements of the paper are the same computation on
a wider L with zero-padded up-projections, so they need no kernel of their own:

* BaseShared (Sec. 3.2): the base cache is shared, every agent a keeps its own low-rank
  cache L_a = X A_a.  Concatenate along the rank, L = [L_0 | L_1 | ...], and give adapter a
  the up-projection whose rows a*r .. (a+1)*r are B_a and whose other rows are zero:
  L . B'_a = L_a . B_a exactly (the added terms are products with zero).
* Separate down-projections for keys and values (LoRA on W_K and on W_V have different A):
  L = [L_K | L_V], B'_K = [B_K ; 0], B'_V = [0 ; B_V].

* Ranks that are not a multiple of 8 (the qkvo setting of App. D.1 uses r = 4): the matrix-core
  kernels move L rows in 16-byte pieces and take ranks that are multiples of 8; other ranks run
  on the vector-ALU kernels.  pad_rank() appends zero columns to L and zero rows to every B up to
  the next multiple of 8 - the same outputs (products with zero), at matrix-core speed.  A
  producer that pads the rows of A the same way (W_cat of lra_cache_append) writes such an L itself.

Both widen the rank to the sum of the parts (the kernels take up to 64) and the low-rank
cache bytes with it - which is the memory cost the paper attributes to these schemes.
Pure concatenation and zero padding: no arithmetic of the method lives here.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import torch


def concat_low_rank(parts: Sequence[torch.Tensor]) -> torch.Tensor:
    """[tokens][r_i] caches (or paged [blocks][block_size][r_i]) -> one cache of rank sum(r_i)."""
    return torch.cat(list(parts), dim=-1).contiguous()


def embed_up_projection(b: torch.Tensor, slot: int, ranks: Sequence[int]) -> torch.Tensor:
    """b [r_slot][Hkv*d] -> [sum(ranks)][Hkv*d], zero except the rows of part `slot`."""
    assert b.shape[0] == ranks[slot]
    out = torch.zeros(sum(ranks), b.shape[1], dtype=b.dtype, device=b.device)
    start = sum(ranks[:slot])
    out[start:start + ranks[slot]] = b
    return out


def base_shared(l_per_agent: Sequence[torch.Tensor], b_k: torch.Tensor, b_v: torch.Tensor
                ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """BaseShared as one call: per-agent caches L_a [tokens][r] and adapter stacks
    b_k, b_v [agents][r][Hkv*d] -> (L [tokens][agents*r], b_k', b_v' [agents][agents*r][Hkv*d])."""
    n_agents = len(l_per_agent)
    ranks = [int(x.shape[-1]) for x in l_per_agent]
    assert b_k.shape[0] == n_agents and b_v.shape[0] == n_agents
    l = concat_low_rank(l_per_agent)
    bk = torch.stack([embed_up_projection(b_k[a], a, ranks) for a in range(n_agents)])
    bv = torch.stack([embed_up_projection(b_v[a], a, ranks) for a in range(n_agents)])
    return l, bk, bv


def separate_key_value(l_k: torch.Tensor, l_v: torch.Tensor, b_k: torch.Tensor, b_v: torch.Tensor
                       ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Different down-projections for keys and values: L_K, L_V [tokens][r] and stacks
    b_k, b_v [agents][r][Hkv*d] -> (L [tokens][2r], b_k' = [B_K ; 0], b_v' = [0 ; B_V])."""
    ranks = [int(l_k.shape[-1]), int(l_v.shape[-1])]
    l = concat_low_rank([l_k, l_v])
    bk = torch.stack([embed_up_projection(b_k[a], 0, ranks) for a in range(b_k.shape[0])])
    bv = torch.stack([embed_up_projection(b_v[a], 1, ranks) for a in range(b_v.shape[0])])
    return l, bk, bv


def pad_rank(l: torch.Tensor, b_k: torch.Tensor, b_v: torch.Tensor, multiple: int = 8
             ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """L [...][r] and stacks b_k, b_v [agents][r][Hkv*d] (either may be None) -> the same with the rank
    padded by zeros to the next multiple of `multiple`: L . B is unchanged."""
    r = int(l.shape[-1])
    pad = (-r) % multiple
    if pad == 0:
        return l, b_k, b_v
    widen = lambda b: None if b is None else torch.cat(
        [b, torch.zeros(b.shape[0], pad, b.shape[2], dtype=b.dtype, device=b.device)], dim=1).contiguous()
    lp = torch.cat([l, torch.zeros(*l.shape[:-1], pad, dtype=l.dtype, device=l.device)], dim=-1).contiguous()
    return lp, widen(b_k), widen(b_v)
