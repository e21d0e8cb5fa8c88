"""Plain fp64 CPU oracle for Flash-LoRA-Attention (LRAgent, arxiv 2602.01053).

TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may call this.  It shares no code with the HIP
library and imports nothing from it.

What it computes is the *definition* the reordered kernel must reproduce
(paper Sec. 3.3, the un-reordered form O = P (V_base + V_lr B); App. B,
P = softmax(Q K^T / sqrt(d_head)); App. D.1 for the same decomposition on the
key side, K = K_base + K_lr B, taken here without a rotation in between):

    K = K_base + L . B_K      V = V_base + L . B_V       (materialised, per agent)
    S = scale . Q K^T  on the visible keys,  P = softmax_rows(S),  O = P V

No tiling, no online softmax, no reordering.  numpy matmul is the only library
primitive.  All arithmetic is float64 on the stored input values widened exactly.

Layouts follow the C header of the library:
  contiguous  k_base, v_base [n][Hkv][d], l [n][r]
  paged       k_base, v_base [num_blocks][Hkv][bs][d], l [num_blocks][bs][r],
              block_table [n_seqs][max_blocks]
  b_k, b_v    [n_adapters][r][Hkv*d]; kv head h owns columns h*d .. (h+1)*d-1
  GQA         q head g reads kv head g // (Hq // Hkv)

Pins (tests/test_oracle_pins.py): scalar brute force on tiny inputs, the n=1 and
Q=0 closed forms, the reordering identity of Sec. 3.3 / App. B on both sides,
the augmented-head identity, a library SDPA in float64 with B=0 and with
materialised K/V, a block-wise transcription of Alg. 1, softmax rows summing to
one, convex-hull / shift / permutation invariances.  The cache-append producer at the end
of the file (projection of new tokens, rotary embedding of the keys, paged scatter) is pinned
by the 2x2 rotation at d = 2, the identity at position 0, norm preservation, additivity of
positions, the relative-position property of rotated dot products, explicit loops on tiny
inputs and the scatter / gather round trip.  The rotary key side (key_rope_theta) is pinned
against attention over keys rotated as a whole, RoPE(K'_base + L B_K), by a scalar loop, and
by its two degenerate cases (B_K = 0, a single token at position 0).  Every function is pinned.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def gather_paged(pool_kv: np.ndarray, block_ids: Sequence[int], n: int) -> np.ndarray:
    """Logical [n][Hkv][d] view of one sequence stored as [num_blocks][Hkv][bs][d].

    Token j lives in physical block block_ids[j // bs], slot j % bs."""
    pool_kv = np.asarray(pool_kv)
    bs = pool_kv.shape[2]
    nb = (n + bs - 1) // bs
    ids = np.asarray(block_ids[:nb], dtype=np.int64)
    if n and (ids.min() < 0 or ids.max() >= pool_kv.shape[0]):
        raise ValueError("block table entry out of range")
    blocks = pool_kv[ids]                                  # [nb][Hkv][bs][d]
    tok_major = np.transpose(blocks, (0, 2, 1, 3))         # [nb][bs][Hkv][d]
    return tok_major.reshape(nb * bs, pool_kv.shape[1], pool_kv.shape[3])[:n]


def gather_paged_l(pool_l: np.ndarray, block_ids: Sequence[int], n: int) -> np.ndarray:
    """Logical [n][r] view of the LR cache stored as [num_blocks][bs][r]."""
    pool_l = np.asarray(pool_l)
    bs = pool_l.shape[1]
    nb = (n + bs - 1) // bs
    ids = np.asarray(block_ids[:nb], dtype=np.int64)
    return pool_l[ids].reshape(nb * bs, pool_l.shape[2])[:n]


def materialise_kv(k_base_h, v_base_h, l, b_k_h, b_v_h, key_rope_theta: float = 0.0):
    """Per-agent keys and values of one kv head (Eq. 3 applied to the cache:
    base output plus LR cache times the agent's up-projection).

    k_base_h, v_base_h [n][d]; l [n][r]; b_k_h, b_v_h [r][d]  ->  K, V [n][d]

    key_rope_theta > 0 is the rotary setting of App. D.1 (LoRA on the key projection of a
    model with rotary embeddings): the cached base keys are the rotated ones, the adapter
    contribution is reconstructed in the head dimension and rotated by its token's position
    (= its cache row) before it is added,  K_j = K_base,j + RoPE_j(L_j B_K)."""
    l = _f64(l)
    k_lr = l @ _f64(b_k_h)
    if key_rope_theta > 0.0:
        n = k_lr.shape[0]
        k_lr = rope_rotate(k_lr[:, None, :], np.arange(n), key_rope_theta)[:, 0, :]
    k = _f64(k_base_h) + k_lr
    v = _f64(v_base_h) + l @ _f64(b_v_h)
    return k, v


def softmax_weights(q_rows, k, scale: float, n_visible) -> np.ndarray:
    """P [rows][n]: max-subtracted softmax of scale * q k^T over the first
    n_visible[row] keys; keys past that get weight exactly 0."""
    q_rows = _f64(q_rows)
    k = _f64(k)
    n = k.shape[0]
    s = scale * (q_rows @ k.T)                             # [rows][n]
    vis = np.arange(n)[None, :] < np.asarray(n_visible, dtype=np.int64)[:, None]
    if not vis.any(axis=1).all():
        raise ValueError("a query row sees no key")
    s = np.where(vis, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def attend(q_tok, k_base, v_base, l, b_k, b_v, scale: float, n_visible,
           q_to_kv: Optional[Sequence[int]] = None, key_rope_theta: float = 0.0) -> np.ndarray:
    """One agent on one sequence.

    q_tok [T][Hq][d] (T query tokens), k_base/v_base [n][Hkv][d], l [n][r],
    b_k/b_v [r][Hkv*d] (this agent's), n_visible [T] keys each token may see.
    Returns O [T][Hq][d] in float64."""
    q_tok = _f64(q_tok)
    t_new, hq, d = q_tok.shape
    n, hkv, _ = np.shape(k_base)
    if q_to_kv is None:
        if hq % hkv:
            raise ValueError("Hq must be a multiple of Hkv")
        q_to_kv = [g // (hq // hkv) for g in range(hq)]
    out = np.empty((t_new, hq, d), dtype=np.float64)
    for h in range(hkv):
        cols = slice(h * d, (h + 1) * d)
        k, v = materialise_kv(np.asarray(k_base)[:, h, :], np.asarray(v_base)[:, h, :], l,
                              np.asarray(b_k)[:, cols], np.asarray(b_v)[:, cols], key_rope_theta)
        for g in range(hq):
            if q_to_kv[g] != h:
                continue
            p = softmax_weights(q_tok[:, g, :], k, scale, n_visible)
            out[:, g, :] = p @ v
    return out


def _sequence_views(k_base, v_base, l, seq_lens, block_size, block_table, t):
    n_t = int(seq_lens[t])
    if block_size:
        ids = np.asarray(block_table)[t]
        return (gather_paged(k_base, ids, n_t), gather_paged(v_base, ids, n_t),
                gather_paged_l(l, ids, n_t))
    if len(seq_lens) != 1:
        raise ValueError("contiguous caches hold one sequence")
    return np.asarray(k_base)[:n_t], np.asarray(v_base)[:n_t], np.asarray(l)[:n_t]


def decode(q, k_base, v_base, l, b_k, b_v, query_adapter, seq_query_start, seq_lens,
           scale: float, block_size: int = 0, block_table=None, q_to_kv=None,
           key_rope_theta: float = 0.0) -> np.ndarray:
    """Every query is one new token that sees all n_t cached tokens of its
    sequence (the cache already holds that token's own K/V/L row).

    q [n_queries][Hq][d] -> O [n_queries][Hq][d] float64."""
    q = _f64(q)
    out = np.empty_like(q)
    start = [int(x) for x in np.asarray(seq_query_start)]
    for t in range(len(seq_lens)):
        if start[t + 1] == start[t]:
            continue
        kb, vb, lr = _sequence_views(k_base, v_base, l, seq_lens, block_size, block_table, t)
        n_t = kb.shape[0]
        for qi in range(start[t], start[t + 1]):
            a = int(np.asarray(query_adapter)[qi])
            out[qi] = attend(q[qi][None], kb, vb, lr, np.asarray(b_k)[a], np.asarray(b_v)[a],
                             scale, [n_t], q_to_kv, key_rope_theta)[0]
    return out


def prefill(q, k_base, v_base, l, b_k_a, b_v_a, n: int, scale: float, rows=None,
            q_to_kv=None, key_rope_theta: float = 0.0) -> np.ndarray:
    """One agent appends T = len(q) tokens at the end of a sequence of n cached
    tokens (n includes them, L = L_p + L_c in Alg. 1).  Causal mask aligned to
    the end: new token i sees keys 0 .. n - T + i.

    rows: optional subset of new-token indices to evaluate (rows are
    independent); the result then has len(rows) tokens."""
    q = _f64(q)
    t_new = q.shape[0]
    idx = np.arange(t_new) if rows is None else np.asarray(rows, dtype=np.int64)
    n_visible = n - t_new + idx + 1
    return attend(q[idx], np.asarray(k_base)[:n], np.asarray(v_base)[:n], np.asarray(l)[:n],
                  b_k_a, b_v_a, scale, n_visible, q_to_kv, key_rope_theta)


# --------------------------------------------------------------------------------------
# Cache-append producer (the step before the attention path; Sec. 3.2 and the caption of
# the base / LR cache diagram: the base cache comes from the pretrained projections, the
# LR cache from the shared LoRA down-projection, both for the newly appended tokens only).
# The paper fixes WHAT is stored - X W_K and X W_V as base cache, X A as LR cache, keys
# rotated by the model's rotary position embedding before they are cached (App. D.1 speaks
# of post-rotation keys) - not how; the rotation below is the usual rotate-half form.
# --------------------------------------------------------------------------------------
def rope_rotate(x, positions, theta: float) -> np.ndarray:
    """Rotary position embedding, rotate-half convention, on x [n][H][d] (d even).

    Pair (i, i + d/2) of token t is rotated by the angle positions[t] * theta**(-2i/d):
        out[i]       = x[i] cos - x[i + d/2] sin
        out[i + d/2] = x[i + d/2] cos + x[i] sin"""
    x = _f64(x)
    n, _, d = x.shape
    half = d // 2
    pos = _f64(positions).reshape(n, 1, 1)
    inv_freq = float(theta) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = pos * inv_freq.reshape(1, 1, half)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def project_new_tokens(x, w_cat, n_kv_heads: int, head_dim: int, rank: int, positions, rope_theta: float):
    """Rows the producer appends for the new tokens x [n_new][d_model].

    w_cat [2*Hkv*d + r][d_model] holds, one output feature per row, W_K (kv head h owns rows
    h*d .. (h+1)*d-1), then W_V, then the shared down-projection A transposed.  Returns
    (k_rows [n_new][Hkv][d], v_rows [n_new][Hkv][d], l_rows [n_new][r]); keys are rotated
    when rope_theta > 0."""
    x, w_cat = _f64(x), _f64(w_cat)
    hd = n_kv_heads * head_dim
    if w_cat.shape != (2 * hd + rank, x.shape[1]):
        raise ValueError("w_cat must be [2*Hkv*d + r][d_model]")
    y = x @ w_cat.T
    n = x.shape[0]
    k = y[:, :hd].reshape(n, n_kv_heads, head_dim)
    v = y[:, hd:2 * hd].reshape(n, n_kv_heads, head_dim)
    l = y[:, 2 * hd:]
    if rope_theta > 0:
        k = rope_rotate(k, positions, rope_theta)
    return k, v, l


def scatter_paged(pool_kv: np.ndarray, block_ids: Sequence[int], start: int, rows: np.ndarray) -> None:
    """Write rows [m][Hkv][d] as tokens start .. start+m-1 of a sequence stored as
    [num_blocks][Hkv][bs][d] (in place; the inverse of gather_paged on that range)."""
    bs = pool_kv.shape[2]
    for i in range(rows.shape[0]):
        j = start + i
        pool_kv[block_ids[j // bs], :, j % bs, :] = rows[i]


def scatter_paged_l(pool_l: np.ndarray, block_ids: Sequence[int], start: int, rows: np.ndarray) -> None:
    """The same for the LR cache stored as [num_blocks][bs][r]."""
    bs = pool_l.shape[1]
    for i in range(rows.shape[0]):
        j = start + i
        pool_l[block_ids[j // bs], j % bs, :] = rows[i]
