"""Other cache-sharing schemes of the paper run through the same calls on a widened L
(paper_2602_01053_amd/layouts.py).  CPU part: the embedding is exact.  GPU part: the HIP
path on the embedded layout equals the oracle evaluated scheme by scheme - every agent with
its OWN low-rank cache (BaseShared, Sec. 3.2), and keys and values with different ones."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01053_amd import layouts
from paper_2602_01053_amd.workloads import Workload


def _case(seed, n, agents, hq, hkv, d, r, dtype=torch.bfloat16):
    gen = torch.Generator().manual_seed(seed)
    rn = lambda *s, std=1.0: (std * torch.randn(*s, generator=gen)).to(dtype)
    return dict(q=rn(agents, hq, d), k=rn(n, hkv, d), v=rn(n, hkv, d),
                l=[rn(n, r) for _ in range(agents)], l_v=[rn(n, r) for _ in range(agents)],
                b_k=rn(agents, r, hkv * d, std=0.05), b_v=rn(agents, r, hkv * d, std=0.05))


def _f(t):
    return t.to(torch.float64).numpy()


def test_embedding_is_exact():
    c = _case(1, 40, 3, 4, 2, 64, 8, dtype=torch.float64)
    l, bk, bv = layouts.base_shared(c["l"], c["b_k"], c["b_v"])
    assert l.shape == (40, 24) and bk.shape == (3, 24, 128)
    for a in range(3):
        np.testing.assert_array_equal(_f(l) @ _f(bk[a]), _f(c["l"][a]) @ _f(c["b_k"][a]))
        np.testing.assert_array_equal(_f(l) @ _f(bv[a]), _f(c["l"][a]) @ _f(c["b_v"][a]))
    l2, bk2, bv2 = layouts.separate_key_value(c["l"][0], c["l_v"][0], c["b_k"], c["b_v"])
    assert l2.shape == (40, 16)
    for a in range(3):
        np.testing.assert_array_equal(_f(l2) @ _f(bk2[a]), _f(c["l"][0]) @ _f(c["b_k"][a]))
        np.testing.assert_array_equal(_f(l2) @ _f(bv2[a]), _f(c["l_v"][0]) @ _f(c["b_v"][a]))


def test_rank_padding_is_exact():
    """pad_rank: zero columns of L against zero rows of B - the products L B_K and L B_V do not change by a bit."""
    c = _case(31, 50, 3, 4, 2, 8, 4, dtype=torch.float64)
    l, bk, bv = layouts.pad_rank(c["l"][0], c["b_k"], c["b_v"])
    assert l.shape == (50, 8) and bk.shape == (3, 8, 16) and bv.shape == (3, 8, 16)
    assert bool((l[:, 4:] == 0).all()) and bool((bk[:, 4:] == 0).all()) and bool((bv[:, 4:] == 0).all())
    for a in range(3):
        assert torch.equal(l @ bk[a], c["l"][0] @ c["b_k"][a]) and torch.equal(l @ bv[a], c["l"][0] @ c["b_v"][a])
    same = layouts.pad_rank(l, bk, None)
    assert same[0] is l and same[1] is bk and same[2] is None


def _workload(name, c, l, b_k, b_v, hq, hkv, d):
    agents = c["q"].shape[0]
    n = c["k"].shape[0]
    return Workload(name=name, kind="decode", dtype=torch.bfloat16, n_q_heads=hq, n_kv_heads=hkv, head_dim=d,
                    rank=int(l.shape[-1]), scale=1.0 / d ** 0.5, seq_lens=[n], n_new=1, q=c["q"], k_base=c["k"],
                    v_base=c["v"], l=l, b_k=b_k, b_v=b_v, query_adapter=torch.arange(agents, dtype=torch.int32),
                    seq_query_start=torch.tensor([0, agents], dtype=torch.int32))


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [(3000, 4, 32, 8, 128, 16), (777, 3, 8, 2, 64, 8), (1500, 2, 28, 4, 128, 32)],
                         ids=["llama_4x16", "small_3x8", "qwen_2x32"])
def test_base_shared_decode(shape):
    """Every agent attends over K_base + L_a B_K,a and V_base + L_a B_V,a with its own L_a."""
    from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors, run_decode
    n, agents, hq, hkv, d, r = shape
    c = _case(900 + n, n, agents, hq, hkv, d, r)
    l, bk, bv = layouts.base_shared(c["l"], c["b_k"], c["b_v"])
    got = run_decode(_workload("base_shared", c, l, bk, bv, hq, hkv, d), "cuda:0")
    ref = np.concatenate([
        oracle.decode(_f(c["q"][a:a + 1]), _f(c["k"]), _f(c["v"]), _f(c["l"][a]), _f(c["b_k"]), _f(c["b_v"]),
                      np.array([a], dtype=np.int32), np.array([0, 1], dtype=np.int32), [n], 1.0 / d ** 0.5)
        for a in range(agents)])
    rel, mx = errors(got, ref)
    print(f"base_shared {shape}: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


@pytest.mark.gpu
def test_separate_key_and_value_caches_decode():
    """Keys use L_K B_K,a, values L_V B_V,a: the oracle materialises both sides one by one."""
    from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors, run_decode
    n, agents, hq, hkv, d, r = 2100, 4, 32, 8, 128, 16
    c = _case(950, n, agents, hq, hkv, d, r)
    l_k, l_v = c["l"][0], c["l_v"][0]
    l, bk, bv = layouts.separate_key_value(l_k, l_v, c["b_k"], c["b_v"])
    got = run_decode(_workload("separate_kv", c, l, bk, bv, hq, hkv, d), "cuda:0")
    g = hq // hkv
    ref = np.zeros((agents, hq, d))
    for a in range(agents):
        k_full = _f(c["k"]) + (_f(l_k) @ _f(c["b_k"][a])).reshape(n, hkv, d)
        v_full = _f(c["v"]) + (_f(l_v) @ _f(c["b_v"][a])).reshape(n, hkv, d)
        for h in range(hq):
            s = k_full[:, h // g, :] @ _f(c["q"][a, h]) / d ** 0.5
            p = np.exp(s - s.max())
            ref[a, h] = (p / p.sum()) @ v_full[:, h // g, :]
    rel, mx = errors(got, ref)
    print(f"separate_kv: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


@pytest.mark.gpu
def test_rank_four_padded_to_eight_decode():
    """The qkvo rank of App. D.1 (r = 4) on the matrix-core kernels through pad_rank; the oracle sees rank 4."""
    from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors, run_decode
    n, agents, hq, hkv, d, r = 2100, 4, 32, 8, 128, 4
    c = _case(960, n, agents, hq, hkv, d, r)
    l, bk, bv = layouts.pad_rank(c["l"][0], c["b_k"], c["b_v"])
    assert l.shape[-1] == 8
    got = run_decode(_workload("rank4_padded", c, l, bk, bv, hq, hkv, d), "cuda:0")
    ref = oracle.decode(_f(c["q"]), _f(c["k"]), _f(c["v"]), _f(c["l"][0]), _f(c["b_k"]), _f(c["b_v"]),
                        np.arange(agents, dtype=np.int32), np.array([0, agents], dtype=np.int32), [n], 1.0 / d ** 0.5)
    rel, mx = errors(got, ref)
    print(f"rank 4 padded to 8: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


# ---------------------------------------------------------------------------------------------
# BaseShared as a layout of the cache itself (lra_cache.l_adapter_stride > 0): every adapter has its
# own low-rank cache and the kernels read each agent's own rows - no widened rank, no zero padding.
# ---------------------------------------------------------------------------------------------
def _per_adapter_l(parts, storage, dev):
    """parts: list of [n][r] tensors -> device view indexed [adapter][n][r] over the given storage order."""
    stacked = torch.stack(parts)                                  # [A][n][r]
    if storage == "token_major":                                  # [n][A][r] storage
        return stacked.permute(1, 0, 2).contiguous().to(dev).permute(1, 0, 2)
    return stacked.contiguous().to(dev)                           # [A][n][r] storage


NATIVE_SHAPES = [
    # n, agents, Hq, Hkv, d, r
    (3000, 4, 32, 8, 128, 16),     # the Llama-3-8B decode shape: four agent slots per tile
    (777, 3, 8, 2, 64, 8),         # rank 8 in 16-rank column blocks
    (1500, 2, 28, 4, 128, 32),     # group of 7, two slots per tile
    (1200, 9, 8, 2, 128, 16),      # more agents than a tile holds: three row groups share the key stream
    (900, 3, 16, 4, 128, 64),      # rank 64: one agent per tile
    (500, 5, 4, 4, 64, 40),        # rank 40 in a 64-rank block, group of 1
    (300, 140, 32, 8, 128, 16),    # 35 row groups x 8 kv heads: more units than compute units, split-KV form of the column-block tile
    (1, 2, 4, 2, 128, 16),         # a single key
]


@pytest.mark.gpu
@pytest.mark.parametrize("storage", ["token_major", "adapter_major"])
@pytest.mark.parametrize("shape", NATIVE_SHAPES, ids=lambda c: "n%d_a%d_hq%d_hkv%d_d%d_r%d" % c)
@pytest.mark.parametrize("variant", [0, 1], ids=["mfma", "vector_alu"])
def test_base_shared_native_decode(shape, storage, variant):
    """Decode with one low-rank cache per adapter, agents mapped to adapters out of order; the oracle evaluates
    every agent with its own L_a."""
    import paper_2602_01053_amd as lra
    from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors
    n, agents, hq, hkv, d, r = shape
    dev = "cuda:0"
    c = _case(1700 + n + agents, n, agents, hq, hkv, d, r)
    adapter_of = torch.tensor([(3 * a + 1) % agents for a in range(agents)], dtype=torch.int32)   # a permutation
    q, k, v = c["q"].to(dev), c["k"].to(dev), c["v"].to(dev)
    l = _per_adapter_l(c["l"], storage, dev)
    bk, bv = c["b_k"].to(dev), c["b_v"].to(dev)
    lens = torch.tensor([n], dtype=torch.int32, device=dev)
    shape_c = lra.make_shape(q, hkv, r)
    cache = lra.make_cache(k, v, l, lens, n, None, l_per_adapter=True)
    out = torch.full_like(q, float("nan"))
    prev = lra.lra_set_kernel_variant(variant)
    try:
        ws = torch.empty(max(lra.lra_workspace_bytes(shape_c, cache, agents, agents), 256), dtype=torch.uint8, device=dev)
        qa, qstart = adapter_of.to(dev), torch.tensor([0, agents], dtype=torch.int32, device=dev)
        lra.lra_attn_decode(shape_c, cache, bk, bv, agents, q, qa, qstart, agents, out, ws)
        torch.cuda.synchronize()
    finally:
        lra.lra_set_kernel_variant(prev)
    ref = np.concatenate([
        oracle.decode(_f(c["q"][i:i + 1]), _f(c["k"]), _f(c["v"]), _f(c["l"][int(adapter_of[i])]), _f(c["b_k"]), _f(c["b_v"]),
                      np.array([int(adapter_of[i])], dtype=np.int32), np.array([0, 1], dtype=np.int32), [n], 1.0 / d ** 0.5)
        for i in range(agents)])
    rel, mx = errors(out.to(torch.float64).cpu().numpy(), ref)
    # a wrong low-rank cache (agent i reading adapter 0's rows) must be visible to the gate
    wrong = np.concatenate([
        oracle.decode(_f(c["q"][i:i + 1]), _f(c["k"]), _f(c["v"]), _f(c["l"][0]), _f(c["b_k"]), _f(c["b_v"]),
                      np.array([int(adapter_of[i])], dtype=np.int32), np.array([0, 1], dtype=np.int32), [n], 1.0 / d ** 0.5)
        for i in range(agents)])
    print(f"native base_shared {shape} {storage}: relL2={rel:.3e} maxabs={mx:.3e}; "
          f"the wrong cache would move it by {np.linalg.norm(wrong - ref) / np.linalg.norm(ref):.2e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL
    assert np.linalg.norm(wrong - ref) / np.linalg.norm(ref) > 4 * REL_L2_TOL


@pytest.mark.gpu
@pytest.mark.parametrize("n_new", [300, 7], ids=["tile_walking", "few_tokens_split_kv"])
@pytest.mark.parametrize("storage", ["token_major", "adapter_major"])
def test_base_shared_native_prefill(n_new, storage):
    """Prefill of adapter 2 over its own low-rank cache: the tile-walking kernel reads its rows with their
    stride; a few new tokens take the causal form of the split-KV kernel."""
    import paper_2602_01053_amd as lra
    from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors
    n, agents, hq, hkv, d, r, a = 1100, 3, 8, 2, 128, 16, 2
    dev = "cuda:0"
    c = _case(1800 + n_new, n, agents, hq, hkv, d, r)
    gen = torch.Generator().manual_seed(77)
    q = torch.randn(n_new, hq, d, generator=gen).to(torch.bfloat16)
    qd, k, v = q.to(dev), c["k"].to(dev), c["v"].to(dev)
    l = _per_adapter_l(c["l"], storage, dev)
    lens = torch.tensor([n], dtype=torch.int32, device=dev)
    shape_c = lra.make_shape(qd, hkv, r)
    cache = lra.make_cache(k, v, l, lens, n, None, l_per_adapter=True)
    out = torch.full_like(qd, float("nan"))
    ws = torch.empty(max(lra.lra_workspace_bytes(shape_c, cache, 1, 1, n_new), 256), dtype=torch.uint8, device=dev)
    bk, bv = c["b_k"].to(dev), c["b_v"].to(dev)
    lra.lra_attn_prefill(shape_c, cache, bk, bv, agents, qd, 0, a, out, ws)
    torch.cuda.synchronize()
    ref = oracle.prefill(_f(q), _f(c["k"]), _f(c["v"]), _f(c["l"][a]), _f(c["b_k"][a]), _f(c["b_v"][a]), n=n, scale=1.0 / d ** 0.5)
    rel, mx = errors(out.to(torch.float64).cpu().numpy(), ref)
    print(f"native base_shared prefill {n_new} {storage}: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


@pytest.mark.gpu
def test_base_shared_native_paged_decode():
    """Per-adapter low-rank caches on a paged ragged batch (vector-ALU kernels): [adapter][block][16][r] rows."""
    import paper_2602_01053_amd as lra
    from paper_2602_01053_amd import workloads as W
    from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors
    dev = "cuda:0"
    w = W.make_paged("bs_paged", seed=1900, seq_lens=[17, 300, 1027], agents_per_seq=2, n_adapters=3, n_q_heads=8, n_kv_heads=2,
                     head_dim=128, rank=16, d_model=None, b_std=0.05)
    gen = torch.Generator().manual_seed(1901)
    l_pools = [w.l] + [torch.where(torch.isnan(w.l.float()), w.l.float(), torch.randn(w.l.shape, generator=gen)).to(torch.bfloat16)
                       for _ in range(2)]
    l_dev = torch.stack(l_pools).to(dev)                           # [adapter][block][16][r]
    qd, k, v = w.q.to(dev), w.k_base.to(dev), w.v_base.to(dev)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
    shape_c = lra.make_shape(qd, w.n_kv_heads, w.rank)
    # the cache struct holds raw device pointers: every tensor it or the call names stays referenced until the sync
    table, bk, bv = w.block_table.to(dev), w.b_k.to(dev), w.b_v.to(dev)
    qa, qstart = w.query_adapter.to(dev), w.seq_query_start.to(dev)
    cache = lra.make_cache(k, v, l_dev, lens, max(w.seq_lens), table, l_per_adapter=True)
    out = torch.full_like(qd, float("nan"))
    nq = qd.shape[0]
    ws = torch.empty(max(lra.lra_workspace_bytes(shape_c, cache, nq, 2), 256), dtype=torch.uint8, device=dev)
    lra.lra_attn_decode(shape_c, cache, bk, bv, w.n_adapters, qd, qa, qstart, 2, out, ws)
    torch.cuda.synchronize()
    ref = np.zeros(tuple(w.q.shape))
    for i in range(nq):
        a = int(w.query_adapter[i])
        t = int(np.searchsorted(w.seq_query_start.numpy(), i, side="right") - 1)
        ref[i] = oracle.decode(_f(w.q[i:i + 1]), _f(w.k_base), _f(w.v_base), _f(l_pools[a]), _f(w.b_k), _f(w.b_v),
                               np.array([a], dtype=np.int32), np.array([0] * (t + 1) + [1] * (len(w.seq_lens) - t), dtype=np.int32),
                               w.seq_lens, w.scale, block_size=16, block_table=w.block_table.numpy())[0]
    rel, mx = errors(out.to(torch.float64).cpu().numpy(), ref)
    print(f"native base_shared paged: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL
