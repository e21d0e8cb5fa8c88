"""Parity of the HIP library against the fp64 oracle, through the C ABI.

Bar (stated for bf16 inputs with fp32 accumulation): relative L2 <= 5e-3 over the
whole output AND over every single query / new token, max-abs <= 2e-2.  fp32
inputs are additionally held to relative L2 <= 2e-5.
"""
import numpy as np
import pytest
import torch

import paper_2602_01053_amd as lra
from paper_2602_01053_amd import workloads as W
from tests.harness import (MAX_ABS_TOL, REL_L2_TOL, DeviceWorkload, errors, oracle_decode,
                           oracle_prefill, oracle_prefill_by_blocks, run_decode, run_prefill)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# 0: automatic choice (bf16: MFMA kernels, and among them the one-workgroup-per-CU streaming form of the
# split-KV kernel wherever a call qualifies); 1: vector-ALU kernels; 2: MFMA kernels without the streaming form
@pytest.fixture(params=[0, 1, 2], ids=["auto", "valu", "mfma_no_stream_form"])
def variant(request):
    old = lra.lra_set_kernel_variant(request.param)
    yield request.param
    lra.lra_set_kernel_variant(old)


def _gate(got, ref, fp32=False, label=""):
    rel, mx = errors(got, ref)
    print(f"{label}: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL, (label, rel, mx)
    if fp32:
        assert rel <= 2e-5, (label, rel)


# ---- the five named configurations at full size -----------------------------
def test_config1_tiny_decode_fp32(variant):
    w = W.config(1)
    _gate(run_decode(w, DEV), oracle_decode(w), fp32=True, label=w.name)


@pytest.mark.parametrize("head_major", [False, True], ids=["token_major", "head_major"])
def test_config2_llama_decode(variant, head_major):
    w = W.config(2)
    _gate(run_decode(w, DEV, head_major), oracle_decode(w), label=w.name)


def test_config4_long_multi_agent_decode(variant):
    w = W.config(4)
    _gate(run_decode(w, DEV), oracle_decode(w), label=w.name)


def test_config5_ragged_paged_decode():
    w = W.config(5)
    print("sum of lengths", sum(w.seq_lens), flush=True)
    _gate(run_decode(w, DEV), oracle_decode(w), label=w.name)


def test_config3_prefill_every_row():
    """Full-size causal prefill in the launch configuration the benchmark times, compared with the
    oracle on every one of its 2048 x 32 output rows."""
    w = W.config(3)
    got = run_prefill(w, DEV)
    assert np.isfinite(got).all()
    _gate(got, oracle_prefill_by_blocks(w), label=w.name)


# ---- small shapes: several tiles, ragged tails, odd groups ------------------
DECODE_CASES = [
    # n, agents, Hq, Hkv, d, r
    (1, 1, 4, 4, 64, 8),
    (17, 3, 8, 2, 128, 16),
    (63, 2, 4, 1, 64, 4),
    (64, 5, 8, 8, 128, 1),
    (65, 1, 14, 2, 128, 32),     # group of 7
    (257, 4, 32, 8, 128, 16),
    (1000, 7, 16, 4, 64, 24),
    (1031, 9, 16, 1, 128, 64),   # group of 16, > 8 agents
    (4099, 17, 4, 2, 128, 48),
]


@pytest.mark.parametrize("case", DECODE_CASES, ids=lambda c: "n%d_a%d_hq%d_hkv%d_d%d_r%d" % c)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "fp32"])
def test_decode_small_shapes(variant, case, dtype):
    n, agents, hq, hkv, d, r = case
    w = W.make_contiguous("small", "decode", seed=1000 + n, dtype=dtype, n_agents=agents,
                          n_q_heads=hq, n_kv_heads=hkv, head_dim=d, rank=r, n=n, d_model=None,
                          b_std=0.05)
    _gate(run_decode(w, DEV), oracle_decode(w), fp32=dtype == torch.float32, label=str(case))


PREFILL_CASES = [
    # n, n_new, Hq, Hkv, d, r
    (1, 1, 4, 4, 64, 8),
    (40, 40, 4, 2, 128, 16),       # no old context
    (130, 3, 8, 2, 128, 16),
    (200, 129, 4, 4, 64, 8),
    (513, 257, 14, 2, 128, 32),
    (1500, 300, 8, 1, 128, 64),
    (700, 200, 8, 2, 128, 24),     # rank padded to 32 inside the MFMA kernel
    (391, 150, 6, 2, 64, 48),      # rank padded to 64, half-empty last block
    (260, 131, 4, 4, 128, 20),     # rank not a multiple of 8: vector-ALU kernels
]


@pytest.mark.parametrize("case", PREFILL_CASES, ids=lambda c: "n%d_new%d_hq%d_hkv%d_d%d_r%d" % c)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "fp32"])
def test_prefill_small_shapes(variant, case, dtype):
    n, n_new, hq, hkv, d, r = case
    w = W.make_contiguous("small", "prefill", seed=2000 + n, dtype=dtype, n_agents=1, n_q_heads=hq,
                          n_kv_heads=hkv, head_dim=d, rank=r, n=n, n_new=n_new, d_model=None,
                          b_std=0.05)
    _gate(run_prefill(w, DEV), oracle_prefill(w), fp32=dtype == torch.float32, label=str(case))


SHORT_PREFILL_CASES = [
    # n, n_new, Hq, Hkv, d, r
    (1000, 1, 8, 2, 128, 16),
    (1000, 7, 8, 2, 128, 16),
    (4099, 16, 32, 8, 128, 16),    # two row tiles, several splits
    (300, 13, 14, 2, 128, 32),     # group of 7: 8 rows per token, several row groups
    (777, 16, 16, 1, 64, 64),      # group of 16
    (64, 16, 4, 4, 64, 8),         # context exactly four times the new tokens
    (2000, 8, 8, 2, 128, 64),      # 4 token slots x 4 rank blocks x 2 row tiles: Qt comes from the pre-pass kernel
    (1500, 6, 16, 4, 64, 40),      # the same at d = 64, rank 40 (3 rank blocks), a ragged last row tile
]


@pytest.mark.parametrize("case", SHORT_PREFILL_CASES, ids=lambda c: "n%d_new%d_hq%d_hkv%d_d%d_r%d" % c)
@pytest.mark.parametrize("path", ["split_kv", "tile_walk"])
def test_short_prefill_both_paths(case, path):
    """A few new tokens after a longer context: served by the split-KV decode kernels with a
    causal limit per row (default) or by the tile-walking prefill kernel (path switched off);
    both must match the oracle."""
    n, n_new, hq, hkv, d, r = case
    w = W.make_contiguous("short_prefill", "prefill", seed=3000 + n + n_new, n_agents=1, n_q_heads=hq,
                          n_kv_heads=hkv, head_dim=d, rank=r, n=n, n_new=n_new, d_model=None, b_std=0.05)
    old = lra.lra_set_short_prefill(64 if path == "split_kv" else 0)
    old_s = lra.lra_set_prefill_splits(1)
    try:
        dw = DeviceWorkload(w, DEV)
        nbytes = dw.alloc_workspace()
        assert (nbytes > 0) == (path == "split_kv")
        dw.out.fill_(float("nan"))
        dw.prefill()
        torch.cuda.synchronize()
        got = dw.out.to(torch.float64).cpu().numpy()
    finally:
        lra.lra_set_short_prefill(old)
        lra.lra_set_prefill_splits(old_s)
    _gate(got, oracle_prefill(w), label=f"{case} {path}")


SPLIT_PREFILL_CASES = [
    # n, n_new, Hq, Hkv, d, r, splits (0 = automatic)
    (3000, 200, 8, 2, 128, 16, 0),     # automatic: few q tiles, several shares
    (2048, 130, 4, 4, 64, 8, 3),
    (5000, 700, 14, 2, 128, 32, 4),    # ragged last q tile, group of 7
    (1100, 1100, 4, 1, 128, 64, 2),    # no old context: later shares hold rows that see nothing of them
    (700, 300, 8, 2, 64, 48, 32),      # more shares than key tiles: empty shares
]


@pytest.mark.parametrize("case", SPLIT_PREFILL_CASES, ids=lambda c: "n%d_new%d_hq%d_hkv%d_d%d_r%d_s%d" % c)
def test_prefill_key_tiles_shared_by_workgroups(case):
    """The tile-walking prefill kernel with the key tiles of each q tile divided among several
    workgroups plus the merge kernel."""
    n, n_new, hq, hkv, d, r, splits = case
    w = W.make_contiguous("split_prefill", "prefill", seed=4000 + n + n_new, n_agents=1, n_q_heads=hq,
                          n_kv_heads=hkv, head_dim=d, rank=r, n=n, n_new=n_new, d_model=None, b_std=0.05)
    old_s = lra.lra_set_prefill_splits(splits)
    old_t = lra.lra_set_short_prefill(0)
    try:
        dw = DeviceWorkload(w, DEV)
        nbytes = dw.alloc_workspace()
        assert nbytes > 0
        dw.out.fill_(float("nan"))
        dw.prefill()
        torch.cuda.synchronize()
        got = dw.out.to(torch.float64).cpu().numpy()
    finally:
        lra.lra_set_prefill_splits(old_s)
        lra.lra_set_short_prefill(old_t)
    _gate(got, oracle_prefill(w), label=str(case))


def test_short_prefill_on_paged_cache_value_only():
    """Split-KV prefill of 5 new tokens on a paged, ragged cache without B_K."""
    w = W.make_paged("paged_short_prefill", seed=92, seq_lens=[40, 333, 1500], agents_per_seq=1, n_adapters=3,
                     n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, d_model=None, b_std=0.05)
    import oracle
    f = lambda t: t.to(torch.float64).numpy()
    for seq, n_new in [(0, 5), (1, 16), (2, 9)]:
        gen = torch.Generator().manual_seed(600 + seq)
        q = torch.randn(n_new, 8, 128, generator=gen).to(torch.bfloat16)
        adapter = seq % 3
        dw = DeviceWorkload(w, DEV)
        qd = q.to(DEV)
        out = torch.full_like(qd, float("nan"))
        ws_bytes = lra.lra_workspace_bytes(dw.shape, dw.cache, 1, 1, n_new)
        assert ws_bytes > 0
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
        lra.lra_attn_prefill(dw.shape, dw.cache, None, dw.b_v, w.n_adapters, qd, seq, adapter, out, ws)
        torch.cuda.synchronize()
        n_t = w.seq_lens[seq]
        ids = w.block_table[seq].numpy()
        kb = oracle.gather_paged(f(w.k_base), ids, n_t)
        vb = oracle.gather_paged(f(w.v_base), ids, n_t)
        lr = oracle.lra_oracle.gather_paged_l(f(w.l), ids, n_t)
        ref = oracle.prefill(f(q), kb, vb, lr, np.zeros_like(f(w.b_k[adapter])), f(w.b_v[adapter]), n=n_t, scale=w.scale)
        _gate(out.to(torch.float64).cpu().numpy(), ref, label=f"paged short prefill seq {seq} n_new {n_new}")


@pytest.mark.parametrize("seq,n_new", [(0, 1), (1, 77), (2, 300), (3, 1027)])
def test_prefill_on_paged_cache(variant, seq, n_new):
    """Causal prefill of the last n_new tokens of one sequence of a paged, ragged cache
    (block table lookups, a last block that is partly filled, NaN in the free slots)."""
    w = W.make_paged("paged_prefill", seed=91, seq_lens=[1, 130, 300, 1027], agents_per_seq=1, n_adapters=3,
                     n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, d_model=None, b_std=0.05)
    gen = torch.Generator().manual_seed(500 + seq)
    q = torch.randn(n_new, 8, 128, generator=gen).to(torch.bfloat16)
    adapter = (seq + 1) % 3
    dw = DeviceWorkload(w, DEV)
    dw.alloc_workspace()
    qd = q.to(DEV)
    out = torch.full_like(qd, float("nan"))
    ws_bytes = lra.lra_workspace_bytes(dw.shape, dw.cache, 1, 1, n_new)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    lra.lra_attn_prefill(dw.shape, dw.cache, dw.b_k, dw.b_v, w.n_adapters, qd, seq, adapter, out, ws)
    torch.cuda.synchronize()
    import oracle
    f = lambda t: t.to(torch.float64).numpy()
    n_t = w.seq_lens[seq]
    ids = w.block_table[seq].numpy()
    kb = oracle.gather_paged(f(w.k_base), ids, n_t)
    vb = oracle.gather_paged(f(w.v_base), ids, n_t)
    lr = oracle.lra_oracle.gather_paged_l(f(w.l), ids, n_t)
    ref = oracle.prefill(f(q), kb, vb, lr, f(w.b_k[adapter]), f(w.b_v[adapter]), n=n_t, scale=w.scale)
    _gate(out.to(torch.float64).cpu().numpy(), ref, label=f"paged prefill seq {seq} n_new {n_new}")


def test_paged_small_ragged_distinct_adapters(variant):
    """Lengths that end inside a block, one adapter per query, NaN-poisoned free
    slots: nothing outside a sequence's own tokens may reach its output."""
    w = W.make_paged("paged_small", seed=77, seq_lens=[1, 15, 16, 17, 250, 1027], agents_per_seq=3,
                     n_adapters=0, n_q_heads=14, n_kv_heads=2, head_dim=128, rank=32, d_model=None,
                     distinct_adapter_per_query=True, b_std=0.05)
    _gate(run_decode(w, DEV), oracle_decode(w), label=w.name)


@pytest.mark.parametrize("mirror", ["none", "exact", "all_zero", "too_long"])
def test_host_copy_of_the_lengths_only_steers_planning(mirror):
    """lra_cache.seq_lens_host: the decode of a batch sizes its key shares from it; the results do not depend on
    it, whatever it holds, and a workspace sized without it serves the call with it."""
    import paper_2602_01053_amd as lra
    from paper_2602_01053_amd.runner import DeviceWorkload
    lens = [6000, 5500, 7000, 6500, 5300, 6900, 5251, 7001]
    w = W.make_paged("mirror", seed=79, seq_lens=lens, agents_per_seq=2, n_adapters=3, n_q_heads=16, n_kv_heads=4,
                     head_dim=128, rank=16, d_model=None, b_std=0.05)
    host = {"none": None, "exact": lens, "all_zero": [0] * len(lens), "too_long": [10 ** 6] * len(lens)}[mirror]
    dw = DeviceWorkload(w, DEV, host_lens=False)
    need_without = dw.alloc_workspace()
    dw.cache = lra.make_cache(dw.k_base, dw.v_base, dw.l, dw.seq_lens, max(lens), dw.block_table, seq_lens_host=host)
    need_with = lra.lra_workspace_bytes(dw.shape, dw.cache, w.n_queries, dw.max_queries_per_seq, 0)
    assert need_with <= need_without
    if mirror in ("exact", "too_long"):
        assert need_with < need_without  # 8 sequences x 4 kv heads of 5251 to 7001 keys: fewer, longer key shares
    dw.out.fill_(float("nan"))
    dw.decode()                        # on the workspace sized without the lengths
    torch.cuda.synchronize()
    _gate(dw.out.to(torch.float64).cpu().numpy(), oracle_decode(w), label=f"{w.name} {mirror}")


def test_one_long_sequence_in_a_paged_cache():
    """One sequence of 33000 tokens in a paged cache with 8 kv heads: long enough that the planner gives the split-KV
    kernel two workgroups per compute unit (512 key shares x kv heads), with a ragged last share and last block."""
    w = W.make_paged("long_paged", seed=80, seq_lens=[33001], agents_per_seq=3, n_adapters=3, n_q_heads=32, n_kv_heads=8,
                     head_dim=128, rank=16, d_model=None, b_std=0.05)
    _gate(run_decode(w, DEV), oracle_decode(w), label=w.name)


def test_uneven_queries_per_sequence(variant):
    """Sequences with 0, 1 and many queries in one call."""
    w = W.make_paged("uneven", seed=78, seq_lens=[300, 77, 129, 512], agents_per_seq=2, n_adapters=3,
                     n_q_heads=8, n_kv_heads=2, head_dim=64, rank=16, d_model=None, b_std=0.05)
    w.seq_query_start = torch.tensor([0, 5, 5, 6, 8], dtype=torch.int32)   # 5, 0, 1, 2 queries
    _gate(run_decode(w, DEV), oracle_decode(w), label=w.name)


def test_null_adapters_reduce_to_plain_attention(variant):
    """b_k = b_v = NULL is the fully shared cache: equals the oracle with B = 0."""
    w = W.config(2, shrink=8)
    dw = DeviceWorkload(w, DEV)
    dw.alloc_workspace()
    dw.b_k = None
    dw.b_v = None
    dw.decode()
    torch.cuda.synchronize()
    w.b_k.zero_()
    w.b_v.zero_()
    _gate(dw.out.to(torch.float64).cpu().numpy(), oracle_decode(w), label="null adapters")


@pytest.mark.parametrize("kind", ["decode_contiguous", "decode_paged", "prefill_contiguous", "prefill_r64"])
def test_value_only_adapters(variant, kind):
    """b_k = NULL with b_v present: the paper's main setting (keys fully shared, LoRA on the
    value side only, Sec. 3.2).  Equals the oracle with B_K = 0."""
    if kind == "decode_contiguous":
        w = W.config(2, shrink=8)
    elif kind == "decode_paged":
        w = W.make_paged("value_only_paged", seed=79, seq_lens=[5, 64, 333, 1500], agents_per_seq=3, n_adapters=4,
                         n_q_heads=14, n_kv_heads=2, head_dim=128, rank=32, d_model=None, b_std=0.05)
    elif kind == "prefill_contiguous":
        w = W.make_contiguous("value_only_prefill", "prefill", seed=80, n_agents=1, n_q_heads=8, n_kv_heads=2,
                              head_dim=128, rank=16, n=700, n_new=300, d_model=None, b_std=0.05)
    else:
        w = W.make_contiguous("value_only_prefill_r64", "prefill", seed=81, n_agents=1, n_q_heads=4, n_kv_heads=4,
                              head_dim=64, rank=64, n=391, n_new=391, d_model=None, b_std=0.05)
    dw = DeviceWorkload(w, DEV)
    dw.alloc_workspace()
    dw.b_k = None
    dw.out.fill_(float("nan"))
    if w.kind == "decode":
        dw.decode()
    else:
        dw.prefill()
    torch.cuda.synchronize()
    w.b_k.zero_()
    ref = oracle_decode(w) if w.kind == "decode" else oracle_prefill(w)
    _gate(dw.out.to(torch.float64).cpu().numpy(), ref, label=kind)


def test_deterministic_and_inputs_untouched(variant):
    w = W.config(2, shrink=4)
    dw = DeviceWorkload(w, DEV)
    dw.alloc_workspace()
    dw.decode()
    torch.cuda.synchronize()
    first = dw.out.clone()
    dw.workspace.fill_(0xFF)
    dw.out.zero_()
    dw.decode()
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16), dw.out.view(torch.int16))
    assert torch.equal(dw.k_base.cpu(), w.k_base) and torch.equal(dw.l.cpu(), w.l)
    assert torch.equal(dw.q.cpu(), w.q) and torch.equal(dw.b_v.cpu(), w.b_v)


def test_split_size_does_not_change_result_beyond_rounding():
    w = W.config(2, shrink=4)
    ref = oracle_decode(w)
    try:
        for keys in (64, 192, 1024, 1 << 20):
            lra.lra_set_decode_split_keys(keys)
            _gate(run_decode(w, DEV), ref, label=f"split_keys={keys}")
    finally:
        lra.lra_set_decode_split_keys(0)


def test_runs_on_a_side_stream():
    w = W.config(2, shrink=8)
    dw = DeviceWorkload(w, DEV)
    dw.alloc_workspace()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        dw.decode(s)
    s.synchronize()
    _gate(dw.out.to(torch.float64).cpu().numpy(), oracle_decode(w), label="side stream")


def test_machine_probes_run():
    """The benchmark's two probe kernels complete, leave their sink alone and report their work."""
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    buf = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    lra.lra_probe_stream_read(buf, sink)
    lra.lra_probe_stream_read(buf[:1000], sink)       # a length that leaves a remainder pass
    flops = lra.lra_probe_mfma_bf16(100, sink)
    assert lra.lra_probe_mfma_bf16(100, sink, random_operands=True) == flops
    torch.cuda.synchronize()
    assert flops == 512 * 4 * 4 * 100 * 2 * 32 * 32 * 16
    assert int(sink.abs().sum()) == 0


@pytest.mark.parametrize("case", [
    # sequences, agents per sequence, Hq, Hkv, d, r  -> rows = sequences x agents x Hq
    (40, 8, 4, 1, 128, 16),     # 1280 rows, group of 4
    (30, 5, 14, 2, 64, 24),     # 2100 rows, group of 7 (two workgroups of four waves per kv head, one wave idle)
    (20, 4, 16, 1, 128, 64),    # 1280 rows, group of 16
    (70, 3, 5, 5, 64, 8),       # 1050 rows, group of 1 (three of four waves idle)
], ids=lambda c: "s%d_a%d_hq%d_hkv%d_d%d_r%d" % c)
def test_many_rows_take_the_wave_per_row_merge(case):
    """Calls with 1024 rows or more end with the wave-per-row form of the merge kernel: ragged paged batches
    with many short sequences (so that most key shares of most rows are empty), every group size class."""
    n_seqs, agents, hq, hkv, d, r = case
    rng = np.random.default_rng(sum(case))
    lens = [int(x) for x in rng.integers(1, 700, size=n_seqs)]
    w = W.make_paged("many_rows", seed=4000 + sum(case), seq_lens=lens, agents_per_seq=agents, n_adapters=3,
                     n_q_heads=hq, n_kv_heads=hkv, head_dim=d, rank=r, d_model=None, b_std=0.05)
    assert w.q.shape[0] * hq >= 1024
    prev = lra.lra_set_decode_split_keys(128)   # up to six shares per sequence
    try:
        got = run_decode(w, DEV)
    finally:
        lra.lra_set_decode_split_keys(prev)
    _gate(got, oracle_decode(w), label=w.name)


def test_many_rows_fp32_and_vector_alu_partials():
    """The wave-per-row merge behind the vector-ALU partial kernels: fp32 (held to 2e-5), and bf16 with the
    vector-ALU kernels forced."""
    lens = [int(x) for x in np.random.default_rng(77).integers(1, 400, size=36)]
    for dtype, variant, fp32 in ((torch.float32, 0, True), (torch.bfloat16, 1, False)):
        w = W.make_paged("many_rows_valu", seed=4200, dtype=dtype, seq_lens=lens, agents_per_seq=4, n_adapters=3,
                         n_q_heads=8, n_kv_heads=2, head_dim=64, rank=12, d_model=None, b_std=0.05)
        assert w.q.shape[0] * 8 >= 1024
        prev = lra.lra_set_kernel_variant(variant)
        try:
            got = run_decode(w, DEV)
        finally:
            lra.lra_set_kernel_variant(prev)
        _gate(got, oracle_decode(w), fp32=fp32, label=f"{w.name} {dtype}")


def test_prefill_with_shared_key_tiles_and_many_rows():
    """64 new tokens x 16 q heads = 1024 rows, key tiles shared by 4 workgroups: the wave-per-row merge after the
    tile-walking prefill kernel."""
    w = W.make_contiguous("pf_many_rows", "prefill", seed=4100, n_agents=1, n_q_heads=16, n_kv_heads=4, head_dim=128,
                          rank=16, n=1500, n_new=64, d_model=None, b_std=0.05)
    prev_s, prev_p = lra.lra_set_short_prefill(0), lra.lra_set_prefill_splits(4)
    try:
        got = run_prefill(w, DEV)
    finally:
        lra.lra_set_short_prefill(prev_s)
        lra.lra_set_prefill_splits(prev_p)
    _gate(got, oracle_prefill(w), label=w.name)


def test_adapter_ids_outside_the_table_are_clamped(variant):
    """query_adapter is device data the host cannot check: every kernel keeps an id inside [0, n_adapters) by
    clamping, so a bad id gives the result of the nearest valid adapter and no read outside B_K / B_V."""
    w = W.make_contiguous("bad_ids", "decode", seed=88, n_agents=5, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16,
                          n=700, d_model=None, b_std=0.05)
    good = w.query_adapter.clone()
    bad = good.clone()
    bad[1], bad[3] = 99, -7                       # clamp to the last and to the first adapter
    good[1], good[3] = w.n_adapters - 1, 0
    w.query_adapter = bad
    got = run_decode(w, DEV)
    w.query_adapter = good
    _gate(got, oracle_decode(w), label="clamped adapter ids")
