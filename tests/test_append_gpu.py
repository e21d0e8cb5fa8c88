"""Parity of the cache-append producer (lra_cache_append) against the fp64 oracle, through
the C ABI.  Bar as for the attention calls: relative L2 <= 5e-3 over every written tensor
and over every token, max-abs <= 2e-2 (outputs are O(1): x ~ N(0,1), w ~ N(0, 1/d_model))."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_01053_amd as lra
from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SENTINEL = 7.0   # value of every cache element before the call: rows that are not appended must keep it


def _inputs(seed, n_new, d_model, hkv, d, r):
    gen = torch.Generator().manual_seed(seed)
    x = torch.randn(n_new, d_model, generator=gen).to(torch.bfloat16)
    w = (torch.randn(2 * hkv * d + r, d_model, generator=gen) / d_model ** 0.5).to(torch.bfloat16)
    return x, w


def _gate(got, ref, label):
    rel, mx = errors(got, ref)
    print(f"{label}: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL, (label, rel, mx)


CASES = [
    # n (after the append), n_new, d_model, Hkv, d, r, rope_theta
    (1, 1, 64, 1, 64, 8, 10000.0),
    (200, 129, 256, 2, 128, 16, 500000.0),      # ragged token tile
    (300, 300, 512, 3, 64, 24, 10000.0),        # no old rows; Hkv*d = 192: a partly filled feature tile
    (70000, 130, 1024, 8, 128, 16, 500000.0),   # positions in the tens of thousands
    (513, 257, 4096, 8, 128, 64, 0.0),          # Llama-3-8B projection shape, keys stored unrotated
    (1000, 512, 1024, 4, 128, 32, 500000.0),
]


# few new tokens: the weight-streaming kernel (and, with it switched off, the tiled one on the same inputs)
SMALL = [
    (1, 1, 64, 1, 64, 8, 10000.0),
    (4097, 1, 4096, 8, 128, 16, 500000.0),     # a decode step at the Llama-3-8B shape
    (9, 2, 192, 2, 64, 8, 10000.0),            # matrix-vector kernel, d_model/8 = 24 pieces: lanes without one
    (31, 3, 1088, 2, 128, 24, 500000.0),       # three tokens on the four-token instantiation; 136 pieces: a ragged second round
    (40000, 4, 4096, 8, 128, 16, 500000.0),
    (50, 7, 320, 2, 64, 24, 10000.0),          # d_model/32 = 10 steps over 8 waves; rank 24: a partly filled L group
    (100, 16, 512, 2, 128, 16, 500000.0),
    (100, 17, 512, 2, 128, 40, 500000.0),
    (65000, 33, 1024, 4, 128, 16, 500000.0),
    (64, 64, 768, 3, 64, 64, 10000.0),
    (300, 150, 512, 2, 128, 16, 500000.0),     # beyond the default limit: runs streamed only when the limit is raised
    (20, 3, 128, 2, 64, 8, 0.0),               # unrotated keys on the matrix-vector kernel
    (40, 12, 256, 2, 128, 16, 0.0),            # and on the weight-streaming one
]


@pytest.mark.parametrize("skinny", [0, 64, 1 << 30], ids=["tiled", "default", "streamed"])
@pytest.mark.parametrize("case", SMALL, ids=lambda c: "n%d_new%d_dm%d_hkv%d_d%d_r%d_th%g" % c)
def test_append_few_tokens(case, skinny):
    prev = lra.lra_set_append_skinny(skinny)
    try:
        test_append_contiguous(case)
    finally:
        lra.lra_set_append_skinny(prev)


@pytest.mark.parametrize("stages", [2, 3, 4])
@pytest.mark.parametrize("case", [SMALL[0], (200, 129, 256, 2, 128, 16, 500000.0), (700, 300, 704, 3, 64, 24, 10000.0)],
                         ids=lambda c: "n%d_new%d_dm%d_hkv%d_d%d_r%d_th%g" % c)
def test_append_tiled_stage_counts(case, stages):
    """The tiled GEMM with 2, 3 and 4 LDS stages (d_model of 1, 4 and 11 steps: shorter than the ring, and ragged against it)."""
    prev_s, prev_k = lra.lra_set_append_stages(stages), lra.lra_set_append_skinny(0)
    try:
        test_append_contiguous(case)
    finally:
        lra.lra_set_append_stages(prev_s)
        lra.lra_set_append_skinny(prev_k)


@pytest.mark.parametrize("case", [SMALL[0], (200, 129, 256, 2, 128, 16, 500000.0), (700, 300, 704, 3, 64, 24, 10000.0),
                                  (66000, 515, 1024, 8, 128, 64, 500000.0), (520, 520, 512, 1, 64, 8, 10000.0),
                                  (1000, 257, 4096, 8, 128, 16, 0.0)],
                         ids=lambda c: "n%d_new%d_dm%d_hkv%d_d%d_r%d_th%g" % c)
@pytest.mark.parametrize("tile", [64, 128, 256])
def test_append_tile_sizes(case, tile):
    """Every tile size of the GEMM kernels, forced: ragged token tiles, feature regions of 64, 192 and 1024
    (a tile that is partly filled, one that straddles the K and V rows of w), rank 8 to 64."""
    prev_t, prev_k = lra.lra_set_append_tile(tile), lra.lra_set_append_skinny(0)
    try:
        test_append_contiguous(case)
    finally:
        lra.lra_set_append_tile(prev_t)
        lra.lra_set_append_skinny(prev_k)


GUARD = 4096  # bytes of a bit pattern on either side of a workspace


def _guarded_workspace(nbytes):
    """A 256-byte aligned workspace of nbytes between two guard bands; returns (workspace view, whole buffer)."""
    whole = torch.full((nbytes + 2 * GUARD,), 0xA5, dtype=torch.uint8, device=DEV)
    return whole[GUARD:GUARD + nbytes], whole


def _guards_intact(whole):
    return bool((whole[:GUARD] == 0xA5).all()) and bool((whole[-GUARD:] == 0xA5).all())


@pytest.mark.parametrize("case", CASES, ids=lambda c: "n%d_new%d_dm%d_hkv%d_d%d_r%d_th%g" % c)
def test_append_contiguous(case):
    _append_contiguous(case, False)


def _append_contiguous(case, with_workspace):
    """Runs one append on a contiguous cache against the oracle; returns the workspace bytes the library asked for."""
    n, n_new, d_model, hkv, d, r, theta = case
    x, w = _inputs(5000 + n + n_new, n_new, d_model, hkv, d, r)
    k_base = torch.full((n, hkv, d), SENTINEL, dtype=torch.bfloat16, device=DEV)
    v_base = torch.full_like(k_base, SENTINEL)
    l = torch.full((n, r), SENTINEL, dtype=torch.bfloat16, device=DEV)
    seq_lens = torch.tensor([n], dtype=torch.int32, device=DEV)
    q_like = torch.empty(1, hkv, d, dtype=torch.bfloat16, device=DEV)
    shape = lra.make_shape(q_like, hkv, r, 0.0)
    cache = lra.make_cache(k_base, v_base, l, seq_lens, n, None)
    xd, wd = x.to(DEV), w.to(DEV)
    need = 0
    if with_workspace:
        need = lra.lra_append_workspace_bytes(shape, cache, wd, theta, n_new)
        ws, whole = _guarded_workspace(max(need, 256))
        lra.lra_cache_append(shape, cache, wd, theta, xd, 0, workspace=ws)
    else:
        lra.lra_cache_append(shape, cache, wd, theta, xd, 0)
    torch.cuda.synchronize()
    if with_workspace:
        assert _guards_intact(whole)
    f = lambda t: t.to(torch.float64).cpu().numpy()
    pos = np.arange(n - n_new, n)
    k_ref, v_ref, l_ref = oracle.project_new_tokens(f(x), f(w), hkv, d, r, pos, theta)
    _gate(f(k_base)[n - n_new:], k_ref, "K rows")
    _gate(f(v_base)[n - n_new:], v_ref, "V rows")
    _gate(f(l)[n - n_new:], l_ref, "L rows")
    for t in (k_base, v_base, l):   # older rows untouched
        assert bool((t[:n - n_new] == SENTINEL).all())
    return need


SPLIT_CASES = [
    # n, n_new, d_model, Hkv, d, r, theta, parts the automatic choice takes (0: it keeps one kernel)
    (100, 17, 512, 2, 128, 16, 500000.0, 0),        # up to 32 tokens: the weight-streaming kernel
    (200, 40, 512, 2, 128, 16, 500000.0, 2),        # 8 steps of d_model: two parts of four
    (65000, 33, 1024, 4, 128, 16, 500000.0, 4),
    (64, 64, 768, 3, 64, 64, 10000.0, 2),           # 12 steps: two parts of six
    (200, 129, 256, 2, 128, 16, 500000.0, 0),       # 4 steps: too short to divide
    (700, 300, 704, 3, 64, 24, 10000.0, 0),         # 11 steps: no part count divides them
    (513, 257, 4096, 8, 128, 64, 0.0, 2),           # Llama-3-8B projection shape, r = 64, unrotated keys
    (1000, 512, 1024, 4, 128, 32, 500000.0, 2),
    (4300, 100, 4096, 8, 128, 16, 500000.0, 4),     # Llama-3-8B shape, a trace-sized chunk
    (40000, 400, 4096, 8, 128, 16, 500000.0, 2),    # ... and about the largest chunk that still divides
    (40000, 1000, 4096, 8, 128, 16, 500000.0, 0),   # more than half a chip of tiles: one kernel
    (2048, 2048, 4096, 8, 128, 16, 500000.0, 0),    # enough tiles for the chip: one kernel
    (31, 16, 4096, 8, 128, 16, 500000.0, 0),        # few tokens: the weight-streaming kernel
]


@pytest.mark.parametrize("case", SPLIT_CASES, ids=lambda c: "n%d_new%d_dm%d_hkv%d_d%d_r%d_th%g_auto%d" % c)
def test_append_split_over_d_model_automatic(case):
    """lra_cache_append with a workspace: mid-sized chunks divide d_model among several workgroups per output
    tile and finish in a second kernel.  Same oracle, same gate, guard bands around the workspace intact, and
    the workspace asked for is the size of the parts the automatic choice takes."""
    *plain, parts = case
    n, n_new, d_model, hkv, d, r, theta = plain
    need = _append_contiguous(tuple(plain), True)
    expect = parts * n_new * (2 * hkv * d + r) * 4 if parts else 0
    assert need == (expect + 255) // 256 * 256


@pytest.mark.parametrize("parts", [2, 4, 16])
@pytest.mark.parametrize("case", [(200, 129, 256, 2, 128, 16, 500000.0), (5000, 40, 1024, 2, 64, 8, 10000.0),
                                  (513, 257, 4096, 8, 128, 64, 0.0), (300, 300, 512, 3, 64, 24, 10000.0)],
                         ids=lambda c: "n%d_new%d_dm%d_hkv%d_d%d_r%d_th%g" % c)
def test_append_split_over_d_model_forced(case, parts):
    """Part counts forced through the tuning struct, down to one step of d_model per part; counts that do not
    divide the steps leave the call on one kernel (and the workspace request at 0)."""
    prev = lra.lra_set_append_k_splits(parts)
    try:
        need = _append_contiguous(case, True)
    finally:
        lra.lra_set_append_k_splits(prev)
    n, n_new, d_model, hkv, d, r, theta = case
    divides = (d_model // 64) % parts == 0
    assert (need > 0) == divides


@pytest.mark.parametrize("skinny,tile,parts", [(0, 64, 0), (0, 128, 0), (0, 256, 0), (1 << 30, 0, 0), (64, 0, 2), (64, 0, 8)],
                         ids=["tile64", "tiled", "wide", "streamed", "two_parts", "eight_parts"])
def test_append_paged_then_attend(skinny, tile, parts):
    prev, prev_t, prev_p = lra.lra_set_append_skinny(skinny), lra.lra_set_append_tile(tile), lra.lra_set_append_k_splits(parts)
    try:
        _paged_then_attend(parts > 1)
    finally:
        lra.lra_set_append_skinny(prev)
        lra.lra_set_append_tile(prev_t)
        lra.lra_set_append_k_splits(prev_p)


def _paged_then_attend(with_workspace=False):
    """Appends to two sequences of a paged cache (a last block that is partly filled, blocks in
    permuted order), checks the written rows and that nothing else moved, then runs the
    attention prefill on the appended tokens and compares it with the oracle evaluated on
    the cache the producer wrote."""
    hkv, hq, d, r, d_model, theta = 2, 8, 128, 16, 512, 500000.0
    seq_lens = [77, 300]
    n_new = [30, 130]
    bs, max_blocks = 16, 20
    num_blocks = 45
    gen = torch.Generator().manual_seed(6001)
    perm = torch.randperm(num_blocks, generator=gen).to(torch.int32)
    table = torch.stack([perm[:max_blocks], perm[max_blocks:2 * max_blocks]])
    k_pool = torch.randn(num_blocks, hkv, bs, d, generator=gen).to(torch.bfloat16)
    v_pool = torch.randn(num_blocks, hkv, bs, d, generator=gen).to(torch.bfloat16)
    l_pool = torch.randn(num_blocks, bs, r, generator=gen).to(torch.bfloat16)
    kd, vd, ld = k_pool.to(DEV), v_pool.to(DEV), l_pool.to(DEV)
    lens_d = torch.tensor(seq_lens, dtype=torch.int32, device=DEV)
    table_d = table.to(DEV)
    q_like = torch.empty(1, hq, d, dtype=torch.bfloat16, device=DEV)
    shape = lra.make_shape(q_like, hkv, r, 0.0)
    cache = lra.make_cache(kd, vd, ld, lens_d, max(seq_lens), table_d)
    f = lambda t: t.to(torch.float64).cpu().numpy()
    k_exp, v_exp, l_exp = f(k_pool).copy(), f(v_pool).copy(), f(l_pool).copy()
    w = None
    for s in range(2):
        x, w = _inputs(6100 + s, n_new[s], d_model, hkv, d, r)
        if with_workspace:
            wd = w.to(DEV)
            need = lra.lra_append_workspace_bytes(shape, cache, wd, theta, n_new[s])
            assert need > 0
            ws, whole = _guarded_workspace(need)
            lra.lra_cache_append(shape, cache, wd, theta, x.to(DEV), s, workspace=ws)
            torch.cuda.synchronize()
            assert _guards_intact(whole)
        else:
            lra.lra_cache_append(shape, cache, w.to(DEV), theta, x.to(DEV), s)
        torch.cuda.synchronize()
        pos = np.arange(seq_lens[s] - n_new[s], seq_lens[s])
        k_ref, v_ref, l_ref = oracle.project_new_tokens(f(x), f(w), hkv, d, r, pos, theta)
        ids = table[s].numpy()
        got_k = oracle.gather_paged(f(kd), ids, seq_lens[s])[seq_lens[s] - n_new[s]:]
        got_v = oracle.gather_paged(f(vd), ids, seq_lens[s])[seq_lens[s] - n_new[s]:]
        got_l = oracle.lra_oracle.gather_paged_l(f(ld), ids, seq_lens[s])[seq_lens[s] - n_new[s]:]
        _gate(got_k, k_ref, f"paged K rows seq {s}")
        _gate(got_v, v_ref, f"paged V rows seq {s}")
        _gate(got_l, l_ref, f"paged L rows seq {s}")
        # everything except the appended rows is bit-identical to before
        oracle.scatter_paged(k_exp, ids, seq_lens[s] - n_new[s], got_k)
        oracle.scatter_paged(v_exp, ids, seq_lens[s] - n_new[s], got_v)
        oracle.scatter_paged_l(l_exp, ids, seq_lens[s] - n_new[s], got_l)
        np.testing.assert_array_equal(f(kd), k_exp)
        np.testing.assert_array_equal(f(vd), v_exp)
        np.testing.assert_array_equal(f(ld), l_exp)
    # attention over the cache the producer wrote (sequence 1, its 130 new tokens)
    s = 1
    gen = torch.Generator().manual_seed(6200)
    q = torch.randn(n_new[s], hq, d, generator=gen).to(torch.bfloat16)
    b_k = (0.05 * torch.randn(2, r, hkv * d, generator=gen)).to(torch.bfloat16)
    b_v = (0.05 * torch.randn(2, r, hkv * d, generator=gen)).to(torch.bfloat16)
    qd = q.to(DEV)
    out = torch.full_like(qd, float("nan"))
    ws = torch.empty(max(lra.lra_workspace_bytes(shape, cache, 1, 1, n_new[s]), 256), dtype=torch.uint8, device=DEV)
    lra.lra_attn_prefill(shape, cache, b_k.to(DEV), b_v.to(DEV), 2, qd, s, 1, out, ws)
    torch.cuda.synchronize()
    ids = table[s].numpy()
    kb = oracle.gather_paged(f(kd), ids, seq_lens[s])
    vb = oracle.gather_paged(f(vd), ids, seq_lens[s])
    lr = oracle.lra_oracle.gather_paged_l(f(ld), ids, seq_lens[s])
    ref = oracle.prefill(f(q), kb, vb, lr, f(b_k[1]), f(b_v[1]), n=seq_lens[s], scale=1.0 / d ** 0.5)
    _gate(f(out), ref, "attention over the appended cache")


def test_append_rejects_what_it_cannot_do():
    hkv, d, r = 2, 128, 16
    k_base = torch.zeros(64, hkv, d, dtype=torch.bfloat16, device=DEV)
    l = torch.zeros(64, r, dtype=torch.bfloat16, device=DEV)
    seq_lens = torch.tensor([64], dtype=torch.int32, device=DEV)
    shape = lra.make_shape(torch.empty(1, hkv, d, dtype=torch.bfloat16, device=DEV), hkv, r, 0.0)
    cache = lra.make_cache(k_base, k_base.clone(), l, seq_lens, 64, None)
    w = torch.zeros(2 * hkv * d + r, 96, dtype=torch.bfloat16, device=DEV)   # d_model not a multiple of 64
    x = torch.zeros(4, 96, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(lra.LraError) as e:
        lra.lra_cache_append(shape, cache, w, 10000.0, x, 0)
    assert e.value.status == 4
    w = torch.zeros(2 * hkv * d + r, 128, dtype=torch.bfloat16, device=DEV)
    x = torch.zeros(65, 128, dtype=torch.bfloat16, device=DEV)              # more new tokens than the cache holds
    with pytest.raises(lra.LraError) as e:
        lra.lra_cache_append(shape, cache, w, 10000.0, x, 0)
    assert e.value.status == 2


@pytest.mark.parametrize("n_new,prior", [(2048, 16384), (16384, 0), (1, 40000)], ids=["2048_after_16384", "16384_from_empty", "decode_step"])
def test_append_llama3_8b_full_size_sampled_rows(n_new, prior):
    """The benchmark's configuration (d_model 4096 -> 8 kv heads x 128 + rank 16, rotary base 500000) in the
    launch shape bench.py times; the oracle evaluates a sample of the new tokens (rows are independent)."""
    hkv, d, r, dm, theta = 8, 128, 16, 4096, 500000.0
    n = prior + n_new
    x, w = _inputs(7000 + n_new, n_new, dm, hkv, d, r)
    k_base = torch.full((n, hkv, d), SENTINEL, dtype=torch.bfloat16, device=DEV)
    v_base = torch.full_like(k_base, SENTINEL)
    l = torch.full((n, r), SENTINEL, dtype=torch.bfloat16, device=DEV)
    seq_lens = torch.tensor([n], dtype=torch.int32, device=DEV)
    shape = lra.make_shape(torch.empty(1, hkv, d, dtype=torch.bfloat16, device=DEV), hkv, r, 0.0)
    cache = lra.make_cache(k_base, v_base, l, seq_lens, n, None)
    lra.lra_cache_append(shape, cache, w.to(DEV), theta, x.to(DEV), 0)
    torch.cuda.synchronize()
    rng = np.random.default_rng(n_new)
    rows = np.unique(np.concatenate([[0, n_new - 1], rng.integers(0, n_new, size=min(96, n_new))]))
    f = lambda t: t.to(torch.float64).cpu().numpy()
    k_ref, v_ref, l_ref = oracle.project_new_tokens(f(x[rows]), f(w), hkv, d, r, prior + rows, theta)
    _gate(f(k_base[prior + rows]), k_ref, "K rows")
    _gate(f(v_base[prior + rows]), v_ref, "V rows")
    _gate(f(l[prior + rows]), l_ref, "L rows")
    if prior:
        assert bool((k_base[:prior] == SENTINEL).all()) and bool((l[:prior] == SENTINEL).all())


@pytest.mark.parametrize("n_new", [1, 5, 200, 2048], ids=lambda n: f"new{n}")
def test_append_writes_nothing_when_the_device_length_exceeds_the_bound(n_new):
    """max_seq_len sizes the caches: a device-side sequence length beyond it cannot be honoured, and the call must
    leave every cache row as it was (all four kernels: matrix-vector, weight-streaming, tiled, wide tile)."""
    hkv, d, r, d_model, rows = 2, 128, 16, 256, 2100
    x, w = _inputs(900 + n_new, n_new, d_model, hkv, d, r)
    k = torch.full((rows, hkv, d), SENTINEL, dtype=torch.bfloat16, device=DEV)
    v = torch.full_like(k, SENTINEL)
    l = torch.full((rows, r), SENTINEL, dtype=torch.bfloat16, device=DEV)
    lens = torch.tensor([rows + 50], dtype=torch.int32, device=DEV)       # longer than the cache can hold
    shape = lra.make_shape(torch.empty(1, hkv, d, dtype=torch.bfloat16, device=DEV), hkv, r, 0.0)
    wd, xd = w.to(DEV), x.to(DEV)   # referenced until the synchronisation: the call only enqueues
    lra.lra_cache_append(shape, lra.make_cache(k, v, l, lens, rows, None), wd, 500000.0, xd, 0)
    torch.cuda.synchronize()
    for name, t in (("K", k), ("V", v), ("L", l)):
        assert bool((t == SENTINEL).all()), f"{name} rows were overwritten"
