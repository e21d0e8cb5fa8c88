"""The library's calls under HIP graph capture (what bench.py times and what a serving loop does): every entry
point is captured once on a side stream and replayed several times, with the program's own eager work and
synchronisations between the replays and with new inputs written into the captured buffers before each replay;
every replay must reproduce, bit for bit, what the same call gives eagerly on the same inputs (the kernels are
deterministic), and one of them is held to the oracle as well."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_01053_amd as lra
from paper_2602_01053_amd import workloads as W
from paper_2602_01053_amd.runner import DeviceWorkload
from tests.harness import MAX_ABS_TOL, REL_L2_TOL, _f64, errors, oracle_decode

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _replay_against_eager(call, refresh, outputs, replays=3):
    """call(stream): enqueue the library call(s); refresh(i): write replay i's inputs into the captured
    buffers; outputs(): the tensors the call writes.  Returns the outputs of the last replay."""
    side = torch.cuda.Stream()
    refresh(0)
    with torch.cuda.stream(side):
        call(side)                      # warm-up outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(side)
    last = None
    for i in range(replays):
        refresh(i)
        torch.cuda.synchronize()
        call(None)                      # eager, on the current stream
        torch.cuda.synchronize()
        eager = [t.clone() for t in outputs()]
        for t in outputs():
            t.fill_(float("nan")) if t.is_floating_point() else t.zero_()
        scratch = torch.randn(1 << 16, device=DEV).sum()   # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outputs(), eager):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), f"replay {i} differs from the eager call"
        last = [t.clone() for t in outputs()]
        del scratch
    return last


def _decode_case(w):
    dw = DeviceWorkload(w, DEV)
    dw.alloc_workspace()
    gen = torch.Generator().manual_seed(77)
    qs = [w.q] + [torch.randn(w.q.shape, generator=gen).to(w.q.dtype) for _ in range(2)]

    def refresh(i):
        dw.q.copy_(qs[i].to(DEV))

    last = _replay_against_eager(lambda st: dw.decode(st), refresh, lambda: [dw.out])
    return dw, qs, last


def test_decode_streaming_form_replays():
    w = W.make_contiguous("graph_dec", "decode", seed=401, n_agents=4, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=16,
                          n=3000, n_new=1, d_model=None)
    dw, qs, last = _decode_case(w)
    w.q = qs[2]
    rel, mx = errors(_f64(last[0].cpu()), oracle_decode(w))
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


def test_decode_with_qt_prepass_replays():
    w = W.make_contiguous("graph_dec_r64", "decode", seed=402, n_agents=8, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=64,
                          n=2100, n_new=1, d_model=None)
    _decode_case(w)


def test_decode_paged_batch_replays():
    w = W.make_paged("graph_paged", seed=403, seq_lens=[5, 64, 700, 1500], agents_per_seq=3, n_adapters=3,
                     n_q_heads=28, n_kv_heads=4, head_dim=128, rank=32, d_model=None)
    _decode_case(w)


def test_decode_static_workspace_replays():
    w = W.make_contiguous("graph_static", "decode", seed=404, n_agents=4, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=16,
                          n=1500, n_new=1, d_model=None)
    dw = DeviceWorkload(w, DEV)
    gen = torch.Generator().manual_seed(78)
    qs = [w.q] + [torch.randn(w.q.shape, generator=gen).to(w.q.dtype) for _ in range(2)]

    def call(st):
        lra.lra_attn_decode_static(dw.shape, dw.cache, dw.b_k, dw.b_v, w.n_adapters, dw.q, dw.query_adapter,
                                   dw.seq_query_start, dw.max_queries_per_seq, dw.out, st)

    call(None)   # the first call on a device looks up the static buffer: outside any capture
    torch.cuda.synchronize()
    _replay_against_eager(call, lambda i: dw.q.copy_(qs[i].to(DEV)), lambda: [dw.out])


@pytest.mark.parametrize("theta", [0.0, 500000.0], ids=["plain_key_side", "rotary_key_side_with_key_prepass"])
def test_prefill_replays(theta):
    w = W.make_contiguous("graph_pre", "prefill", seed=405, n_agents=1, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16,
                          n=900, n_new=300, d_model=None, b_std=0.1)
    dw = DeviceWorkload(w, DEV, key_rope_theta=theta)
    dw.alloc_workspace()
    gen = torch.Generator().manual_seed(79)
    qs = [w.q] + [torch.randn(w.q.shape, generator=gen).to(w.q.dtype) for _ in range(2)]
    last = _replay_against_eager(lambda st: dw.prefill(st), lambda i: dw.q.copy_(qs[i].to(DEV)), lambda: [dw.out])
    a = int(w.query_adapter[0])
    ref = oracle.prefill(_f64(qs[2]), _f64(w.k_base), _f64(w.v_base), _f64(w.l), _f64(w.b_k[a]), _f64(w.b_v[a]),
                         n=w.seq_lens[0], scale=w.scale, key_rope_theta=theta)
    rel, mx = errors(_f64(last[0].cpu()), ref)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


@pytest.mark.parametrize("n_new", [1, 100], ids=["one_token", "split_over_d_model"])
def test_append_then_decode_replays(n_new):
    """lra_cache_append followed by lra_attn_decode on the cache it wrote, as one captured sequence."""
    hkv, hq, d, r, dm, n = 2, 8, 128, 16, 1024, 700
    gen = torch.Generator().manual_seed(80)
    bf = torch.bfloat16
    rn = lambda *sh, std=1.0: (std * torch.randn(*sh, generator=gen)).to(bf)
    k, v, l = rn(n, hkv, d).to(DEV), rn(n, hkv, d).to(DEV), rn(n, r).to(DEV)
    w_cat = rn(2 * hkv * d + r, dm, std=dm ** -0.5).to(DEV)
    xs = [rn(n_new, dm) for _ in range(3)]
    x = xs[0].to(DEV)
    q = rn(2, hq, d).to(DEV)
    b_k, b_v = rn(2, r, hkv * d, std=0.05).to(DEV), rn(2, r, hkv * d, std=0.05).to(DEV)
    lens = torch.tensor([n], dtype=torch.int32, device=DEV)
    adapters = torch.tensor([0, 1], dtype=torch.int32, device=DEV)
    qstart = torch.tensor([0, 2], dtype=torch.int32, device=DEV)
    out = torch.empty_like(q)
    shape = lra.make_shape(q, hkv, r, 0.0)
    cache = lra.make_cache(k, v, l, lens, n, None)
    ws = torch.empty(max(lra.lra_workspace_bytes(shape, cache, 2, 2, 0), 256), dtype=torch.uint8, device=DEV)
    aws_bytes = lra.lra_append_workspace_bytes(shape, cache, w_cat, 500000.0, n_new)
    assert (aws_bytes > 0) == (n_new == 100)
    aws = torch.empty(max(aws_bytes, 256), dtype=torch.uint8, device=DEV)

    def call(st):
        lra.lra_cache_append(shape, cache, w_cat, 500000.0, x, 0, st, workspace=aws)
        lra.lra_attn_decode(shape, cache, b_k, b_v, 2, q, adapters, qstart, 2, out, ws, st)

    # (only the appended rows are outputs: the rest of the caches is input to the decode call)
    _replay_against_eager(call, lambda i: x.copy_(xs[i].to(DEV)), lambda: [out, k[n - n_new:], v[n - n_new:], l[n - n_new:]])
