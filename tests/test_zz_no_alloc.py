"""lra_attn_decode_static (the decode entry point that allocates nothing: its split-KV workspace is a
buffer inside the library's device image) against lra_attn_decode, through the C ABI.  Same kernels,
same launch plan: the outputs must agree bit for bit, and each is also held to the oracle's gate.
Two calls in a row share the buffer, the second on a smaller input, so anything the first call left
behind that the second one wrongly read would show."""
import numpy as np
import pytest
import torch

import paper_2602_01053_amd as lra
from paper_2602_01053_amd import workloads as W
from tests.harness import MAX_ABS_TOL, REL_L2_TOL, DeviceWorkload, errors, oracle_decode

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(w):
    dw = DeviceWorkload(w, DEV)
    need = dw.alloc_workspace()
    assert 0 < need <= lra.binding.STATIC_WORKSPACE_BYTES
    dw.out.fill_(float("nan"))
    dw.decode()
    torch.cuda.synchronize()
    want = dw.out.clone()
    dw.out.fill_(float("nan"))
    lra.lra_attn_decode_static(dw.shape, dw.cache, dw.b_k, dw.b_v, w.n_adapters, dw.q, dw.query_adapter,
                               dw.seq_query_start, dw.max_queries_per_seq, dw.out)
    torch.cuda.synchronize()
    return want, dw.out.clone()


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def test_static_workspace_decode_two_calls_in_a_row():
    big = W.make_paged("no_alloc_big", seed=501, seq_lens=[2500, 77, 1300, 4099], agents_per_seq=3, n_adapters=3,
                       n_q_heads=14, n_kv_heads=2, head_dim=128, rank=32, d_model=None, b_std=0.05)
    small = W.make_contiguous("no_alloc_small", "decode", seed=502, n_agents=2, n_q_heads=8, n_kv_heads=2,
                              head_dim=128, rank=16, n=333, d_model=None, b_std=0.05)
    for w in (big, small):           # the second, smaller call finds the first one's states in the buffer
        want, got = _both(w)
        print(f"{w.name}: static-workspace call done", flush=True)
        assert torch.equal(_bits(want), _bits(got)), w.name
        rel, mx = errors(got.to(torch.float64).cpu().numpy(), oracle_decode(w))
        print(f"{w.name}: relL2={rel:.3e} maxabs={mx:.3e}", flush=True)
        assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


def test_static_workspace_decode_fp32_and_full_config_2():
    for w in (W.config(2), W.config(1)):
        want, got = _both(w)
        assert torch.equal(_bits(want), _bits(got)), w.name


def test_static_workspace_decode_rejects_what_does_not_fit():
    """A call whose partial states exceed the buffer is refused before anything is enqueued."""
    q = torch.zeros(4096, 32, 128, dtype=torch.bfloat16, device=DEV)
    k = torch.zeros(8192, 8, 128, dtype=torch.bfloat16, device=DEV)
    l = torch.zeros(8192, 16, dtype=torch.bfloat16, device=DEV)
    b = torch.zeros(1, 16, 1024, dtype=torch.bfloat16, device=DEV)
    lens = torch.tensor([8192], dtype=torch.int32, device=DEV)
    qa = torch.zeros(4096, dtype=torch.int32, device=DEV)
    sqs = torch.tensor([0, 4096], dtype=torch.int32, device=DEV)
    shape, cache = lra.make_shape(q, 8, 16), lra.make_cache(k, k, l, lens, 8192)
    assert lra.lra_workspace_bytes(shape, cache, 4096, 4096) > lra.binding.STATIC_WORKSPACE_BYTES
    out = torch.full_like(q, 7.0)
    with pytest.raises(lra.LraError) as err:
        lra.lra_attn_decode_static(shape, cache, b, b, 1, q, qa, sqs, 4096, out)
    assert err.value.status == 5
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
