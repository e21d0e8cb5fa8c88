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
