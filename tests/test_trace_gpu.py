"""The emulated agent-iteration trace (App. C.5: 17 agent steps, each a prefill of P_k context tokens
followed by G_k generated tokens, three adapters by role) walked end to end on ONE growing cache through
the C ABI: lra_cache_append writes the rows of the new tokens, lra_attn_prefill attends for the step's
context tokens, then every generated token is appended and attended by lra_attn_decode.

The oracle checks, on the cache the producer wrote (read back from the device at that point of the
walk): the output of every prefill call and of the first and the last decode call of every step; and at
the end the whole cache against the oracle's projection of all hidden states.  L_ctx = 256 (1936 tokens,
297 attention calls).  Same gate as everywhere: relative L2 <= 5e-3, max-abs <= 2e-2."""
import numpy as np
import pytest
import torch

import bench_trace
import oracle
import paper_2602_01053_amd as lra
from tests.harness import MAX_ABS_TOL, REL_L2_TOL, errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HQ, HKV, D, R, D_MODEL = 32, 8, 128, 16, 512
ROPE_THETA = 500000.0
ADAPTER = {"plan": 0, "action": 1, "reflect": 2}


def _f64(t):
    return t.to(torch.float64).cpu().numpy()


@pytest.mark.parametrize("key_rope_theta", [0.0, ROPE_THETA], ids=["plain_key_side", "rotary_key_side"])
def test_agent_iteration_trace_on_one_growing_cache(key_rope_theta):
    l_ctx = 256
    steps = [(a, l_ctx if p is None else p, g) for a, p, g in bench_trace.TRACE]
    total = sum(p + g for _, p, g in steps)
    assert len(steps) == 17 and total == 1936
    gen = torch.Generator().manual_seed(20260217)
    bf = torch.bfloat16
    x_all = torch.randn(total, D_MODEL, generator=gen).to(bf)                      # hidden states of every token
    w_cat = (torch.randn(2 * HKV * D + R, D_MODEL, generator=gen) / D_MODEL ** 0.5).to(bf)
    q_all = torch.randn(total, HQ, D, generator=gen).to(bf)                        # one query row per token
    b_std = 0.1 if key_rope_theta > 0 else 0.05
    b_k = (b_std * torch.randn(3, R, HKV * D, generator=gen)).to(bf)
    b_v = (b_std * torch.randn(3, R, HKV * D, generator=gen)).to(bf)

    sentinel = 7.0  # rows not yet appended must never be read: they hold a value that would show
    k = torch.full((total, HKV, D), sentinel, dtype=bf, device=DEV)
    v = torch.full((total, HKV, D), sentinel, dtype=bf, device=DEV)
    l = torch.full((total, R), sentinel, dtype=bf, device=DEV)
    xd, wd, qd, bkd, bvd = x_all.to(DEV), w_cat.to(DEV), q_all.to(DEV), b_k.to(DEV), b_v.to(DEV)
    lens = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = torch.empty(max(p for _, p, _ in steps), HQ, D, dtype=bf, device=DEV)
    qstart = torch.tensor([0, 1], dtype=torch.int32, device=DEV)
    adapters_dev = torch.tensor([0, 1, 2], dtype=torch.int32, device=DEV)
    shape = lra.make_shape(qd[:1], HKV, R, 0.0, key_rope_theta)
    scale = D ** -0.5
    fb_k, fb_v = _f64(b_k), _f64(b_v)

    def cache_of(n):
        return lra.make_cache(k, v, l, lens, n, None)

    held = {"t": torch.empty(256, dtype=torch.uint8, device=DEV)}

    def workspace(nbytes):
        if nbytes > held["t"].numel():
            torch.cuda.synchronize()
            held["t"] = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        return held["t"]

    def host_cache(n):
        return _f64(k[:n]), _f64(v[:n]), _f64(l[:n])

    worst = 0.0
    checked = 0
    n = 0
    for step, (agent, n_pre, n_gen) in enumerate(steps):
        a = ADAPTER[agent]
        # ---- context tokens of the step: append, then causal prefill ----
        n += n_pre
        lens.fill_(n)
        c = cache_of(n)
        lra.lra_cache_append(shape, c, wd, ROPE_THETA, xd[n - n_pre:n], 0)
        ws = workspace(lra.lra_workspace_bytes(shape, c, 1, 1, n_pre))
        out.fill_(float("nan"))
        lra.lra_attn_prefill(shape, c, bkd, bvd, 3, qd[n - n_pre:n], 0, a, out[:n_pre], ws)
        torch.cuda.synchronize()
        kb, vb, lr = host_cache(n)
        ref = oracle.prefill(_f64(q_all[n - n_pre:n]), kb, vb, lr, fb_k[a], fb_v[a], n=n, scale=scale,
                             key_rope_theta=key_rope_theta)
        rel, mx = errors(_f64(out[:n_pre]), ref)
        print(f"step {step + 1:2d} {agent:7s} prefill {n_pre:4d} tokens at n = {n:4d}: relL2={rel:.2e} maxabs={mx:.2e}", flush=True)
        assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL, (step, "prefill", rel, mx)
        worst, checked = max(worst, rel), checked + 1
        # ---- generated tokens: append one, decode one ----
        for g in range(n_gen):
            n += 1
            lens.fill_(n)
            c = cache_of(n)
            lra.lra_cache_append(shape, c, wd, ROPE_THETA, xd[n - 1:n], 0)
            ws = workspace(lra.lra_workspace_bytes(shape, c, 1, 1, 0))
            lra.lra_attn_decode(shape, c, bkd, bvd, 3, qd[n - 1:n], adapters_dev[a:a + 1], qstart, 1, out[:1], ws)
            if g in (0, n_gen - 1):
                torch.cuda.synchronize()
                kb, vb, lr = host_cache(n)
                ref = oracle.decode(_f64(q_all[n - 1:n]), kb, vb, lr, fb_k, fb_v, [a], [0, 1], [n], scale,
                                    key_rope_theta=key_rope_theta)
                rel, mx = errors(_f64(out[:1]), ref)
                assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL, (step, "decode", g, rel, mx)
                worst, checked = max(worst, rel), checked + 1
    assert n == total and checked == 17 * 3
    # ---- the cache itself: every row the producer wrote, against the oracle's projection ----
    torch.cuda.synchronize()
    refs = oracle.project_new_tokens(_f64(x_all), _f64(w_cat), HKV, D, R, np.arange(total), ROPE_THETA)
    for name, got, ref in zip("KVL", (k, v, l), refs):
        rel, mx = errors(_f64(got), ref)
        print(f"cache {name}: relL2={rel:.2e} maxabs={mx:.2e}", flush=True)
        assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL, (name, rel, mx)
    print(f"{checked} attention outputs checked, worst relL2 {worst:.2e}", flush=True)
