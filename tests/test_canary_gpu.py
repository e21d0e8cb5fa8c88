"""Guard bands around everything the library writes: `out` and the workspace sit in the middle of
larger allocations whose margins hold a byte pattern; after a call on a ragged paged batch, a short
prefill and a prefill with shared key tiles the margins must be untouched (NaN-filling the buffers
themselves, as the parity tests do, cannot see a write past the last row)."""
import pytest
import torch

import paper_2602_01053_amd as lra
from paper_2602_01053_amd import workloads as W
from tests.harness import MAX_ABS_TOL, REL_L2_TOL, DeviceWorkload, errors, oracle_decode, oracle_prefill

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 4096
PATTERN = 0xA5


def _guarded(nbytes):
    """(whole allocation, the 256-byte aligned view of nbytes in its middle)"""
    whole = torch.full((GUARD + nbytes + GUARD + 256,), PATTERN, dtype=torch.uint8, device=DEV)
    start = GUARD + (-(whole.data_ptr() + GUARD)) % 256
    return whole, whole[start:start + nbytes], start


def _margins_intact(whole, start, nbytes):
    return bool((whole[:start] == PATTERN).all()) and bool((whole[start + nbytes:] == PATTERN).all())


def _run_guarded(w, kind):
    dw = DeviceWorkload(w, DEV)
    need = dw.alloc_workspace()
    ws_whole, ws_view, ws_start = _guarded(max(need, 256))
    out_bytes = dw.out.numel() * dw.out.element_size()
    out_whole, out_view, out_start = _guarded(out_bytes)
    dw.workspace = ws_view[:max(need, 256)]
    dw.out = out_view.view(dw.q.dtype).view(dw.q.shape)
    dw.out.fill_(float("nan"))
    if kind == "decode":
        dw.decode()
    else:
        dw.prefill()
    torch.cuda.synchronize()
    assert _margins_intact(ws_whole, ws_start, max(need, 256)), "write outside the workspace"
    assert _margins_intact(out_whole, out_start, out_bytes), "write outside out"
    return dw.out.to(torch.float64).cpu().numpy(), need


@pytest.mark.parametrize("variant", [0, 1, 2], ids=["auto", "valu", "mfma_no_stream_form"])
def test_ragged_paged_batch_stays_inside_its_buffers(variant):
    w = W.make_paged("canary_paged", seed=611, seq_lens=[1, 15, 16, 17, 250, 1027, 4099], agents_per_seq=3, n_adapters=4,
                     n_q_heads=14, n_kv_heads=2, head_dim=128, rank=32, d_model=None, b_std=0.05)
    prev = lra.lra_set_kernel_variant(variant)
    try:
        got, need = _run_guarded(w, "decode")
    finally:
        lra.lra_set_kernel_variant(prev)
    assert need > 0
    rel, mx = errors(got, oracle_decode(w))
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


@pytest.mark.parametrize("case", [
    # n, n_new, Hq, Hkv, d, r
    (4099, 7, 32, 8, 128, 16),     # a few new tokens: split-KV path, ragged last row tile
    (3000, 200, 8, 2, 128, 16),    # key tiles of a q tile shared by several workgroups + merge
    (2000, 8, 8, 2, 128, 64),      # split-KV path with the Qt pre-pass (its output lives in the workspace)
    (513, 257, 14, 2, 128, 32),    # one kernel, no workspace: ragged last q tile
], ids=lambda c: "n%d_new%d_hq%d_hkv%d_d%d_r%d" % c)
def test_prefill_stays_inside_its_buffers(case):
    n, n_new, hq, hkv, d, r = case
    w = W.make_contiguous("canary_prefill", "prefill", seed=612 + n, n_agents=1, n_q_heads=hq, n_kv_heads=hkv,
                          head_dim=d, rank=r, n=n, n_new=n_new, d_model=None, b_std=0.05)
    got, _ = _run_guarded(w, "prefill")
    rel, mx = errors(got, oracle_prefill(w))
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


def test_contiguous_decode_with_prepass_stays_inside_its_buffers():
    """8 agents x rank 64 on one sequence: streaming form, Qt from the pre-pass kernel, exact-size workspace."""
    w = W.make_contiguous("canary_decode", "decode", seed=613, n_agents=8, n_q_heads=32, n_kv_heads=8, head_dim=128,
                          rank=64, n=3001, d_model=None, b_std=0.05)
    got, need = _run_guarded(w, "decode")
    assert need > 0
    rel, mx = errors(got, oracle_decode(w))
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


@pytest.mark.parametrize("paged", [False, True], ids=["contiguous", "paged"])
def test_rotary_prefill_key_prepass_stays_inside_its_workspace(paged):
    """Rotary key side, tile-walking prefill: the pre-pass writes the completed keys of the call's sequence into the
    workspace (contiguous: the extent of K_base; paged: the sequence's blocks in logical order, here the longest
    sequence with a partly filled last block).  Exact-size workspace between guard bands."""
    import numpy as np
    import oracle
    theta, hq, hkv, d, r, n_new = 500000.0, 8, 2, 128, 16, 150
    gen = torch.Generator().manual_seed(614)
    q = torch.randn(n_new, hq, d, generator=gen).to(torch.bfloat16)
    f = lambda t: t.to(torch.float64).numpy()
    if paged:
        w = W.make_paged("canary_rot_paged", seed=615, seq_lens=[40, 1003, 333], agents_per_seq=1, n_adapters=2, n_q_heads=hq,
                         n_kv_heads=hkv, head_dim=d, rank=r, d_model=None, b_std=0.1)
        seq, n = 1, 1003
        table = w.block_table.to(DEV)
        ids = w.block_table[seq].numpy()
        kb, vb = oracle.gather_paged(f(w.k_base), ids, n), oracle.gather_paged(f(w.v_base), ids, n)
        lr = oracle.lra_oracle.gather_paged_l(f(w.l), ids, n)
    else:
        w = W.make_contiguous("canary_rot", "decode", seed=616, n_agents=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, rank=r,
                              n=1003, d_model=None, b_std=0.1)
        seq, n, table = 0, 1003, None
        kb, vb, lr = f(w.k_base), f(w.v_base), f(w.l)
    qd, kd, vd, ld, bk, bv = q.to(DEV), w.k_base.to(DEV), w.v_base.to(DEV), w.l.to(DEV), w.b_k.to(DEV), w.b_v.to(DEV)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = lra.make_shape(qd, hkv, r, 0.0, theta)
    cache = lra.make_cache(kd, vd, ld, lens, max(w.seq_lens), table)
    need = lra.lra_workspace_bytes(shape, cache, 1, 1, n_new)
    assert need >= n * hkv * d * 2  # room for the completed keys
    ws_whole, ws_view, ws_start = _guarded(need)
    out = torch.full_like(qd, float("nan"))
    lra.lra_attn_prefill(shape, cache, bk, bv, 2, qd, seq, 1, out, ws_view)
    torch.cuda.synchronize()
    assert _margins_intact(ws_whole, ws_start, need), "write outside the workspace"
    ref = oracle.prefill(f(q), kb, vb, lr, f(w.b_k[1]), f(w.b_v[1]), n=n, scale=1.0 / d ** 0.5, key_rope_theta=theta)
    rel, mx = errors(out.to(torch.float64).cpu().numpy(), ref)
    assert np.isfinite(out.float().cpu().numpy()).all()
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL


@pytest.mark.parametrize("theta", [0.0, 500000.0], ids=["plain", "rotary"])
def test_base_shared_paged_batch_stays_inside_its_buffers(theta):
    """One low-rank cache per adapter over a ragged paged batch (column-block L tile; with the rotary key side one
    agent per tile): guard bands around out and the workspace, parity with the oracle evaluated query by query."""
    import numpy as np
    import oracle
    w = W.make_paged("canary_bs", seed=612, seq_lens=[1, 16, 17, 250, 1027, 2051], agents_per_seq=3, n_adapters=3,
                     n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, d_model=None, b_std=0.1 if theta > 0 else 0.05)
    gen = torch.Generator().manual_seed(613)
    pools = [w.l] + [torch.where(torch.isnan(w.l.float()), w.l.float(), torch.randn(w.l.shape, generator=gen)).to(torch.bfloat16)
                     for _ in range(2)]
    l_dev = torch.stack(pools).to(DEV)
    qd, k, v = w.q.to(DEV), w.k_base.to(DEV), w.v_base.to(DEV)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    table, bk, bv = w.block_table.to(DEV), w.b_k.to(DEV), w.b_v.to(DEV)
    qa, qs = w.query_adapter.to(DEV), w.seq_query_start.to(DEV)
    shape = lra.make_shape(qd, w.n_kv_heads, w.rank, 0.0, theta)
    cache = lra.make_cache(k, v, l_dev, lens, max(w.seq_lens), table, l_per_adapter=True)
    nq = qd.shape[0]
    need = max(lra.lra_workspace_bytes(shape, cache, nq, 3), 256)
    ws_whole, ws_view, ws_start = _guarded(need)
    out_bytes = qd.numel() * qd.element_size()
    out_whole, out_view, out_start = _guarded(out_bytes)
    out = out_view.view(qd.dtype).view(qd.shape)
    out.fill_(float("nan"))
    lra.lra_attn_decode(shape, cache, bk, bv, w.n_adapters, qd, qa, qs, 3, out, ws_view)
    torch.cuda.synchronize()
    assert _margins_intact(ws_whole, ws_start, need), "write outside the workspace"
    assert _margins_intact(out_whole, out_start, out_bytes), "write outside out"
    f = lambda t: t.to(torch.float64).numpy()
    ref = np.zeros(tuple(w.q.shape))
    starts = w.seq_query_start.numpy()
    for i in range(nq):
        a = int(w.query_adapter[i])
        t = int(np.searchsorted(starts, i, side="right") - 1)
        ref[i] = oracle.decode(f(w.q[i:i + 1]), f(w.k_base), f(w.v_base), f(pools[a]), f(w.b_k), f(w.b_v), np.array([a], dtype=np.int32),
                               np.array([0] * (t + 1) + [1] * (len(w.seq_lens) - t), dtype=np.int32), w.seq_lens, w.scale,
                               block_size=16, block_table=w.block_table.numpy(), key_rope_theta=theta)[0]
    rel, mx = errors(out.to(torch.float64).cpu().numpy(), ref)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL
