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
