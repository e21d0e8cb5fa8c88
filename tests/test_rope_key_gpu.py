"""The rotary key side (lra_shape.key_rope_theta > 0: K_j = K_base,j + RoPE_j(L_j B_K), the
setting of the paper's qkvo ablation, App. D.1) against the oracle, through the C ABI:
decode and prefill, contiguous and paged, bf16 and fp32.  Same gate as everywhere
(relative L2 <= 5e-3, max-abs <= 2e-2); fp32 is also held to 1e-4."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01053_amd import workloads as W
from paper_2602_01053_amd.runner import DeviceWorkload
from tests.harness import MAX_ABS_TOL, REL_L2_TOL, _f64, errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(w, theta):
    dw = DeviceWorkload(w, DEV, key_rope_theta=theta)
    dw.alloc_workspace()
    dw.out.fill_(float("nan"))
    if w.kind == "decode":
        dw.decode()
    else:
        dw.prefill()
    torch.cuda.synchronize()
    return dw.out.to(torch.float64).cpu().numpy()


def _oracle(w, theta):
    if w.kind == "decode":
        return oracle.decode(_f64(w.q), _f64(w.k_base), _f64(w.v_base), _f64(w.l), _f64(w.b_k), _f64(w.b_v),
                             w.query_adapter.numpy(), w.seq_query_start.numpy(), w.seq_lens, w.scale,
                             block_size=w.block_size,
                             block_table=None if w.block_table is None else w.block_table.numpy(),
                             key_rope_theta=theta)
    a = int(w.query_adapter[0])
    return oracle.prefill(_f64(w.q), _f64(w.k_base), _f64(w.v_base), _f64(w.l), _f64(w.b_k[a]), _f64(w.b_v[a]),
                          n=w.seq_lens[0], scale=w.scale, key_rope_theta=theta)


def _cases():
    yield "decode_llama_shape", W.make_contiguous("rope_dec", "decode", seed=301, n_agents=4, n_q_heads=32, n_kv_heads=8,
                                                  head_dim=128, rank=16, n=1500, n_new=1, d_model=None, b_std=0.1), 500000.0, None
    yield "decode_d64_r24", W.make_contiguous("rope_dec64", "decode", seed=302, n_agents=3, n_q_heads=8, n_kv_heads=2,
                                              head_dim=64, rank=24, n=333, n_new=1, d_model=None, b_std=0.1), 10000.0, None
    yield "decode_paged", W.make_paged("rope_paged", seed=303, seq_lens=[5, 64, 700], agents_per_seq=2, n_adapters=3,
                                       n_q_heads=8, n_kv_heads=2, head_dim=128, rank=8, d_model=None, b_std=0.1), 500000.0, None
    yield "prefill", W.make_contiguous("rope_pre", "prefill", seed=304, n_agents=1, n_q_heads=8, n_kv_heads=2,
                                       head_dim=128, rank=16, n=400, n_new=150, d_model=None, b_std=0.1), 500000.0, None
    yield "decode_fp32", W.make_contiguous("rope_f32", "decode", seed=305, dtype=torch.float32, n_agents=2, n_q_heads=4,
                                           n_kv_heads=2, head_dim=64, rank=5, n=200, n_new=1, d_model=None, b_std=0.1), 10000.0, 1e-4


@pytest.mark.parametrize("name,w,theta,tight", list(_cases()), ids=[c[0] for c in _cases()])
def test_rotary_key_side(name, w, theta, tight):
    got = _run(w, theta)
    ref = _oracle(w, theta)
    rel, mx = errors(got, ref)
    plain = _oracle(w, 0.0)
    moved = np.linalg.norm(ref - plain) / np.linalg.norm(ref)
    print(f"{name}: relL2={rel:.3e} maxabs={mx:.3e}; the rotation moves the output by {moved:.3e}", flush=True)
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL
    if tight:
        assert rel <= tight
    assert moved > 4 * REL_L2_TOL      # the gate would see a missing rotation


def test_rotary_key_side_without_key_adapter_is_the_plain_path():
    """b_k = NULL: nothing to rotate; the result agrees with key_rope_theta = 0 (which runs on the MFMA kernels)."""
    w = W.make_contiguous("rope_nobk", "decode", seed=306, n_agents=2, n_q_heads=8, n_kv_heads=2, head_dim=128,
                          rank=16, n=300, n_new=1, d_model=None, b_std=0.1)
    outs = []
    for theta in (0.0, 500000.0):
        dw = DeviceWorkload(w, DEV, key_rope_theta=theta)
        dw.alloc_workspace()
        dw.b_k = None
        dw.decode()
        torch.cuda.synchronize()
        outs.append(dw.out.to(torch.float64).cpu().numpy())
    w.b_k.zero_()
    rel, mx = errors(outs[1], _oracle(w, 500000.0))
    assert rel <= REL_L2_TOL and mx <= MAX_ABS_TOL
    rel, mx = errors(outs[0], outs[1])
    assert rel <= REL_L2_TOL
