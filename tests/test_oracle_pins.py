"""Pins for the fp64 oracle: everything here is CPU-only and checks oracle/
against things fixed by the paper and by mathematics, never against itself and
never against the HIP path.

The paper prints no numeric worked example for the kernel, so the pins are:
brute force, closed forms, the paper's own identities, a library routine on the
special cases that reduce to textbook attention, and a block-wise transcription
of Alg. 1.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import lra_oracle

RNG = np.random.default_rng(12345)


def _tiny(n=7, d=4, r=2, hq=4, hkv=2, agents=2, t_new=1, rng=RNG, b_std=0.5):
    return dict(
        q=rng.standard_normal((agents if t_new == 1 else t_new, hq, d)),
        k_base=rng.standard_normal((n, hkv, d)),
        v_base=rng.standard_normal((n, hkv, d)),
        l=rng.standard_normal((n, r)),
        b_k=b_std * rng.standard_normal((agents, r, hkv * d)),
        b_v=b_std * rng.standard_normal((agents, r, hkv * d)),
    )


# --------------------------------------------------------------------------
# P1: scalar brute force written with Python floats and loops only.
# --------------------------------------------------------------------------
def _brute_one_row(q_row, k_base, v_base, l, b_k_a, b_v_a, h, scale, n_vis):
    n, _, d = k_base.shape
    r = l.shape[1]
    scores = []
    vals = []
    for j in range(n_vis):
        krow = []
        vrow = []
        for c in range(d):
            kk = float(k_base[j, h, c])
            vv = float(v_base[j, h, c])
            for rho in range(r):
                kk += float(l[j, rho]) * float(b_k_a[rho, h * d + c])
                vv += float(l[j, rho]) * float(b_v_a[rho, h * d + c])
            krow.append(kk)
            vrow.append(vv)
        s = 0.0
        for c in range(d):
            s += float(q_row[c]) * krow[c]
        scores.append(scale * s)
        vals.append(vrow)
    big = max(scores)
    w = [math.exp(s - big) for s in scores]
    tot = sum(w)
    return [sum(w[j] * vals[j][c] for j in range(n_vis)) / tot for c in range(d)]


@pytest.mark.parametrize("hq,hkv", [(4, 2), (2, 2), (3, 1)])
def test_p1_brute_force_decode(hq, hkv):
    x = _tiny(hq=hq, hkv=hkv)
    n, d = x["k_base"].shape[0], x["k_base"].shape[2]
    scale = 0.37
    out = oracle.decode(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"], x["b_v"],
                        query_adapter=[1, 0], seq_query_start=[0, 2], seq_lens=[n], scale=scale)
    for qi, a in enumerate([1, 0]):
        for g in range(hq):
            h = g // (hq // hkv)
            ref = _brute_one_row(x["q"][qi, g], x["k_base"], x["v_base"], x["l"],
                                 x["b_k"][a], x["b_v"][a], h, scale, n)
            np.testing.assert_allclose(out[qi, g], ref, rtol=1e-12, atol=1e-13)


def test_p1_brute_force_prefill_causal():
    t_new, n = 3, 8
    x = _tiny(n=n, t_new=t_new, agents=1)
    scale = 1.0 / math.sqrt(4)
    out = oracle.prefill(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"][0], x["b_v"][0],
                         n=n, scale=scale)
    for i in range(t_new):
        for g in range(4):
            ref = _brute_one_row(x["q"][i, g], x["k_base"], x["v_base"], x["l"],
                                 x["b_k"][0], x["b_v"][0], g // 2, scale, n - t_new + i + 1)
            np.testing.assert_allclose(out[i, g], ref, rtol=1e-12, atol=1e-13)


def test_p1_prefill_row_subset_brute_force_and_selection():
    """prefill(rows=R) - what the full-size prefill parity checks and the benchmark's CPU
    baseline call - against the scalar brute force directly, row by row (each row with its
    own causal limit n - T + i + 1 and its own query), for an unsorted R with a repeat; and
    equal (to the last bits) to the same rows taken out of the full result, with and without the
    rotary key side."""
    t_new, n, hq, hkv, d = 6, 11, 4, 2, 4
    x = _tiny(n=n, t_new=t_new, agents=1, hq=hq, hkv=hkv, d=d)
    scale = 0.41
    rows = [4, 0, 5, 4, 2]
    args = (x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"][0], x["b_v"][0])
    sub = oracle.prefill(*args, n=n, scale=scale, rows=rows)
    assert sub.shape == (len(rows), hq, d)
    for k, i in enumerate(rows):
        for g in range(hq):
            ref = _brute_one_row(x["q"][i, g], x["k_base"], x["v_base"], x["l"],
                                 x["b_k"][0], x["b_v"][0], g // (hq // hkv), scale, n - t_new + i + 1)
            np.testing.assert_allclose(sub[k, g], ref, rtol=1e-12, atol=1e-13)
    # a different causal limit or a different query row must show: neighbouring rows differ
    assert np.abs(sub[0] - sub[2]).max() > 1e-3 and np.abs(sub[1] - sub[4]).max() > 1e-3
    for theta in (0.0, 100.0):
        full = oracle.prefill(*args, n=n, scale=scale, key_rope_theta=theta)
        part = oracle.prefill(*args, n=n, scale=scale, rows=rows, key_rope_theta=theta)
        np.testing.assert_allclose(part, full[rows], rtol=1e-13, atol=1e-14)  # same rows, up to BLAS blocking
    # a numpy index array and a sequence shorter than the cache arrays behave the same
    longer = dict(x)
    for name in ("k_base", "v_base", "l"):
        longer[name] = np.concatenate([x[name], 9.0 + x[name][:3]])
    part = oracle.prefill(x["q"], longer["k_base"], longer["v_base"], longer["l"], x["b_k"][0], x["b_v"][0],
                          n=n, scale=scale, rows=np.asarray(rows))
    np.testing.assert_allclose(part, sub, rtol=1e-13, atol=1e-14)


# --------------------------------------------------------------------------
# P2 / P3: closed forms.
# --------------------------------------------------------------------------
def test_p2_single_key_is_its_value():
    x = _tiny(n=1)
    out = oracle.decode(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"], x["b_v"],
                        [0, 1], [0, 2], [1], scale=0.5)
    d = 4
    for qi in range(2):
        for g in range(4):
            h = g // 2
            want = x["v_base"][0, h] + x["l"][0] @ x["b_v"][qi][:, h * d:(h + 1) * d]
            np.testing.assert_allclose(out[qi, g], want, rtol=1e-14, atol=1e-15)


def test_p3_zero_query_averages_visible_values():
    t_new, n, d = 4, 9, 4
    x = _tiny(n=n, t_new=t_new, agents=1)
    x["q"][:] = 0.0
    out = oracle.prefill(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"][0], x["b_v"][0],
                         n=n, scale=0.5)
    for i in range(t_new):
        vis = n - t_new + i + 1
        for g in range(4):
            h = g // 2
            want = x["v_base"][:vis, h].mean(0) + x["l"][:vis].mean(0) @ x["b_v"][0][:, h * d:(h + 1) * d]
            np.testing.assert_allclose(out[i, g], want, rtol=1e-13, atol=1e-14)


# --------------------------------------------------------------------------
# P4 / P5: the paper's reordering identity (Sec. 3.3, App. B Eq. reorder) on the
# value side, the same associativity on the key side (App. D.1), and the
# augmented-head form.
# --------------------------------------------------------------------------
def _reordered(q_rows, kb, vb, l, bk, bv, scale):
    s = scale * (q_rows @ kb.T + (q_rows @ bk.T) @ l.T)
    s -= s.max(1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(1, keepdims=True)
    return p @ vb + (p @ l) @ bv


def test_p4_reordered_equals_materialised():
    n, d, r, hq, hkv = 37, 8, 3, 6, 2
    x = _tiny(n=n, d=d, r=r, hq=hq, hkv=hkv, agents=3)
    scale = d ** -0.5
    out = oracle.decode(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"], x["b_v"],
                        [2, 0, 1], [0, 3], [n], scale)
    for qi, a in enumerate([2, 0, 1]):
        for g in range(hq):
            h = g // 3
            c = slice(h * d, (h + 1) * d)
            want = _reordered(x["q"][qi, g][None], x["k_base"][:, h], x["v_base"][:, h], x["l"],
                              x["b_k"][a][:, c], x["b_v"][a][:, c], scale)[0]
            np.testing.assert_allclose(out[qi, g], want, rtol=1e-11, atol=1e-12)


def test_p5_augmented_head_identity():
    n, d, r = 29, 8, 4
    x = _tiny(n=n, d=d, r=r, hq=2, hkv=2, agents=1)
    scale = d ** -0.5
    out = oracle.decode(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"], x["b_v"],
                        [0], [0, 1], [n], scale)
    for g in range(2):
        c = slice(g * d, (g + 1) * d)
        q_aug = np.concatenate([x["q"][0, g], x["q"][0, g] @ x["b_k"][0][:, c].T])[None]
        k_aug = np.concatenate([x["k_base"][:, g], x["l"]], axis=1)
        v_aug = np.concatenate([x["v_base"][:, g], x["l"]], axis=1)
        s = scale * q_aug @ k_aug.T
        p = np.exp(s - s.max())
        p /= p.sum()
        o_aug = (p @ v_aug)[0]
        want = o_aug[:d] + o_aug[d:] @ x["b_v"][0][:, c]
        np.testing.assert_allclose(out[0, g], want, rtol=1e-11, atol=1e-12)


# --------------------------------------------------------------------------
# P6 / P7: library scaled-dot-product attention in float64.
# --------------------------------------------------------------------------
def _sdpa64(q_tok, k, v, scale, n_visible):
    """q_tok [T][Hq][d], k/v [n][Hq][d] (already expanded per q head)."""
    qt = torch.from_numpy(q_tok).permute(1, 0, 2)[None]
    kt = torch.from_numpy(k).permute(1, 0, 2)[None]
    vt = torch.from_numpy(v).permute(1, 0, 2)[None]
    n = k.shape[0]
    mask = torch.arange(n)[None, :] < torch.as_tensor(n_visible)[:, None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


@pytest.mark.parametrize("zero_b", [True, False])
def test_p6_p7_library_sdpa(zero_b):
    t_new, n, d, r, hq, hkv = 5, 40, 16, 4, 8, 2
    x = _tiny(n=n, d=d, r=r, hq=hq, hkv=hkv, agents=1, t_new=t_new)
    if zero_b:
        x["b_k"][:] = 0.0
        x["b_v"][:] = 0.0
    scale = d ** -0.5
    out = oracle.prefill(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"][0], x["b_v"][0],
                         n=n, scale=scale)
    k_full = x["k_base"] + (x["l"] @ x["b_k"][0]).reshape(n, hkv, d)
    v_full = x["v_base"] + (x["l"] @ x["b_v"][0]).reshape(n, hkv, d)
    k_rep = np.repeat(k_full, hq // hkv, axis=1)
    v_rep = np.repeat(v_full, hq // hkv, axis=1)
    want = _sdpa64(x["q"], k_rep, v_rep, scale, n - t_new + np.arange(t_new) + 1)
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-12)


# --------------------------------------------------------------------------
# P8: Alg. 1 written block-wise (online softmax with the extra rank-r
# accumulator, epilogue O += O_lr B then O /= l), any block sizes.
# --------------------------------------------------------------------------
def _alg1(q, k, v_base, v_lr, b, scale, n_visible, b_r, b_c):
    t_new, d = q.shape
    n = k.shape[0]
    out = np.zeros((t_new, d))
    for i0 in range(0, t_new, b_r):
        qi = q[i0:i0 + b_r]
        rows = qi.shape[0]
        o = np.zeros((rows, d))
        o_lr = np.zeros((rows, v_lr.shape[1]))
        m = np.full(rows, -np.inf)
        ell = np.zeros(rows)
        for j0 in range(0, n, b_c):
            kj = k[j0:j0 + b_c]
            s = scale * qi @ kj.T
            cols = j0 + np.arange(kj.shape[0])
            s = np.where(cols[None, :] < n_visible[i0:i0 + rows, None], s, -np.inf)
            m_new = np.maximum(m, s.max(1))
            safe = np.where(np.isinf(m_new), 0.0, m_new)
            alpha = np.exp(m - safe)
            p = np.exp(s - safe[:, None])
            ell = alpha * ell + p.sum(1)
            o = alpha[:, None] * o + p @ v_base[j0:j0 + b_c]
            o_lr = alpha[:, None] * o_lr + p @ v_lr[j0:j0 + b_c]
            m = m_new
        o = o + o_lr @ b
        out[i0:i0 + rows] = o / ell[:, None]
    return out


@pytest.mark.parametrize("b_r,b_c", [(1, 1), (2, 5), (4, 16), (7, 64)])
def test_p8_blockwise_alg1(b_r, b_c):
    t_new, n, d, r = 6, 45, 8, 3
    x = _tiny(n=n, d=d, r=r, hq=2, hkv=1, agents=1, t_new=t_new)
    scale = d ** -0.5
    out = oracle.prefill(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"][0], x["b_v"][0],
                         n=n, scale=scale)
    n_vis = n - t_new + np.arange(t_new) + 1
    k_full = x["k_base"][:, 0] + x["l"] @ x["b_k"][0]          # Alg. 1 takes K as given
    for g in range(2):
        want = _alg1(x["q"][:, g], k_full, x["v_base"][:, 0], x["l"], x["b_v"][0], scale,
                     n_vis, b_r, b_c)
        np.testing.assert_allclose(out[:, g], want, rtol=1e-11, atol=1e-12)


# --------------------------------------------------------------------------
# P9: invariants.
# --------------------------------------------------------------------------
def test_p9_softmax_rows_sum_to_one_and_mask_is_exact_zero():
    k = RNG.standard_normal((33, 8)) * 30.0
    q = RNG.standard_normal((5, 8)) * 30.0
    vis = [1, 7, 20, 33, 33]
    p = oracle.softmax_weights(q, k, 1.0, vis)
    np.testing.assert_allclose(p.sum(1), 1.0, rtol=0, atol=1e-14)
    assert (p >= 0).all()
    for i, nv in enumerate(vis):
        assert (p[i, nv:] == 0).all()
        assert p[i, :nv].max() > 0


def test_p9_output_in_hull_shift_and_permutation():
    n, d, r, hq, hkv = 50, 8, 4, 4, 2
    x = _tiny(n=n, d=d, r=r, hq=hq, hkv=hkv, agents=2)
    args = ([0, 1], [0, 2], [n], 0.3)
    out = oracle.decode(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"], x["b_v"], *args)
    for qi in range(2):
        for g in range(hq):
            h = g // 2
            _, v = oracle.materialise_kv(x["k_base"][:, h], x["v_base"][:, h], x["l"],
                                         x["b_k"][qi][:, h * d:(h + 1) * d],
                                         x["b_v"][qi][:, h * d:(h + 1) * d])
            assert (out[qi, g] <= v.max(0) + 1e-12).all() and (out[qi, g] >= v.min(0) - 1e-12).all()
    # adding one vector to every key changes nothing, even a huge one
    u = 1e3 * RNG.standard_normal((1, hkv, d))
    out_shift = oracle.decode(x["q"], x["k_base"] + u, x["v_base"], x["l"], x["b_k"], x["b_v"], *args)
    np.testing.assert_allclose(out_shift, out, rtol=1e-7, atol=1e-9)
    # permuting tokens of all three caches together changes nothing without a mask
    perm = RNG.permutation(n)
    out_perm = oracle.decode(x["q"], x["k_base"][perm], x["v_base"][perm], x["l"][perm],
                             x["b_k"], x["b_v"], *args)
    np.testing.assert_allclose(out_perm, out, rtol=1e-11, atol=1e-12)


def test_p9_agents_are_independent_and_equal_adapters_agree():
    n, d, r = 31, 8, 4
    x = _tiny(n=n, d=d, r=r, hq=4, hkv=2, agents=3)
    args = ([0, 1, 2], [0, 3], [n], 0.3)
    out = oracle.decode(x["q"], x["k_base"], x["v_base"], x["l"], x["b_k"], x["b_v"], *args)
    bk2, bv2 = x["b_k"].copy(), x["b_v"].copy()
    bk2[1] += 1.0
    bv2[2] -= 1.0
    out2 = oracle.decode(x["q"], x["k_base"], x["v_base"], x["l"], bk2, bv2, *args)
    np.testing.assert_array_equal(out2[0], out[0])
    assert np.abs(out2[1] - out[1]).max() > 1e-3 and np.abs(out2[2] - out[2]).max() > 1e-3
    q3 = x["q"].copy()
    q3[1] = q3[0]
    bk3, bv3 = x["b_k"].copy(), x["b_v"].copy()
    bk3[1], bv3[1] = bk3[0], bv3[0]
    out3 = oracle.decode(q3, x["k_base"], x["v_base"], x["l"], bk3, bv3, *args)
    np.testing.assert_array_equal(out3[0], out3[1])


def test_p9_split_merge_rule_equals_unsplit():
    """Flash-decoding merge: partial (m, l, O) over key ranges recombine exactly."""
    n, d = 64, 8
    k = RNG.standard_normal((n, d))
    v = RNG.standard_normal((n, d))
    q = RNG.standard_normal((1, d))
    full = oracle.softmax_weights(q, k, 0.4, [n]) @ v
    cuts = [0, 5, 6, 40, 64]
    ms, ls, os_ = [], [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        s = 0.4 * q @ k[a:b].T
        m = s.max()
        p = np.exp(s - m)
        ms.append(m)
        ls.append(p.sum())
        os_.append(p @ v[a:b])
    big = max(ms)
    w = [math.exp(m - big) for m in ms]
    ell = sum(wi * li for wi, li in zip(w, ls))
    o = sum(wi * oi for wi, oi in zip(w, os_)) / ell
    np.testing.assert_allclose(o, full, rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------
# Paged layout: gather against a scalar index walk.
# --------------------------------------------------------------------------
def test_gather_paged_matches_index_walk():
    nb, hkv, bs, d, r = 9, 2, 4, 3, 2
    pool = RNG.standard_normal((nb, hkv, bs, d))
    pool_l = RNG.standard_normal((nb, bs, r))
    ids = [7, 2, 5, 0]
    n = 14
    kv = oracle.gather_paged(pool, ids, n)
    lr = lra_oracle.gather_paged_l(pool_l, ids, n)
    assert kv.shape == (n, hkv, d) and lr.shape == (n, r)
    for j in range(n):
        for h in range(hkv):
            np.testing.assert_array_equal(kv[j, h], pool[ids[j // bs], h, j % bs])
        np.testing.assert_array_equal(lr[j], pool_l[ids[j // bs], j % bs])
    with pytest.raises(ValueError):
        oracle.gather_paged(pool, [1, -1, 0, 0], n)


def test_paged_decode_equals_contiguous_decode():
    from paper_2602_01053_amd import workloads as W
    w = W.make_paged("t", seed=5, dtype=torch.float32, seq_lens=[19, 33, 16], agents_per_seq=2,
                     n_adapters=3, n_q_heads=4, n_kv_heads=2, head_dim=8, rank=4, d_model=None,
                     block_size=16)
    f = lambda t: t.to(torch.float64).numpy()
    out = oracle.decode(f(w.q), f(w.k_base), f(w.v_base), f(w.l), f(w.b_k), f(w.b_v),
                        w.query_adapter.numpy(), w.seq_query_start.numpy(), w.seq_lens, w.scale,
                        block_size=16, block_table=w.block_table.numpy())
    assert np.isfinite(out).all()          # NaN-poisoned free slots never leak
    for t, n_t in enumerate(w.seq_lens):
        ids = w.block_table[t].numpy()
        kb = oracle.gather_paged(f(w.k_base), ids, n_t)
        vb = oracle.gather_paged(f(w.v_base), ids, n_t)
        lr = lra_oracle.gather_paged_l(f(w.l), ids, n_t)
        for qi in range(2 * t, 2 * t + 2):
            a = int(w.query_adapter[qi])
            one = oracle.decode(f(w.q)[qi][None], kb, vb, lr, f(w.b_k), f(w.b_v), [a], [0, 1],
                                [n_t], w.scale)
            np.testing.assert_array_equal(one[0], out[qi])


# --------------------------------------------------------------------------
# P10: the tolerance gate can see the LoRA term at the configured scales.
# --------------------------------------------------------------------------
def _rel_l2(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def test_p10_gate_sees_missing_or_swapped_adapters():
    from paper_2602_01053_amd import workloads as W
    w = W.config(2, shrink=8)
    f = lambda t: t.to(torch.float64).numpy()
    args = (w.query_adapter.numpy(), w.seq_query_start.numpy(), w.seq_lens, w.scale)
    base = (f(w.q), f(w.k_base), f(w.v_base), f(w.l))
    out = oracle.decode(*base, f(w.b_k), f(w.b_v), *args)
    zero = np.zeros_like(f(w.b_k))
    assert _rel_l2(oracle.decode(*base, zero, f(w.b_v), *args), out) > 5e-3 * 4
    assert _rel_l2(oracle.decode(*base, f(w.b_k), zero, *args), out) > 5e-3 * 4
    assert _rel_l2(oracle.decode(*base, f(w.b_v), f(w.b_k), *args), out) > 5e-3 * 4
    swapped = w.query_adapter.numpy()[::-1].copy()
    assert _rel_l2(oracle.decode(*base, f(w.b_k), f(w.b_v), swapped, *args[1:]), out) > 5e-3 * 4


# --------------------------------------------------------------------------
# P11: cache-append producer (projection of the new tokens, rotary embedding
# of the keys, paged scatter).
# --------------------------------------------------------------------------
def test_p11_rope_is_a_plane_rotation_for_d2():
    """d = 2 has the single pair (0, 1) and frequency theta**0 = 1: the rotation by the
    position itself, written as a 2x2 matrix."""
    rng = np.random.default_rng(110)
    x = rng.standard_normal((5, 3, 2))
    pos = np.array([0, 1, 2, 7, 100])
    out = oracle.rope_rotate(x, pos, 10000.0)
    for t in range(5):
        c, s = math.cos(pos[t]), math.sin(pos[t])
        rot = np.array([[c, -s], [s, c]])
        np.testing.assert_allclose(out[t], x[t] @ rot.T, rtol=0, atol=1e-12)


def test_p11_rope_identity_norm_additivity_and_relative_position():
    rng = np.random.default_rng(111)
    n, H, d, theta = 6, 2, 16, 500000.0
    x = rng.standard_normal((n, H, d))
    y = rng.standard_normal((n, H, d))
    pos = np.array([0, 3, 17, 100, 4095, 65535])
    # position 0 changes nothing
    np.testing.assert_array_equal(oracle.rope_rotate(x, np.zeros(n), theta), x)
    # every pair keeps its length
    out = oracle.rope_rotate(x, pos, theta)
    half = d // 2
    np.testing.assert_allclose(out[..., :half] ** 2 + out[..., half:] ** 2,
                               x[..., :half] ** 2 + x[..., half:] ** 2, rtol=1e-12)
    # rotating by a then by b is rotating by a + b
    twice = oracle.rope_rotate(oracle.rope_rotate(x, pos, theta), 2 * pos + 1, theta)
    np.testing.assert_allclose(twice, oracle.rope_rotate(x, 3 * pos + 1, theta), rtol=0, atol=1e-9)
    # dot products of rotated vectors depend on the position difference only
    a = np.einsum("thd,thd->th", oracle.rope_rotate(x, pos, theta), oracle.rope_rotate(y, pos + 5, theta))
    b = np.einsum("thd,thd->th", oracle.rope_rotate(x, pos + 1000, theta), oracle.rope_rotate(y, pos + 1005, theta))
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-9)
    # the pair index i uses theta**(-2i/d): the slowest pair of token 1 turns by theta**(-(d-2)/d)
    e = np.zeros((2, 1, d))
    e[:, 0, half - 1] = 1.0
    ang = theta ** (-(d - 2) / d)
    got = oracle.rope_rotate(e, np.array([0, 1]), theta)[1, 0]
    assert abs(got[half - 1] - math.cos(ang)) < 1e-15 and abs(got[d - 1] - math.sin(ang)) < 1e-15


def test_p11_projection_matches_explicit_loops():
    rng = np.random.default_rng(112)
    n, dm, Hkv, d, r, theta = 3, 5, 2, 4, 3, 100.0
    x = rng.standard_normal((n, dm))
    w = rng.standard_normal((2 * Hkv * d + r, dm))
    pos = np.array([4, 5, 6])
    k, v, l = oracle.project_new_tokens(x, w, Hkv, d, r, pos, theta)
    for t in range(n):
        y = [sum(x[t, c] * w[o, c] for c in range(dm)) for o in range(w.shape[0])]
        for h in range(Hkv):
            kh = y[h * d:(h + 1) * d]
            for i in range(d // 2):
                ang = pos[t] * theta ** (-2.0 * i / d)
                assert abs(k[t, h, i] - (kh[i] * math.cos(ang) - kh[i + d // 2] * math.sin(ang))) < 1e-12
                assert abs(k[t, h, i + d // 2] - (kh[i + d // 2] * math.cos(ang) + kh[i] * math.sin(ang))) < 1e-12
            for i in range(d):
                assert abs(v[t, h, i] - y[Hkv * d + h * d + i]) < 1e-12
        for i in range(r):
            assert abs(l[t, i] - y[2 * Hkv * d + i]) < 1e-12
    # without rotation the keys are the plain projection
    k0, _, _ = oracle.project_new_tokens(x, w, Hkv, d, r, pos, 0.0)
    np.testing.assert_allclose(k0.reshape(n, -1), x @ w[:Hkv * d].T, rtol=1e-13)


def test_p11_paged_scatter_is_the_inverse_of_gather():
    rng = np.random.default_rng(113)
    nb, Hkv, bs, d, r = 7, 2, 16, 4, 3
    pool = rng.standard_normal((nb, Hkv, bs, d))
    pool_l = rng.standard_normal((nb, bs, r))
    ids = [5, 2, 6, 0]
    before = oracle.gather_paged(pool, ids, 50).copy()
    rows = rng.standard_normal((20, Hkv, d))
    rows_l = rng.standard_normal((20, r))
    oracle.scatter_paged(pool, ids, 30, rows)
    oracle.scatter_paged_l(pool_l, ids, 30, rows_l)
    after = oracle.gather_paged(pool, ids, 50)
    np.testing.assert_array_equal(after[30:50], rows)
    np.testing.assert_array_equal(after[:30], before[:30])
    np.testing.assert_array_equal(lra_oracle.gather_paged_l(pool_l, ids, 50)[30:50], rows_l)


# --------------------------------------------------------------------------
# P12: the rotary key side (App. D.1: the adapter's key contribution is reconstructed in the
# head dimension and rotated before the score).
# --------------------------------------------------------------------------
def test_p12_rotary_key_side_equals_attention_over_keys_rotated_as_a_whole():
    """K = RoPE(K'_base + L B_K) by the definition of the model; the cache holds
    RoPE(K'_base), so by linearity of the rotation the oracle's K_base + RoPE(L B_K) must
    give the same attention as textbook attention over the fully rotated keys."""
    rng = np.random.default_rng(120)
    n, hq, hkv, d, r, theta = 37, 4, 2, 8, 3, 10000.0
    k_pre = rng.standard_normal((n, hkv, d))
    v = rng.standard_normal((n, hkv, d))
    l = rng.standard_normal((n, r))
    b_k = 0.7 * rng.standard_normal((2, r, hkv * d))
    b_v = 0.7 * rng.standard_normal((2, r, hkv * d))
    q = rng.standard_normal((2, hq, d))
    k_cache = oracle.rope_rotate(k_pre, np.arange(n), theta)
    got = oracle.decode(q, k_cache, v, l, b_k, b_v, np.array([0, 1]), np.array([0, 2]), [n], 0.3,
                        key_rope_theta=theta)
    for a in range(2):
        k_full = oracle.rope_rotate(k_pre + (l @ b_k[a]).reshape(n, hkv, d), np.arange(n), theta)
        v_full = v + (l @ b_v[a]).reshape(n, hkv, d)
        for g in range(hq):
            h = g // (hq // hkv)
            s = 0.3 * (k_full[:, h, :] @ q[a, g])
            p = np.exp(s - s.max())
            np.testing.assert_allclose(got[a, g], (p / p.sum()) @ v_full[:, h, :], rtol=0, atol=1e-12)


def test_p12_rotary_key_side_scalar_loop_and_degenerate_cases():
    rng = np.random.default_rng(121)
    n, d, r, theta = 9, 4, 2, 100.0
    w = _tiny(n=n, d=d, r=r, hq=2, hkv=1, agents=1, rng=rng)
    t_new = 4
    q = rng.standard_normal((t_new, 2, d))
    got = oracle.prefill(q, w["k_base"], w["v_base"], w["l"], w["b_k"][0], w["b_v"][0], n=n, scale=0.5,
                         key_rope_theta=theta)
    half = d // 2
    for i in range(t_new):
        n_vis = n - t_new + i + 1
        for g in range(2):
            scores, vals = [], []
            for j in range(n_vis):
                delta = [sum(w["l"][j, p] * w["b_k"][0][p, c] for p in range(r)) for c in range(d)]
                key = []
                for c in range(d):
                    ang = j * theta ** (-2.0 * (c % half) / d)
                    rot = (delta[c] * math.cos(ang) - delta[c + half] * math.sin(ang)) if c < half else \
                          (delta[c] * math.cos(ang) + delta[c - half] * math.sin(ang))
                    key.append(w["k_base"][j, 0, c] + rot)
                scores.append(0.5 * sum(q[i, g, c] * key[c] for c in range(d)))
                vals.append([w["v_base"][j, 0, c] + sum(w["l"][j, p] * w["b_v"][0][p, c] for p in range(r))
                             for c in range(d)])
            m = max(scores)
            e = [math.exp(x - m) for x in scores]
            z = sum(e)
            ref = [sum(e[j] / z * vals[j][c] for j in range(n_vis)) for c in range(d)]
            np.testing.assert_allclose(got[i, g], ref, rtol=0, atol=1e-12)
    # B_K = 0: the rotation has nothing to act on
    zero = np.zeros_like(w["b_k"][0])
    np.testing.assert_array_equal(
        oracle.prefill(q, w["k_base"], w["v_base"], w["l"], zero, w["b_v"][0], n=n, scale=0.5, key_rope_theta=theta),
        oracle.prefill(q, w["k_base"], w["v_base"], w["l"], zero, w["b_v"][0], n=n, scale=0.5))
    # one cached token at position 0: no rotation
    np.testing.assert_allclose(
        oracle.prefill(q[:1], w["k_base"], w["v_base"], w["l"], w["b_k"][0], w["b_v"][0], n=1, scale=0.5, key_rope_theta=theta),
        oracle.prefill(q[:1], w["k_base"], w["v_base"], w["l"], w["b_k"][0], w["b_v"][0], n=1, scale=0.5), rtol=0, atol=1e-15)
    # and it does change the result otherwise
    plain = oracle.prefill(q, w["k_base"], w["v_base"], w["l"], w["b_k"][0], w["b_v"][0], n=n, scale=0.5)
    assert np.abs(plain - got).max() > 1e-3
