"""Pins for the oracle's projection (step 4), scatter (step 5), sparse causal attention
(step 6) and the chained layer: the two end points the paper names (full reuse at ratio 0,
full computation at ratio 1), causality, and planted-token recovery."""
import math

import numpy as np
import pytest
import torch

from oracle import qcf_oracle as orc
from paper_2604_08585_amd import inputs


def _rng(seed=0):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- qkv

def test_qkv_brute_force_tiny():
    r = _rng(0)
    H, Hkv, d, dm, M = 2, 1, 4, 6, 3
    x = r.standard_normal((M, dm))
    w = r.standard_normal(((H + 2 * Hkv) * d, dm))
    pos = np.array([0, 7, 31])
    q, k, v = orc.recompute_qkv(x, w, pos, H, Hkv, d, 10000.0)
    theta = [10000.0 ** (-2.0 * i / d) for i in range(d // 2)]
    for m in range(M):
        y = [sum(x[m, c] * w[n, c] for c in range(dm)) for n in range((H + 2 * Hkv) * d)]
        for head in range(H + Hkv):                         # Q heads then the K head
            seg = y[head * d:(head + 1) * d]
            out = q[m, head] if head < H else k[m, head - H]
            for i in range(d // 2):
                c, s = math.cos(pos[m] * theta[i]), math.sin(pos[m] * theta[i])
                assert abs(out[i] - (seg[i] * c - seg[i + d // 2] * s)) < 1e-12
                assert abs(out[i + d // 2] - (seg[i + d // 2] * c + seg[i] * s)) < 1e-12
        assert np.allclose(v[m, 0], y[(H + Hkv) * d:], atol=1e-13)      # V rows come last, unrotated


def test_qkv_position_zero_is_plain_projection():
    r = _rng(1)
    x = r.standard_normal((4, 8)); w = r.standard_normal((4 * 8, 8))
    q, k, v = orc.recompute_qkv(x, w, np.zeros(4, dtype=int), 2, 1, 8, 10000.0)
    y = torch.from_numpy(x) @ torch.from_numpy(w).T
    assert np.allclose(q.reshape(4, -1), y[:, :16].numpy(), atol=1e-13)
    assert np.allclose(k.reshape(4, -1), y[:, 16:24].numpy(), atol=1e-13)
    assert np.allclose(v.reshape(4, -1), y[:, 24:].numpy(), atol=1e-13)


# ---------------------------------------------------------------- scatter

def test_scatter_properties():
    r = _rng(2)
    kf, vf = r.standard_normal((10, 2, 4)), r.standard_normal((10, 2, 4))
    kn, vn = r.standard_normal((3, 2, 4)), r.standard_normal((3, 2, 4))
    rows = np.array([1, 4, 9])
    k2, v2 = orc.scatter(kf, vf, kn, vn, rows)
    keep = np.setdiff1d(np.arange(10), rows)
    assert np.array_equal(k2[keep], kf[keep]) and np.array_equal(v2[keep], vf[keep])
    assert np.array_equal(k2[rows], kn) and np.array_equal(v2[rows], vn)
    k3, v3 = orc.scatter(k2, v2, kn, vn, rows)                 # idempotent
    assert np.array_equal(k3, k2) and np.array_equal(v3, v2)
    k4, v4 = orc.scatter(kf, vf, kn[:0], vn[:0], rows[:0])     # nothing selected
    assert np.array_equal(k4, kf) and np.array_equal(v4, vf)
    assert k2 is not kf


# ---------------------------------------------------------------- attn

def _sdpa_causal(q, k, v, G):
    """torch float64 dense causal attention with KV heads repeated G times."""
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, G, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, G, axis=1)).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    return o[0].permute(1, 0, 2).numpy()


def test_attn_all_rows_is_dense_causal_attention():
    r = _rng(3)
    T, H, Hkv, d = 37, 4, 2, 16
    q = r.standard_normal((T, H, d)); k = r.standard_normal((T, Hkv, d)); v = r.standard_normal((T, Hkv, d))
    o, lse = orc.recompute_attn(q, np.arange(T), k, v)
    assert np.allclose(o, _sdpa_causal(q, k, v, H // Hkv), atol=1e-12)
    # log-sum-exp of row 0 is its single logit; of every row it normalises the probabilities
    assert np.allclose(lse[0], np.einsum("hd,hd->h", q[0], np.repeat(k[0], 2, axis=0)) / math.sqrt(d))


def test_attn_subset_rows_equal_rows_of_dense():
    r = _rng(4)
    T, H, Hkv, d = 50, 2, 1, 8
    q = r.standard_normal((T, H, d)); k = r.standard_normal((T, Hkv, d)); v = r.standard_normal((T, Hkv, d))
    dense = _sdpa_causal(q, k, v, 2)
    idx = np.array([0, 3, 4, 20, 49])
    o, _ = orc.recompute_attn(q[idx], idx, k, v)
    assert np.allclose(o, dense[idx], atol=1e-12)


def test_attn_causality_first_row_and_offset():
    r = _rng(5)
    T, H, Hkv, d = 20, 2, 2, 8
    q = r.standard_normal((3, H, d)); k = r.standard_normal((T, Hkv, d)); v = r.standard_normal((T, Hkv, d))
    pos = np.array([0, 6, 12])
    o, lse = orc.recompute_attn(q, pos, k, v)
    assert np.allclose(o[0], v[0], atol=1e-14)                     # position 0 sees only token 0
    k2, v2 = k.copy(), v.copy()
    k2[13:] += 9.0; v2[13:] -= 4.0                                 # the future of every row
    o2, _ = orc.recompute_attn(q, pos, k2, v2)
    assert np.array_equal(o, o2)
    k3 = k.copy(); k3[12] += 1.0                                   # visible to the last row only
    o3, _ = orc.recompute_attn(q, pos, k3, v)
    assert np.array_equal(o3[:2], o[:2]) and not np.allclose(o3[2], o[2])
    # a context that starts at global position 5: row at position 6 sees fused rows 0..1
    o4, _ = orc.recompute_attn(q[1:2], np.array([6]), k, v, ctx_pos0=5)
    o5, _ = orc.recompute_attn(q[1:2], np.array([1]), k[:2], v[:2])
    assert np.allclose(o4, o5, atol=1e-14)
    # a row placed before the context sees nothing
    o6, lse6 = orc.recompute_attn(q[:1], np.array([2]), k, v, ctx_pos0=5)
    assert np.all(o6 == 0) and np.all(np.isneginf(lse6))


def test_attn_brute_force_tiny():
    r = _rng(6)
    T, H, Hkv, d = 5, 2, 1, 4
    q = r.standard_normal((2, H, d)); k = r.standard_normal((T, Hkv, d)); v = r.standard_normal((T, Hkv, d))
    pos = [1, 3]
    o, lse = orc.recompute_attn(q, np.array(pos), k, v)
    for i in range(2):
        for h in range(H):
            lg = [sum(q[i, h, c] * k[j, 0, c] for c in range(d)) / math.sqrt(d) for j in range(pos[i] + 1)]
            z = sum(math.exp(x) for x in lg)
            ref = [sum(math.exp(lg[j]) / z * v[j, 0, c] for j in range(pos[i] + 1)) for c in range(d)]
            assert np.allclose(o[i, h], ref, atol=1e-13)
            assert abs(lse[i, h] - math.log(z)) < 1e-13


# ---------------------------------------------------------------- chained layer

def _tiny_layer(seed, T=48, H=4, Hkv=2, d=16, dm=32, R=5):
    r = _rng(seed)
    x = r.standard_normal((T, dm))
    w = r.standard_normal(((H + 2 * Hkv) * d, dm)) / math.sqrt(dm)
    qp = r.standard_normal((R, H, d))
    return x, w, qp


def _dense_prefill(x, w, H, Hkv, d, base):
    T = x.shape[0]
    q, k, v = orc.recompute_qkv(x, w, np.arange(T), H, Hkv, d, base)
    return q, k, v, _sdpa_causal(q, k, v, H // Hkv)


def test_ratio_one_is_full_causal_prefill():
    """Full computation end point: recomputing every token reproduces dense causal prefill,
    whatever the stale caches held."""
    H, Hkv, d, base = 4, 2, 16, 10000.0
    x, w, qp = _tiny_layer(10)
    r = _rng(11)
    lens = [16, 20, 12]
    stale_k = [r.standard_normal((n, Hkv, d)) for n in lens]
    stale_v = [r.standard_normal((n, Hkv, d)) for n in lens]
    out = orc.fuse_layer(stale_k, stale_v, [0, 16, 36], qp, x, w, 1.0, H, Hkv, d, base)
    q, k, v, dense = _dense_prefill(x, w, H, Hkv, d, base)
    assert list(out["sel_idx"]) == list(range(48))
    assert np.allclose(out["o_sel"], dense, atol=1e-11)
    assert np.allclose(out["k_patched"], k, atol=1e-12) and np.allclose(out["v_patched"], v, atol=1e-12)


def test_ratio_zero_is_full_reuse():
    H, Hkv, d, base = 4, 2, 16, 10000.0
    x, w, qp = _tiny_layer(12)
    r = _rng(13)
    ks = [r.standard_normal((24, Hkv, d)) for _ in range(2)]
    vs = [r.standard_normal((24, Hkv, d)) for _ in range(2)]
    out = orc.fuse_layer(ks, vs, [0, 24], qp, x, w, 0.0, H, Hkv, d, base)
    kf, vf = orc.rerope(ks, vs, [0, 24], base)
    assert out["sel_idx"].size == 0 and out["o_sel"].shape[0] == 0
    assert np.array_equal(out["k_patched"], kf) and np.array_equal(out["v_patched"], vf)


@pytest.mark.parametrize("ratio", [0.1, 0.5])
def test_true_cache_makes_every_ratio_exact(ratio):
    """If the chunk caches already hold the K/V the full prompt would produce (each chunk stored
    in its local frame), any ratio returns the rows of the dense prefill output and the scatter
    changes nothing beyond rounding."""
    H, Hkv, d, base = 4, 2, 16, 10000.0
    x, w, qp = _tiny_layer(14)
    q, k, v, dense = _dense_prefill(x, w, H, Hkv, d, base)
    bounds = [(0, 10), (10, 30), (30, 48)]
    ks = [orc.rerope([k[a:b]], None, [-a], base)[0] for a, b in bounds]     # back to local frames
    vs = [v[a:b] for a, b in bounds]
    out = orc.fuse_layer(ks, vs, [a for a, _ in bounds], qp, x, w, ratio, H, Hkv, d, base)
    idx = out["sel_idx"]
    assert len(idx) == orc.select_count(48, ratio)
    assert np.allclose(out["k_fused"], k, atol=1e-11)
    assert np.allclose(out["k_patched"], k, atol=1e-11)
    assert np.allclose(out["o_sel"], dense[idx], atol=1e-11)


def test_selected_rows_see_new_kv_of_other_selected_rows():
    """With stale caches and a forced selection, row i's output must use the recomputed K/V of
    earlier selected rows (otherwise ratio 1 could not equal full prefill)."""
    H, Hkv, d, base = 2, 1, 8, 10000.0
    x, w, qp = _tiny_layer(15, T=12, H=H, Hkv=Hkv, d=d, dm=16)
    r = _rng(16)
    ks, vs = [r.standard_normal((12, Hkv, d))], [r.standard_normal((12, Hkv, d))]
    idx = np.array([2, 7])
    out = orc.fuse_layer(ks, vs, [0], qp, x, w, 0.5, H, Hkv, d, base, sel_idx=idx)
    qn, kn, vn = orc.recompute_qkv(x[idx], w, idx, H, Hkv, d, base)
    k_mix, v_mix = ks[0].copy(), vs[0].copy()
    k_mix[idx], v_mix[idx] = kn, vn
    ref, _ = orc.recompute_attn(qn, idx, k_mix, v_mix)
    assert np.allclose(out["o_sel"], ref, atol=1e-13)
    stale, _ = orc.recompute_attn(qn, idx, ks[0], vs[0])
    assert not np.allclose(out["o_sel"], stale)


# ---------------------------------------------------------------- planted tokens

def test_planted_tokens_are_recovered_with_coherent_probes():
    ops = orc.PlantOps()
    wl = inputs.assemble(inputs.make_raw(0), ops, plant_per_chunk=8, coherent_probe=0.25)
    req, sh = wl.requests[0], wl.shape
    assert len(req.planted) == 32
    kf, _ = orc.rerope([c.k for c in req.chunks], None, req.dst_pos0, sh.rope_base)
    s = orc.score(req.q_probe, kf)
    idx = orc.select(s, orc.select_count(req.T, wl.ratio))
    assert set(req.planted) <= set(idx)                 # 32 planted among the 77 selected
    assert set(orc.select(s, 32)) == set(req.planted)   # and they are the top 32 outright


def test_planted_tokens_score_above_chance_in_config_0():
    ops = orc.PlantOps()
    wl = inputs.make_config(0, ops)
    req, sh = wl.requests[0], wl.shape
    kf, _ = orc.rerope([c.k for c in req.chunks], None, req.dst_pos0, sh.rope_base)
    s = orc.score(req.q_probe, kf)
    idx = orc.select(s, orc.select_count(req.T, wl.ratio))
    recall = len(set(idx) & set(req.planted)) / len(req.planted)
    mask = np.zeros(req.T, dtype=bool); mask[req.planted] = True
    assert recall > wl.ratio
    assert s[mask].mean() > s[~mask].mean()
