"""Pins for the oracle's rest-of-the-layer functions (RMSNorm, linear maps, gated SiLU feed-forward)
and for running the user-query rows through the same projection / scatter / attention calls as extra
recomputed rows."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import qcf_oracle as orc


def _rng(seed=0):
    return np.random.default_rng(seed)


def _t(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def test_rmsnorm_closed_forms():
    r = _rng(1)
    x = r.standard_normal((7, 48))
    w = r.standard_normal(48)
    y = orc.rmsnorm(x, np.ones(48), 0.0)
    assert np.allclose(np.mean(y * y, axis=-1), 1.0, atol=1e-12)            # unit mean square
    assert np.allclose(orc.rmsnorm(3.7 * x, w, 0.0), orc.rmsnorm(x, w, 0.0), atol=1e-12)   # scale invariant
    assert np.allclose(orc.rmsnorm(-x, w, 1e-5), -orc.rmsnorm(x, w, 1e-5))   # odd
    c = np.full((1, 48), -2.5)
    assert np.allclose(orc.rmsnorm(c, w, 0.0), -w)                            # constant row -> sign * weight
    # eps enters under the root, next to the mean square: for x = (a, 0, 0, 0), y0 = a / sqrt(a^2/4 + eps)
    e = np.zeros((1, 4)); e[0, 0] = 3.0
    assert np.isclose(orc.rmsnorm(e, np.ones(4), 0.75)[0, 0], 3.0 / np.sqrt(9.0 / 4.0 + 0.75))


def test_rmsnorm_matches_torch():
    r = _rng(2)
    x, w = r.standard_normal((5, 64)), r.standard_normal(64)
    ref = F.rms_norm(_t(x), (64,), _t(w), eps=1e-5).numpy()
    assert np.allclose(orc.rmsnorm(x, w, 1e-5), ref, atol=1e-13)


def test_linear_brute_force_and_layout():
    r = _rng(3)
    x, w, res = r.standard_normal((3, 5)), r.standard_normal((4, 5)), r.standard_normal((3, 4))
    y = orc.linear(x, w, res)
    for m in range(3):
        for n in range(4):                      # w holds one row per output feature
            assert np.isclose(y[m, n], sum(x[m, k] * w[n, k] for k in range(5)) + res[m, n])
    assert np.allclose(orc.linear(x, w), y - res)
    assert np.allclose(orc.linear(x, w), F.linear(_t(x), _t(w)).numpy(), atol=1e-13)


def test_swiglu_values_and_limits():
    gu = np.array([[0.0, 1.0, -1.0, 40.0, -40.0, 2.0, 3.0, 5.0, 7.0, 11.0]])    # gates | ups
    y = orc.swiglu(gu)[0]
    assert y[0] == 0.0                                                      # silu(0) = 0
    assert np.isclose(y[1], 1.0 / (1.0 + np.exp(-1.0)) * 3.0)
    assert np.isclose(y[2], -1.0 / (1.0 + np.exp(1.0)) * 5.0)
    assert np.isclose(y[3], 40.0 * 7.0)                                     # silu(g) -> g for large g
    assert abs(y[4]) < 1e-13                                                # silu(g) -> 0 for very negative g
    r = _rng(4)
    g, u = r.standard_normal((6, 9)), r.standard_normal((6, 9))
    assert np.allclose(orc.swiglu(np.concatenate([g, u], axis=1)), (F.silu(_t(g)) * _t(u)).numpy(), atol=1e-13)


def test_layer_tail_composition_and_special_cases():
    r = _rng(5)
    M, H, d, dm, Fd = 6, 4, 8, 24, 40
    h, o = r.standard_normal((M, dm)), r.standard_normal((M, H, d))
    w_o, g = r.standard_normal((dm, H * d)) / 6, r.standard_normal(dm)
    w_gu, w_dn = r.standard_normal((2 * Fd, dm)) / 5, r.standard_normal((dm, Fd)) / 6
    out = orc.layer_tail(h, o, w_o, g, w_gu, w_dn, 1e-5)
    # the same block written with torch's float64 routines
    h1 = _t(h) + F.linear(_t(o).reshape(M, -1), _t(w_o))
    n = F.rms_norm(h1, (dm,), _t(g), eps=1e-5)
    ref = h1 + F.linear(F.silu(F.linear(n, _t(w_gu[:Fd]))) * F.linear(n, _t(w_gu[Fd:])), _t(w_dn))
    assert np.allclose(out, ref.numpy(), atol=1e-12)
    # a feed-forward that outputs nothing leaves h1; an output projection that outputs nothing leaves h_in in h1
    assert np.allclose(orc.layer_tail(h, o, w_o, g, w_gu, np.zeros_like(w_dn), 1e-5), h1.numpy(), atol=1e-12)
    z = orc.layer_tail(h, o, np.zeros_like(w_o), g, w_gu, np.zeros_like(w_dn), 1e-5)
    assert np.allclose(z, h)
    # rows are independent
    assert np.allclose(orc.layer_tail(h[2:3], o[2:3], w_o, g, w_gu, w_dn, 1e-5), out[2:3], atol=1e-12)


def test_query_rows_as_extra_recomputed_rows_equal_dense_prefill():
    """At ratio 1, appending the user-query rows (positions T .. T+R-1) to the recomputed set, with their
    K/V appended to the fused cache, reproduces dense causal attention over context + query."""
    r = _rng(6)
    H, Hkv, d, dm, base = 4, 2, 16, 32, 10000.0
    T, R = 40, 6
    x = r.standard_normal((T + R, dm))
    w = r.standard_normal(((H + 2 * Hkv) * d, dm)) / np.sqrt(dm)
    pos = np.arange(T + R)
    q, k, v = orc.recompute_qkv(x, w, pos, H, Hkv, d, base)
    # path: context rows are in the cache (here: true values), query rows are projected and appended
    k_f = np.concatenate([k[:T], np.zeros((R, Hkv, d))]); v_f = np.concatenate([v[:T], np.zeros((R, Hkv, d))])
    qq, kq, vq = orc.recompute_qkv(x[T:], w, pos[T:], H, Hkv, d, base)
    k_f, v_f = orc.scatter(k_f, v_f, kq, vq, np.arange(T, T + R))
    o_q, _ = orc.recompute_attn(qq, pos[T:], k_f, v_f)
    rep = H // Hkv
    dense = F.scaled_dot_product_attention(_t(q).permute(1, 0, 2)[None], _t(np.repeat(k, rep, axis=1)).permute(1, 0, 2)[None],
                                           _t(np.repeat(v, rep, axis=1)).permute(1, 0, 2)[None], is_causal=True)[0]
    assert np.allclose(o_q, dense.permute(1, 0, 2).numpy()[T:], atol=1e-11)


# ---------------------------------------------------------------- anchor extraction

def test_key_norm_closed_forms():
    r = _rng(7)
    k = r.standard_normal((9, 3, 8))
    n = orc.key_norm(k)
    assert np.allclose(n, np.linalg.norm(k.reshape(9, -1), axis=1), atol=1e-13)       # heads concatenated
    assert np.allclose(orc.key_norm(-2.5 * k), 2.5 * n)
    e = np.zeros((2, 3, 8)); e[0, 1, 4] = -3.0; e[1, 0, 0] = 3.0; e[1, 2, 7] = 4.0
    assert np.allclose(orc.key_norm(e), [3.0, 5.0])
    # heads add in quadrature
    assert np.allclose(n ** 2, sum(orc.key_norm(k[:, h:h + 1]) ** 2 for h in range(3)))


def test_extract_anchors_picks_the_largest_norms():
    r = _rng(8)
    k, v = r.standard_normal((50, 2, 4)), r.standard_normal((50, 2, 4))
    k[[7, 30, 41]] *= 10.0
    idx, ak, av = orc.extract_anchors(k, v, 3)
    assert list(idx) == [7, 30, 41]
    assert np.array_equal(ak, k[[7, 30, 41]]) and np.array_equal(av, v[[7, 30, 41]])
    norms = np.linalg.norm(k.reshape(50, -1), axis=1)
    idx6, _, _ = orc.extract_anchors(k, v, 6)
    assert sorted(idx6) == sorted(np.argsort(-norms, kind="stable")[:6])
    assert len(orc.extract_anchors(k, v, 0)[0]) == 0
