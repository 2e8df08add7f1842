"""Pins for where the oracle's chained functions apply the storage rounding (`quantize=`).

The GPU path stores the fused K/V, the recomputed Q/K/V rows, the attention output and every intermediate of
the rest of the block in its element type; the chained comparisons hand the oracle a rounding function for
those tensors.  These tests use a deliberately coarse rounding (multiples of 1/8) so that a stage whose
rounding was dropped, applied twice in the wrong place, or fed un-rounded inputs changes the result visibly."""
import numpy as np

from oracle import qcf_oracle as orc


class CoarseRounding:
    """Rounds to multiples of 1/8 and records the shape of everything it is applied to."""

    def __init__(self):
        self.shapes = []

    def __call__(self, a):
        a = np.asarray(a, dtype=np.float64)
        self.shapes.append(a.shape)
        return np.round(a * 8.0) / 8.0


def is_fixed_point(a):
    return np.array_equal(np.round(np.asarray(a) * 8.0) / 8.0, a)


def small_layer(seed=5):
    r = np.random.default_rng(seed)
    H, Hkv, D, dm = 4, 2, 8, 16
    lens = [5, 7, 4]
    k_chunks = [r.standard_normal((n, Hkv, D)) for n in lens]
    v_chunks = [r.standard_normal((n, Hkv, D)) for n in lens]
    deltas = [0, 5, 12]
    T = sum(lens)
    q_probe = r.standard_normal((3, H, D))
    x_ctx = r.standard_normal((T, dm))
    w = r.standard_normal(((H + 2 * Hkv) * D, dm)) / np.sqrt(dm)
    return dict(H=H, Hkv=Hkv, D=D, k_chunks=k_chunks, v_chunks=v_chunks, deltas=deltas, T=T, q_probe=q_probe,
                x_ctx=x_ctx, w=w)


def test_fuse_layer_rounds_each_stored_tensor_once_and_in_order():
    c = small_layer()
    qz = CoarseRounding()
    out = orc.fuse_layer(c["k_chunks"], c["v_chunks"], c["deltas"], c["q_probe"], c["x_ctx"], c["w"], 0.4, c["H"],
                         c["Hkv"], c["D"], 10000.0, quantize=qz)
    T, n = c["T"], orc.select_count(c["T"], 0.4)
    H, Hkv, D = c["H"], c["Hkv"], c["D"]
    assert qz.shapes == [(T, Hkv, D), (T, Hkv, D), (n, H, D), (n, Hkv, D), (n, Hkv, D), (n, H, D)]
    for key in ("k_fused", "v_fused", "q_sel", "k_sel", "v_sel", "k_patched", "v_patched", "o_sel"):
        assert is_fixed_point(out[key]), key
    assert not is_fixed_point(out["score"])            # scores and log-sum-exp stay unrounded (fp32 on the GPU)


def test_fuse_layer_feeds_rounded_tensors_to_the_next_stage():
    c = small_layer()
    args = (c["k_chunks"], c["v_chunks"], c["deltas"], c["q_probe"], c["x_ctx"], c["w"], 0.4, c["H"], c["Hkv"],
            c["D"], 10000.0)
    out = orc.fuse_layer(*args, quantize=CoarseRounding())
    exact = orc.fuse_layer(*args)
    q = lambda a: np.round(np.asarray(a) * 8.0) / 8.0
    # stage by stage, each step called on its own with the rounded outputs of the one before
    kf, vf = orc.rerope(c["k_chunks"], c["v_chunks"], c["deltas"], 10000.0)
    assert np.array_equal(out["k_fused"], q(kf)) and np.array_equal(out["v_fused"], q(vf))
    s = orc.score(c["q_probe"], q(kf))
    assert np.array_equal(out["score"], s)                          # scored on the stored keys ...
    assert not np.allclose(out["score"], exact["score"], rtol=1e-6)   # ... which differ from the exact ones
    idx = orc.select(s, orc.select_count(c["T"], 0.4))
    assert np.array_equal(out["sel_idx"], idx)
    qs, ks, vs = orc.recompute_qkv(c["x_ctx"][idx], c["w"], idx, c["H"], c["Hkv"], c["D"], 10000.0)
    assert np.array_equal(out["q_sel"], q(qs)) and np.array_equal(out["k_sel"], q(ks)) and np.array_equal(out["v_sel"], q(vs))
    kp, vp = orc.scatter(q(kf), q(vf), q(ks), q(vs), idx)
    assert np.array_equal(out["k_patched"], kp) and np.array_equal(out["v_patched"], vp)
    o, lse = orc.recompute_attn(q(qs), idx, kp, vp)
    assert np.array_equal(out["o_sel"], q(o)) and np.array_equal(out["lse"], lse)
    # attention on un-rounded Q (a dropped rounding of stage 4) would give another result
    o_bad, _ = orc.recompute_attn(qs, idx, kp, vp)
    assert not np.array_equal(q(o_bad), out["o_sel"])


def test_layer_tail_rounds_each_stored_intermediate():
    r = np.random.default_rng(9)
    M, H, D, dm, F = 6, 4, 8, 16, 24
    h_in = r.standard_normal((M, dm))
    o = r.standard_normal((M, H, D))
    w_o = r.standard_normal((dm, H * D)) / np.sqrt(H * D)
    g = 1.0 + 0.1 * r.standard_normal(dm)
    w_gu = r.standard_normal((2 * F, dm)) / np.sqrt(dm)
    w_dn = r.standard_normal((dm, F)) / np.sqrt(F)
    qz = CoarseRounding()
    out = orc.layer_tail(h_in, o, w_o, g, w_gu, w_dn, 1e-5, quantize=qz)
    assert qz.shapes == [(M, dm), (M, dm), (M, 2 * F), (M, F), (M, dm)]
    q = lambda a: np.round(np.asarray(a) * 8.0) / 8.0
    h1 = q(orc.linear(o.reshape(M, -1), w_o, h_in))
    n = q(orc.rmsnorm(h1, g, 1e-5))
    gu = q(orc.linear(n, w_gu))
    act = q(orc.swiglu(gu))
    assert np.array_equal(out, q(orc.linear(act, w_dn, h1)))        # the residual is the stored h1
    assert not np.array_equal(out, q(orc.layer_tail(h_in, o, w_o, g, w_gu, w_dn, 1e-5)))
    # a chain that skips the rounding of the activation differs
    assert not np.array_equal(out, q(orc.linear(orc.swiglu(gu), w_dn, h1)))
