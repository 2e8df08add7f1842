"""Pins for the oracle's rotary embedding and re-rotation (step 1) and for the
consistency between re-rotation and the projection's rotary embedding (step 4).
None of the expected values is produced by the functions under test."""
import math
import os

import numpy as np
import pytest

from oracle import qcf_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _rng(seed=0):
    return np.random.default_rng(seed)


def test_quarter_turn_golden():
    base = 4.0 / math.pi ** 2
    theta = orc.rope_frequencies(4, base)
    assert theta[0] == 1.0 and abs(theta[1] - math.pi / 2) < 1e-15
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "rope_quarter_turn.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 6
    for style, delta, a, b, a_out, b_out in rows:
        style, delta = int(style), int(delta)
        a, b, a_out, b_out = map(float, (a, b, a_out, b_out))
        x = np.zeros((1, 1, 4))
        ia, ib = ((1, 3) if style == 0 else (2, 3))
        x[0, 0, ia], x[0, 0, ib] = a, b
        k, v = orc.rerope([x], [x], [delta], base, style)
        assert abs(k[0, 0, ia] - a_out) < 1e-12 and abs(k[0, 0, ib] - b_out) < 1e-12
        # pair 0 was zero and must stay zero; values are copied untouched
        others = [i for i in range(4) if i not in (ia, ib)]
        assert np.all(k[0, 0, others] == 0.0)
        assert np.array_equal(v, x)


def test_frequencies_closed_form():
    th = orc.rope_frequencies(128, 500000.0)
    assert th.shape == (64,) and th[0] == 1.0
    # theta_i is a geometric sequence with ratio base^(-2/d); the last one is base^(-(d-2)/d)
    assert np.allclose(th[1:] / th[:-1], 500000.0 ** (-2.0 / 128), rtol=1e-13)
    assert abs(th[-1] - 500000.0 ** (-126.0 / 128)) < 1e-18


@pytest.mark.parametrize("style", [0, 1])
def test_group_law_and_identity(style):
    r = _rng(1)
    k = r.standard_normal((7, 2, 64))
    base = 10000.0
    k0, _ = orc.rerope([k], None, [0], base, style)
    assert np.array_equal(k0, k)
    for a, b in [(3, 5), (100, -37), (4000, 4191), (-8, 8)]:
        ka, _ = orc.rerope([k], None, [a], base, style)
        kab, _ = orc.rerope([ka], None, [b], base, style)
        kd, _ = orc.rerope([k], None, [a + b], base, style)
        assert np.max(np.abs(kab - kd)) < 1e-11


@pytest.mark.parametrize("style", [0, 1])
def test_pair_norms_preserved_and_complex_form(style):
    r = _rng(2)
    d, base, delta = 64, 10000.0, 1234
    k = r.standard_normal((5, 3, d))
    out, _ = orc.rerope([k], None, [delta], base, style)
    if style == 0:
        zin, zout = k[..., :d // 2] + 1j * k[..., d // 2:], out[..., :d // 2] + 1j * out[..., d // 2:]
    else:
        zin, zout = k[..., 0::2] + 1j * k[..., 1::2], out[..., 0::2] + 1j * out[..., 1::2]
    assert np.allclose(np.abs(zin), np.abs(zout), rtol=1e-12)
    # multiplying by the unit complex number exp(i delta theta_i), with theta_i written out
    # independently as base^(-2i/d)
    th = np.array([base ** (-2.0 * i / d) for i in range(d // 2)])
    assert np.allclose(zout, zin * np.exp(1j * delta * th), atol=1e-11)


def test_concatenation_layout_and_values_copied():
    r = _rng(3)
    lens = [3, 1, 5]
    ks = [r.standard_normal((n, 2, 8)) for n in lens]
    vs = [r.standard_normal((n, 2, 8)) for n in lens]
    deltas = [0, 3, 4]
    kf, vf = orc.rerope(ks, vs, deltas, 10000.0)
    assert kf.shape == (9, 2, 8)
    assert np.array_equal(vf, np.concatenate(vs))
    assert np.array_equal(kf[:3], ks[0])                      # delta 0 chunk is untouched
    one, _ = orc.rerope([ks[2]], None, [4], 10000.0)
    assert np.array_equal(kf[4:], one)                        # each chunk uses its own delta
    assert not np.allclose(kf[3:4], ks[1])


@pytest.mark.parametrize("style", [0, 1])
def test_rerope_matches_rope_at_shifted_position(style):
    """Rotating raw keys at p + delta equals re-rotating keys embedded at p by delta."""
    r = _rng(4)
    raw = r.standard_normal((6, 2, 32))
    pos = np.array([0, 1, 2, 3, 4, 5])
    delta = 777
    at_p = orc.rope_at(raw, pos, 500000.0, style)
    shifted, _ = orc.rerope([at_p], None, [delta], 500000.0, style)
    assert np.allclose(shifted, orc.rope_at(raw, pos + delta, 500000.0, style), atol=1e-11)


@pytest.mark.parametrize("style", [0, 1])
def test_logits_depend_on_relative_position_only(style):
    r = _rng(5)
    q = r.standard_normal((4, 1, 16))
    k = r.standard_normal((4, 1, 16))
    pq, pk = np.array([10, 11, 12, 13]), np.array([0, 3, 5, 9])
    def logits(shift):
        qr = orc.rope_at(q, pq + shift, 10000.0, style)[:, 0]
        kr = orc.rope_at(k, pk + shift, 10000.0, style)[:, 0]
        return qr @ kr.T
    assert np.allclose(logits(0), logits(4096), atol=1e-9)
    # and they do depend on the relative offset (a sign error in one of the two
    # rotation terms would make the embedding a reflection and break the first check;
    # a no-op embedding would break this one)
    kr2 = orc.rope_at(k, pk + 1, 10000.0, style)[:, 0]
    assert not np.allclose(logits(0), orc.rope_at(q, pq, 10000.0, style)[:, 0] @ kr2.T)


def test_styles_are_a_permutation_of_each_other():
    r = _rng(6)
    d = 16
    x = r.standard_normal((3, 2, d))
    perm = np.empty(d, dtype=int)           # interleaved index of each half-split slot
    perm[: d // 2] = np.arange(0, d, 2)
    perm[d // 2:] = np.arange(1, d, 2)
    xi = np.empty_like(x)
    xi[..., perm] = x
    pos = np.array([5, 9, 200])
    a = orc.rope_at(x, pos, 10000.0, 0)
    b = orc.rope_at(xi, pos, 10000.0, 1)
    assert np.allclose(b[..., perm], a, atol=1e-13)


def test_qkv_projection_then_shift_equals_projection_at_global_positions():
    """Step 4's embedding and step 1's shift agree: a chunk prefilled by the projection at
    local positions and moved by delta equals the projection at the global positions."""
    r = _rng(7)
    H, Hkv, d, dm, L, delta = 4, 2, 16, 24, 5, 300
    x = r.standard_normal((L, dm))
    w = r.standard_normal(((H + 2 * Hkv) * d, dm)) / math.sqrt(dm)
    local = np.arange(L)
    _, k_loc, v_loc = orc.recompute_qkv(x, w, local, H, Hkv, d, 10000.0)
    _, k_glob, v_glob = orc.recompute_qkv(x, w, local + delta, H, Hkv, d, 10000.0)
    moved, vm = orc.rerope([k_loc], [v_loc], [delta], 10000.0)
    assert np.allclose(moved, k_glob, atol=1e-11)
    assert np.array_equal(vm, v_glob)
