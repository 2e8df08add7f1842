"""Pins for the oracle's critical-layer scoring (step 2) and Top-N selection (step 3)."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import qcf_oracle as orc


def _rng(seed=0):
    return np.random.default_rng(seed)


def test_scores_are_a_distribution():
    r = _rng(0)
    q = r.standard_normal((5, 4, 16))
    k = r.standard_normal((33, 2, 16))
    s = orc.score(q, k)
    assert s.shape == (33,) and np.all(s >= 0)
    assert abs(s.sum() - 1.0) < 1e-12


def test_single_row_single_head_is_textbook_softmax():
    r = _rng(1)
    d = 8
    q = r.standard_normal((1, 1, d))
    k = r.standard_normal((17, 1, d))
    ref = scipy.special.softmax((k[:, 0] @ q[0, 0]) / math.sqrt(d))
    assert np.allclose(orc.score(q, k), ref, atol=1e-14)


def test_brute_force_tiny():
    r = _rng(2)
    R, H, Hkv, d, T = 3, 4, 2, 4, 6
    q = r.standard_normal((R, H, d))
    k = r.standard_normal((T, Hkv, d))
    G = H // Hkv
    acc = [0.0] * T
    for i in range(R):
        for h in range(H):
            lg = [sum(q[i, h, c] * k[j, h // G, c] for c in range(d)) / math.sqrt(d) for j in range(T)]
            z = sum(math.exp(x) for x in lg)
            for j in range(T):
                acc[j] += math.exp(lg[j]) / z
    ref = np.array(acc) / (R * H)
    assert np.allclose(orc.score(q, k), ref, atol=1e-13)


def test_equal_keys_give_uniform_score():
    r = _rng(3)
    q = r.standard_normal((4, 2, 8))
    k = np.tile(r.standard_normal((1, 2, 8)), (10, 1, 1))
    assert np.allclose(orc.score(q, k), 0.1, atol=1e-14)


def test_permutation_equivariance_and_orthogonal_shift():
    r = _rng(4)
    q = r.standard_normal((3, 2, 8))
    k = r.standard_normal((12, 1, 8))
    s = orc.score(q, k)
    perm = r.permutation(12)
    assert np.allclose(orc.score(q, k[perm]), s[perm], atol=1e-14)
    # a vector orthogonal to every probe query, added to every key, changes no logit
    qs = q.reshape(-1, 8)
    _, _, vt = np.linalg.svd(qs, full_matrices=True)
    u = vt[-1]                       # 6 probe vectors span <= 6 of 8 dims
    assert np.max(np.abs(qs @ u)) < 1e-12
    assert np.allclose(orc.score(q, k + 5.0 * u), s, atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    r = _rng(5)
    q = r.standard_normal((3, 6, 8))
    k = r.standard_normal((9, 2, 8))
    k_rep = np.repeat(k, 3, axis=1)            # head h uses kv head h // 3
    assert np.allclose(orc.score(q, k), orc.score(q, k_rep), atol=1e-14)
    # and the grouping is h // G, not h % Hkv: swapping to the other mapping changes the result
    k_mod = np.tile(k, (1, 3, 1))
    assert not np.allclose(orc.score(q, k), orc.score(q, k_mod))


def test_large_logits_are_stable_and_scale_matters():
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 2000.0
    k = np.zeros((3, 1, 4)); k[1, 0, 0] = 1.0
    s = orc.score(q, k)
    assert np.all(np.isfinite(s)) and s[1] > 0.999999
    # 1/sqrt(d) scaling: with d = 4 and logit difference 2 ln 3, odds must be exactly 3:1
    q2 = np.zeros((1, 1, 4)); q2[0, 0, 0] = 2.0 * math.log(3.0)
    k2 = np.zeros((2, 1, 4)); k2[0, 0, 0] = 1.0
    s2 = orc.score(q2, k2)
    assert abs(s2[0] / s2[1] - 3.0) < 1e-12


def test_probe_limit_masks_later_tokens():
    r = _rng(6)
    q = r.standard_normal((2, 2, 8))
    k = r.standard_normal((7, 1, 8))
    s = orc.score(q, k, probe_limit=np.array([7, 3]))
    full0 = orc.score(q[:1], k)
    part1 = orc.score(q[1:], k[:3])
    ref = 0.5 * full0
    ref[:3] += 0.5 * part1
    assert np.allclose(s, ref, atol=1e-14)


def test_empty_inputs():
    assert orc.score(np.zeros((2, 2, 4)), np.zeros((0, 1, 4))).shape == (0,)


# ---------------------------------------------------------------- select

def test_select_count():
    assert orc.select_count(512, 0.15) == 77
    assert orc.select_count(4096, 0.15) == 615
    assert orc.select_count(8192, 0.05) == 410
    assert orc.select_count(8192, 0.15) == 1229
    assert orc.select_count(8192, 0.30) == 2458
    assert orc.select_count(32768, 0.15) == 4916
    assert orc.select_count(100, 0.0) == 0
    assert orc.select_count(100, 1.0) == 100
    assert orc.select_count(100, 0.07) == 7        # 0.07*100 = 7.000000000000001 in binary
    assert orc.select_count(100, 2.0) == 100
    assert orc.select_count(0, 0.5) == 0


def test_select_against_full_sort():
    r = _rng(7)
    s = r.random(200)
    for n in (0, 1, 17, 199, 200):
        ranked = sorted(range(200), key=lambda j: (-s[j], j))[:n]
        got = orc.select(s, n)
        assert list(got) == sorted(ranked)
        assert len(got) == n and np.all(np.diff(got) > 0)


def test_select_ties_go_to_lower_index():
    s = np.array([0.5, 0.9, 0.5, 0.5, 0.1, 0.9])
    assert list(orc.select(s, 2)) == [1, 5]
    assert list(orc.select(s, 3)) == [0, 1, 5]
    assert list(orc.select(s, 4)) == [0, 1, 2, 5]
    assert list(orc.select(np.zeros(6), 3)) == [0, 1, 2]
    assert list(orc.select(s, 6)) == [0, 1, 2, 3, 4, 5]
    assert list(orc.select(s, 0)) == []


def test_select_uses_values_not_magnitudes():
    # fp32 inputs, as the GPU produces them, keep their order
    s = np.array([1e-5, 3e-5, 2e-5, 0.0], dtype=np.float32)
    assert list(orc.select(s, 2)) == [1, 2]


# ------------------------------------------------------------------ scores over several layers

def _layers(seed, L=3, R=5, H=4, Hkv=2, d=8, T=23):
    r = np.random.default_rng(seed)
    return [r.standard_normal((R, H, d)) for _ in range(L)], [r.standard_normal((T, Hkv, d)) for _ in range(L)]


def test_score_layers_mass_and_special_cases():
    qs, ks = _layers(70)
    s = orc.score_layers(qs, ks)
    assert np.isclose(s.sum(), 1.0) and np.all(s >= 0)                    # a mean of distributions
    w = [0.5, 2.0, 0.25]
    assert np.isclose(orc.score_layers(qs, ks, w).sum(), sum(w))          # every layer carries unit mass
    assert np.allclose(orc.score_layers(qs[:1], ks[:1], [1.0]), orc.score(qs[0], ks[0]))     # one layer = the score
    assert np.allclose(orc.score_layers([qs[0]] * 4, [ks[0]] * 4), orc.score(qs[0], ks[0]))  # equal layers: the mean
    # the last-layer selector is the single term of the last layer
    assert np.allclose(orc.score_layers(qs, ks, [0.0, 0.0, 1.0]), orc.score(qs[2], ks[2]))


def test_score_layers_is_linear_in_the_weights_and_ranking_ignores_scale():
    qs, ks = _layers(71)
    w1, w2 = np.array([0.2, 0.3, 0.5]), np.array([1.0, 0.0, 0.4])
    assert np.allclose(orc.score_layers(qs, ks, w1 + w2), orc.score_layers(qs, ks, w1) + orc.score_layers(qs, ks, w2))
    a, b = orc.score_layers(qs, ks, w1), orc.score_layers(qs, ks, 37.5 * w1)
    for n in (1, 5, 11, 23):
        assert np.array_equal(orc.select(a, n), orc.select(b, n))


def test_score_layers_closed_form_two_layers():
    # layer 0: all keys equal -> uniform 1/T whatever the probes; layer 1: one probe row, one head, logits known
    T, d = 6, 4
    k0 = np.tile(np.array([0.3, -1.0, 2.0, 0.5]), (T, 1, 1))
    q0 = np.random.default_rng(72).standard_normal((3, 2, d))
    q1 = np.zeros((1, 1, d)); q1[0, 0, 0] = 2.0                              # logit_j = 2 * k1[j, 0, 0] / sqrt(4) = k1[j,0,0]
    k1 = np.zeros((T, 1, d)); k1[:, 0, 0] = np.array([0.0, 1.0, -1.0, 2.0, 0.5, -0.5])
    e = np.exp(k1[:, 0, 0])
    ref = 0.25 * np.full(T, 1.0 / T) + 3.0 * e / e.sum()
    assert np.allclose(orc.score_layers([q0, q1], [k0, k1], [0.25, 3.0]), ref, atol=1e-14)

