"""Stage-wise GPU parity: every library call against the matching oracle step on identical
seeded inputs, through the C ABI (ctypes binding).  Sizes span several tiles and ragged tails."""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import qcf_oracle as orc
from paper_2604_08585_amd import binding as qb
from paper_2604_08585_amd import inputs, pipeline
from gpu_util import (DEV, SCORE_REL, TOL, assert_close, assert_indices_match, i32, i64, max_abs, quantizer, run_rerope, to_dev,
                            to_np)

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def shape_bf16(d_model=512, H=8, Hkv=2, D=128, base=500000.0, style=0):
    return inputs.LayerShape(d_model, H, Hkv, D, base, "bf16", style)


def shape_f32(d_model=256, H=4, Hkv=2, D=64, base=10000.0, style=0):
    return inputs.LayerShape(d_model, H, Hkv, D, base, "f32", style)


def rnd(rng, shape, dtype, std=1.0):
    return inputs.round_to_dtype(rng.standard_normal(shape).astype(np.float32) * std, dtype)


# ------------------------------------------------------------------ rerope

@pytest.mark.parametrize("sh", [shape_f32(), shape_f32(style=1), shape_bf16(), shape_bf16(style=1),
                                shape_bf16(D=64), shape_f32(D=128, Hkv=1, H=2), shape_bf16(Hkv=3, H=3)],
                         ids=["f32", "f32-il", "bf16", "bf16-il", "bf16-d64", "f32-d128", "bf16-hkv3"])
def test_rerope_ragged(sh):
    rng = np.random.default_rng(1)
    lens = [1, 37, 128, 5, 300, 64, 2]
    chunks = [(rnd(rng, (n, sh.n_kv_heads, sh.head_dim), sh.dtype), rnd(rng, (n, sh.n_kv_heads, sh.head_dim), sh.dtype))
              for n in lens]
    rows = np.concatenate([[0], np.cumsum(lens)])[:-1]
    pos0 = rows + 0
    src0 = [0, 3, 0, 0, 7, 0, 11]
    say(f"rerope {sh}")
    kf, vf = run_rerope(sh, chunks, rows.tolist(), pos0.tolist(), int(sum(lens)), src_pos0=src0)
    rk, rv = orc.rerope([c[0] for c in chunks], [c[1] for c in chunks],
                        [int(p) - s for p, s in zip(pos0, src0)], sh.rope_base, sh.rope_style)
    assert_close(to_np(kf), rk, sh.dtype, "k_fused")
    assert np.array_equal(to_np(vf), rv), "values must be copied bit-exactly"
    if sh.dtype == "bf16":      # tighter: one bf16 rounding of an fp32-accurate result
        assert np.all(np.abs(to_np(kf) - rk) <= 2.0 ** -8 * np.abs(rk) + 1e-6)


def test_rerope_large_shift_and_gaps():
    """Shifts of tens of thousands of positions need float64 angles; rows no chunk covers stay untouched."""
    sh = shape_f32()
    rng = np.random.default_rng(2)
    chunks = [(rnd(rng, (40, 2, 64), "f32"), rnd(rng, (40, 2, 64), "f32")) for _ in range(3)]
    rows, pos0 = [5, 60, 130], [32000, 500000, 7]
    pre = (rnd(rng, (200, 2, 64), "f32"), rnd(rng, (200, 2, 64), "f32"))
    kf, vf = run_rerope(sh, chunks, rows, pos0, 200, prefill=pre)
    exp_k, exp_v = pre[0].astype(np.float64).copy(), pre[1].astype(np.float64).copy()
    for (k, v), r, p in zip(chunks, rows, pos0):
        ek, _ = orc.rerope([k], None, [p], sh.rope_base)
        exp_k[r:r + 40], exp_v[r:r + 40] = ek, v
    assert_close(to_np(kf), exp_k, "f32", "k_fused")
    assert max_abs(to_np(kf), exp_k) < 2e-6
    assert np.array_equal(to_np(vf), exp_v)


def test_rerope_keys_only_and_empty():
    sh = shape_bf16()
    rng = np.random.default_rng(3)
    k = rnd(rng, (70, 2, 128), "bf16")
    kf, vf = run_rerope(sh, [(k, k)], [0], [1234], 70, with_v=False)
    ek, _ = orc.rerope([k], None, [1234], sh.rope_base)
    assert_close(to_np(kf), ek, "bf16", "k_fused")
    assert torch.count_nonzero(vf).item() == 0           # v_fused = NULL: values not written
    desc = qb.make_desc(sh)
    qb.qcf_rerope(desc, torch.zeros(0, dtype=torch.uint8, device=DEV), 0, 0, kf, None)   # no chunks: no-op


@pytest.mark.parametrize("seed", range(6))
def test_rerope_random_layout(seed):
    # seeded sweep: chunk counts on both sides of the single-kernel limit (256 table entries), lengths from 1,
    # gaps between chunks, arbitrary local and global start positions, both pair conventions and dtypes
    rng = np.random.default_rng(500 + seed)
    dtype = "bf16" if seed % 2 == 0 else "f32"
    Hkv = int(rng.choice([1, 2, 3, 8]))
    D = 128 if dtype == "bf16" else int(rng.choice([64, 128]))
    sh = inputs.LayerShape(256, Hkv, Hkv, D, float(rng.choice([10000.0, 500000.0])), dtype, int(seed % 3 == 0))
    n_chunks = int(rng.choice([1, 3, 40, 300]))
    lens = rng.integers(1, 6 if n_chunks > 100 else 90, size=n_chunks)
    gaps = rng.integers(0, 3, size=n_chunks) * (rng.random(n_chunks) < 0.2)
    rows = np.cumsum(np.concatenate([[0], (lens + gaps)[:-1]])) + int(gaps[0])
    total = int(rows[-1] + lens[-1] + 2)
    pos0 = rng.integers(0, 60000, size=n_chunks)
    src0 = rng.integers(0, 500, size=n_chunks)
    say(f"rerope random: {dtype} Hkv={Hkv} D={D} chunks={n_chunks} rows={total} style={sh.rope_style}")
    chunks = [(rnd(rng, (int(n), Hkv, D), dtype), rnd(rng, (int(n), Hkv, D), dtype)) for n in lens]
    pre = (rnd(rng, (total, Hkv, D), dtype), rnd(rng, (total, Hkv, D), dtype))
    kf, vf = run_rerope(sh, chunks, rows.tolist(), pos0.tolist(), total, src_pos0=src0.tolist(), prefill=pre)
    exp_k, exp_v = pre[0].astype(np.float64).copy(), pre[1].astype(np.float64).copy()
    for (k, v), r, p, s0 in zip(chunks, rows, pos0, src0):
        ek, _ = orc.rerope([k], None, [int(p) - int(s0)], sh.rope_base, sh.rope_style)
        exp_k[r:r + len(k)], exp_v[r:r + len(k)] = ek, v
    assert_close(to_np(kf), exp_k, dtype, "k_fused")
    assert np.array_equal(to_np(vf), exp_v)


# ------------------------------------------------------------------ score

def _score_case(sh, T_list, R_list, seed, limit=None, q_std=1.0):
    rng = np.random.default_rng(seed)
    dt = inputs.torch_dtype(sh.dtype)
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    qs = [rnd(rng, (R, H, D), sh.dtype, std=q_std) for R in R_list]
    ks = [rnd(rng, (T, Hkv, D), sh.dtype) for T in T_list]
    # make a few tokens stand out so that the softmax is far from uniform
    for q, k in zip(qs, ks):
        if k.shape[0] > 3 and q.shape[0] > 0:
            hot = rng.choice(k.shape[0], size=max(1, k.shape[0] // 50), replace=False)
            qbar = q.astype(np.float64).reshape(q.shape[0], Hkv, H // Hkv, D).mean(axis=(0, 2))
            k[hot] = inputs.round_to_dtype(3.0 * qbar[None] + 0.5 * rng.standard_normal((len(hot), Hkv, D)), sh.dtype)
    B = len(T_list)
    ctx_off = np.concatenate([[0], np.cumsum(T_list)])
    probe_off = np.concatenate([[0], np.cumsum(R_list)])
    q_all = np.concatenate(qs) if sum(R_list) else np.zeros((0, H, D), np.float32)
    k_all = np.concatenate(ks)
    score = torch.full((int(ctx_off[-1]),), -1.0, dtype=torch.float32, device=DEV)
    lim_dev = None
    if limit is not None:
        lim_dev = i32(np.concatenate(limit))
    qb.qcf_score(qb.make_desc(sh), B, to_dev(q_all, dt) if q_all.size else torch.zeros(8, dtype=dt, device=DEV),
                 i64(probe_off), int(probe_off[-1]), to_dev(k_all, dt), i64(ctx_off), int(ctx_off[-1]), lim_dev, score)
    torch.cuda.synchronize()
    got = to_np(score)
    for b in range(B):
        ref = orc.score(qs[b], ks[b], None if limit is None else limit[b])
        g = got[ctx_off[b]:ctx_off[b + 1]]
        assert max_abs(g, ref) <= 1e-4, f"request {b}: abs"
        assert np.all(np.abs(g - ref) <= SCORE_REL * ref + 1e-12), \
            f"request {b}: rel err {np.max(np.abs(g - ref) / np.maximum(ref, 1e-30)):.3e}"
        if R_list[b] > 0 and limit is None:
            assert abs(g.sum() - 1.0) < 1e-4
    return got


@pytest.mark.parametrize("sh", [shape_f32(), shape_bf16(), shape_bf16(H=32, Hkv=8, d_model=1024),
                                shape_bf16(D=64), shape_bf16(H=4, Hkv=4)],
                         ids=["f32", "bf16-g4", "bf16-llama", "bf16-d64-generic", "bf16-mha"])
def test_score_single_request(sh):
    say(f"score {sh}")
    _score_case(sh, [777], [20], seed=10)


def test_score_bf16_many_rows_and_tiles():
    # 81 probe rows x G=8 = 648 rows of one group: more than one staged row block; 1500 tokens: ragged tiles
    sh = shape_bf16(H=16, Hkv=2, d_model=1024)
    _score_case(sh, [1500], [81], seed=11)


def test_score_batch_ragged():
    sh = shape_bf16(H=8, Hkv=2)
    _score_case(sh, [300, 1, 64, 1025, 256], [5, 3, 0, 17, 40], seed=12)
    _score_case(shape_f32(), [100, 7, 260], [4, 2, 9], seed=13)


def test_score_probe_limit():
    sh = shape_bf16(H=8, Hkv=2)
    lim = [np.array([0, 10, 300, 64, 65, 999], dtype=np.int32), np.array([1, 130], dtype=np.int32)]
    _score_case(sh, [300, 200], [6, 2], seed=14, limit=lim)
    _score_case(shape_f32(), [300, 200], [6, 2], seed=15, limit=lim)


def test_score_deterministic():
    sh = shape_bf16(H=8, Hkv=2)
    a = _score_case(sh, [2000], [33], seed=16)
    b = _score_case(sh, [2000], [33], seed=16)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("sh,T_list,R_list", [(shape_bf16(H=8, Hkv=2), [900], [24]),               # single-kernel path
                                              (shape_bf16(H=16, Hkv=2), [1500], [81]),             # two-pass path
                                              (shape_bf16(H=8, Hkv=2), [300, 64, 1025], [5, 0, 17]),
                                              (shape_f32(), [260, 100], [9, 4])],
                         ids=["bf16-fused", "bf16-two-pass", "bf16-batch", "f32"])
def test_score_accumulated_over_layers(sh, T_list, R_list):
    # the all-layer selector: one accumulate call per layer into one buffer, against the oracle's weighted sum;
    # then the ranking made from it
    rng = np.random.default_rng(90)
    dt = inputs.torch_dtype(sh.dtype)
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    n_layers, weights = 3, [0.5, 0.2, 0.3]
    qs = [[rnd(rng, (R, H, D), sh.dtype) for R in R_list] for _ in range(n_layers)]
    ks = [[rnd(rng, (T, Hkv, D), sh.dtype) for T in T_list] for _ in range(n_layers)]
    ctx_off = np.concatenate([[0], np.cumsum(T_list)])
    probe_off = np.concatenate([[0], np.cumsum(R_list)])
    probes = [to_dev(np.concatenate(q), dt) for q in qs]
    keys = [to_dev(np.concatenate(k), dt) for k in ks]
    got = to_np(pipeline.score_over_layers(qb.make_desc(sh), probes, keys, i64(probe_off), i64(ctx_off), weights))
    torch.cuda.synchronize()
    for b in range(len(T_list)):
        g = got[ctx_off[b]:ctx_off[b + 1]]
        if R_list[b] == 0:
            assert np.all(g == 0)
            continue
        ref = orc.score_layers([qs[l][b] for l in range(n_layers)], [ks[l][b] for l in range(n_layers)], weights)
        assert np.all(np.abs(g - ref) <= SCORE_REL * ref + 1e-12), f"request {b}"
        assert abs(g.sum() - sum(weights)) < 1e-4
        n = orc.select_count(T_list[b], 0.2)
        sel = torch.empty(n, dtype=torch.int32, device=DEV)
        sc = torch.from_numpy(g.astype(np.float32)).to(DEV)
        qb.qcf_select(1, sc, i64([0, T_list[b]]), T_list[b], i64([0, n]), n, None, sel, None, None)
        assert_indices_match(sel.cpu().numpy(), ref, n, f"request {b}")
    # beta = 0 never reads the buffer: a buffer of NaNs gives the single-layer score
    T, R = T_list[0], R_list[0]
    score = torch.full((int(ctx_off[-1]),), float("nan"), dtype=torch.float32, device=DEV)
    qb.qcf_score_accumulate(qb.make_desc(sh), len(T_list), probes[0], i64(probe_off), int(probe_off[-1]), keys[0],
                            i64(ctx_off), int(ctx_off[-1]), None, 1.0, 0.0, score)
    ref0 = orc.score(qs[0][0], ks[0][0])
    g0 = to_np(score)[:T]
    assert np.all(np.abs(g0 - ref0) <= SCORE_REL * ref0 + 1e-12)


# ------------------------------------------------------------------ select

def _select_case(scores_list, n_list, pos0=None):
    B = len(scores_list)
    T_list = [len(s) for s in scores_list]
    ctx_off = np.concatenate([[0], np.cumsum(T_list)])
    sel_off = np.concatenate([[0], np.cumsum(n_list)])
    total_sel = int(sel_off[-1])
    sc = torch.from_numpy(np.concatenate(scores_list).astype(np.float32)).to(DEV)
    idx = torch.full((max(total_sel, 1),), -7, dtype=torch.int32, device=DEV)
    row = torch.full((max(total_sel, 1),), -7, dtype=torch.int32, device=DEV)
    pos = torch.full((max(total_sel, 1),), -7, dtype=torch.int32, device=DEV)
    qb.qcf_select(B, sc, i64(ctx_off), int(ctx_off[-1]), i64(sel_off), total_sel,
                  None if pos0 is None else i32(pos0), idx, row, pos)
    torch.cuda.synchronize()
    idx, row, pos = idx.cpu().numpy(), row.cpu().numpy(), pos.cpu().numpy()
    for b in range(B):
        n = min(n_list[b], T_list[b])
        ref = orc.select(scores_list[b].astype(np.float32), n)
        g = idx[sel_off[b]:sel_off[b] + n]
        assert np.array_equal(g, ref), f"request {b}: T={T_list[b]} N={n}"
        assert np.array_equal(row[sel_off[b]:sel_off[b] + n], ref + ctx_off[b])
        assert np.array_equal(pos[sel_off[b]:sel_off[b] + n], ref + (0 if pos0 is None else pos0[b]))


@pytest.mark.parametrize("T", [1, 2, 63, 1000, 8192, 8193, 20000, 32768, 40000])
def test_select_sizes(T):
    rng = np.random.default_rng(T)
    s = rng.random(T).astype(np.float32) ** 4 / T          # skewed, magnitude ~1/T like real scores
    for n in sorted({0, 1, T // 7, int(math.ceil(0.15 * T)), T - 1, T}):
        if n < 0:
            continue
        say(f"select T={T} N={n}")
        _select_case([s], [n])


def test_select_ties_and_special_values():
    rng = np.random.default_rng(5)
    vals = np.array([0.0, 1e-30, 1e-5, 0.25, 0.25, 0.5, 1.0], dtype=np.float32)
    s = rng.choice(vals, size=3000).astype(np.float32)
    for n in (1, 10, 400, 1500, 2999):
        _select_case([s], [n])
    _select_case([np.zeros(5000, np.float32)], [77])              # all equal: the first N indices
    _select_case([np.full(9000, 0.125, np.float32)], [8999])
    s2 = np.concatenate([np.full(4000, 0.5), np.full(4000, 0.25)]).astype(np.float32)
    _select_case([s2], [4001])
    _select_case([np.array([-1.0, 2.0, -0.0, 0.0, -3.0, 2.0], np.float32)], [3])   # signed keys still order correctly


def test_select_batch_and_positions():
    rng = np.random.default_rng(6)
    scores = [rng.random(t).astype(np.float32) for t in (100, 1, 3000, 17, 8192)]
    _select_case(scores, [15, 1, 450, 0, 1229], pos0=[0, 50, 7, 1000, 3])
    _select_case(scores, [15, 5, 450, 30, 1229])       # N_b larger than T_b is clamped


# ------------------------------------------------------------------ qkv

def _qkv_case(sh, M, x_rows, seed, gather=True, outputs=(True, True, True), max_pos=40000):
    rng = np.random.default_rng(seed)
    dt = inputs.torch_dtype(sh.dtype)
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    x = rnd(rng, (x_rows, sh.d_model), sh.dtype)
    w = rnd(rng, (sh.qkv_rows, sh.d_model), sh.dtype, std=1 / math.sqrt(sh.d_model))
    g = np.sort(rng.choice(x_rows, size=M, replace=False)).astype(np.int32) if gather else np.arange(M, dtype=np.int32)
    pos = np.sort(rng.integers(0, max_pos, size=M)).astype(np.int32)
    q = torch.full((M, H, D), 7.0, dtype=dt, device=DEV) if outputs[0] else None
    k = torch.full((M, Hkv, D), 7.0, dtype=dt, device=DEV) if outputs[1] else None
    v = torch.full((M, Hkv, D), 7.0, dtype=dt, device=DEV) if outputs[2] else None
    qb.qcf_recompute_qkv(qb.make_desc(sh), to_dev(x, dt), x_rows, i32(g) if gather else None, M, to_dev(w, dt),
                         i32(pos), q, k, v)
    torch.cuda.synchronize()
    rq, rk, rv = orc.recompute_qkv(x[g], w, pos, H, Hkv, D, sh.rope_base, sh.rope_style)
    for t, r, name in ((q, rq, "q"), (k, rk, "k"), (v, rv, "v")):
        if t is not None:
            assert_close(to_np(t), r, sh.dtype, f"{name} ({sh.dtype}, M={M})")
            if sh.dtype == "bf16":
                assert np.all(np.abs(to_np(t) - r) <= 2.0 ** -8 * np.abs(r) + 2e-4)


@pytest.mark.parametrize("sh,M", [(shape_f32(), 77), (shape_f32(style=1), 50), (shape_bf16(), 77),
                                  (shape_bf16(style=1), 130), (shape_bf16(d_model=1024, H=32, Hkv=8), 615),
                                  (shape_bf16(D=64, H=8, Hkv=4), 100), (shape_bf16(d_model=520), 33)],
                         ids=["f32", "f32-il", "bf16", "bf16-il", "bf16-llama-heads", "bf16-d64", "bf16-generic-dmodel"])
def test_qkv(sh, M):
    say(f"qkv {sh} M={M}")
    _qkv_case(sh, M, 900, seed=20)


def test_qkv_large_tile_config_and_partial_outputs():
    # enough row tiles that the 256-row tile configuration is chosen (200 tiles of 256 x 128)
    sh = shape_bf16(d_model=256, H=32, Hkv=8, D=128)
    _qkv_case(sh, 256 * 4 + 19, 1300, seed=21)
    _qkv_case(sh, 256 * 17 + 5, 5000, seed=24)     # 18 row tiles: the workgroup order that deals row tiles to the XCDs
    _qkv_case(shape_bf16(), 40, 40, seed=22, gather=False, outputs=(True, False, False))   # probe rows: Q only
    _qkv_case(shape_bf16(), 70, 100, seed=23, outputs=(False, True, True))


@pytest.mark.parametrize("style", [0, 1])
def test_qkv_large_positions(style):
    # the projection's epilogue forms the rotation itself: positions near and beyond 2^24 (where a float no
    # longer holds the position exactly) up to the largest position the interface takes, both pair styles,
    # small and large row tiles
    sh = shape_bf16(d_model=256, H=32, Hkv=8, D=128, style=style)
    for M, max_pos in ((90, 1 << 20), (90, (1 << 24) + 4096), (1100, (1 << 30) - 1)):
        _qkv_case(sh, M, M + 10, seed=24 + M, max_pos=max_pos)
    rng = np.random.default_rng(31)
    pos = np.array([0, 1, (1 << 24) - 1, 1 << 24, (1 << 24) + 1, (1 << 30) - 1, 123456789, 8191], dtype=np.int32)
    M = len(pos)
    x = rnd(rng, (M, sh.d_model), "bf16")
    w = rnd(rng, (sh.qkv_rows, sh.d_model), "bf16", std=1 / math.sqrt(sh.d_model))
    q = torch.zeros((M, sh.n_q_heads, sh.head_dim), dtype=torch.bfloat16, device=DEV)
    qb.qcf_recompute_qkv(qb.make_desc(sh), to_dev(x, torch.bfloat16), M, None, M, to_dev(w, torch.bfloat16), i32(pos),
                         q, None, None)
    torch.cuda.synchronize()
    rq, _, _ = orc.recompute_qkv(x, w, pos, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.rope_base, style)
    assert np.all(np.abs(to_np(q) - rq) <= 2.0 ** -8 * np.abs(rq) + 2e-4)


def test_qkv_activation_matrix_beyond_4_gib():
    # rows are gathered from both sides of the 4 GiB line of x: byte offsets no longer fit 32 bits, so the
    # launcher must take the tiling that addresses x with 64-bit pointers
    sh = shape_bf16(d_model=256, H=32, Hkv=8, D=128)
    rng = np.random.default_rng(24)
    dt = inputs.torch_dtype(sh.dtype)
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    line = (1 << 32) // (sh.d_model * 2)                 # first row that starts at or beyond 4 GiB
    x_rows = line + 6000
    M = 256 * 4 + 19
    g = np.sort(np.concatenate([rng.choice(3000, size=M // 2, replace=False),
                                line - 200 + rng.choice(6200, size=M - M // 2, replace=False)])).astype(np.int32)
    say(f"qkv x beyond 4 GiB: x_rows={x_rows} M={M} rows past the line: {(g >= line).sum()}")
    xg = rnd(rng, (M, sh.d_model), sh.dtype)
    w = rnd(rng, (sh.qkv_rows, sh.d_model), sh.dtype, std=1 / math.sqrt(sh.d_model))
    pos = np.sort(rng.integers(0, 40000, size=M)).astype(np.int32)
    x_dev = torch.empty((x_rows, sh.d_model), dtype=dt, device=DEV)      # only the gathered rows are defined
    x_dev[torch.from_numpy(g.astype(np.int64)).to(DEV)] = to_dev(xg, dt)
    q = torch.full((M, H, D), 7.0, dtype=dt, device=DEV)
    k = torch.full((M, Hkv, D), 7.0, dtype=dt, device=DEV)
    v = torch.full((M, Hkv, D), 7.0, dtype=dt, device=DEV)
    qb.qcf_recompute_qkv(qb.make_desc(sh), x_dev, x_rows, i32(g), M, to_dev(w, dt), i32(pos), q, k, v)
    torch.cuda.synchronize()
    del x_dev
    rq, rk, rv = orc.recompute_qkv(xg, w, pos, H, Hkv, D, sh.rope_base, sh.rope_style)
    for t, r, name in ((q, rq, "q"), (k, rk, "k"), (v, rv, "v")):
        assert_close(to_np(t), r, sh.dtype, f"{name} (x beyond 4 GiB)")


# ------------------------------------------------------------------ scatter

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scatter(dtype):
    sh = shape_f32() if dtype == "f32" else shape_bf16()
    rng = np.random.default_rng(30)
    dt = inputs.torch_dtype(dtype)
    T, M, Hkv, D = 500, 77, sh.n_kv_heads, sh.head_dim
    kf, vf = rnd(rng, (T, Hkv, D), dtype), rnd(rng, (T, Hkv, D), dtype)
    kn, vn = rnd(rng, (M, Hkv, D), dtype), rnd(rng, (M, Hkv, D), dtype)
    rows = np.sort(rng.choice(T, size=M, replace=False)).astype(np.int32)
    dk, dv = to_dev(kf, dt), to_dev(vf, dt)
    desc = qb.make_desc(sh)
    qb.qcf_scatter(desc, to_dev(kn, dt), to_dev(vn, dt), i32(rows), M, dk, dv, T)
    torch.cuda.synchronize()
    rk, rv = orc.scatter(kf, vf, kn, vn, rows)
    assert np.array_equal(to_np(dk), rk) and np.array_equal(to_np(dv), rv)
    qb.qcf_scatter(desc, to_dev(kn, dt), to_dev(vn, dt), i32(rows), M, dk, dv, T)     # idempotent
    qb.qcf_scatter(desc, to_dev(kn, dt), to_dev(vn, dt), i32(rows), 0, dk, dv, T)     # nothing selected
    torch.cuda.synchronize()
    assert np.array_equal(to_np(dk), rk) and np.array_equal(to_np(dv), rv)


@pytest.mark.parametrize("sh,M", [(shape_f32(), 60), (shape_bf16(), 77), (shape_bf16(style=1), 300),
                                  (shape_bf16(d_model=256, H=32, Hkv=8), 256 * 4 + 19)],
                         ids=["f32-generic", "bf16-128-row-tiles", "bf16-il", "bf16-256-row-tiles"])
def test_qkv_scatter_in_one_call(sh, M):
    # projection and write-back in one call: outputs and cache equal those of the two separate calls bit for bit,
    # the cache rows equal the oracle's scatter of the oracle's K/V; destination rows outside the cache are skipped
    say(f"qkv+scatter {sh} M={M}")
    rng = np.random.default_rng(31)
    dt = inputs.torch_dtype(sh.dtype)
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    T = M + 200
    x = rnd(rng, (T, sh.d_model), sh.dtype)
    w = rnd(rng, (sh.qkv_rows, sh.d_model), sh.dtype, std=1 / math.sqrt(sh.d_model))
    rows = np.sort(rng.choice(T, size=M, replace=False)).astype(np.int32)
    pos = rows.copy()
    dst = rows.copy()
    dst[3] = -1                   # skipped
    dst[M - 2] = T + 5            # skipped
    kf, vf = rnd(rng, (T, Hkv, D), sh.dtype), rnd(rng, (T, Hkv, D), sh.dtype)
    desc = qb.make_desc(sh)
    dx, dw = to_dev(x, dt), to_dev(w, dt)
    # two calls
    q1 = torch.empty((M, H, D), dtype=dt, device=DEV); k1 = torch.empty((M, Hkv, D), dtype=dt, device=DEV); v1 = torch.empty_like(k1)
    kf1, vf1 = to_dev(kf, dt), to_dev(vf, dt)
    qb.qcf_recompute_qkv(desc, dx, T, i32(rows), M, dw, i32(pos), q1, k1, v1)
    qb.qcf_scatter(desc, k1, v1, i32(dst), M, kf1, vf1, T)
    # one call
    q2 = torch.full_like(q1, 7.0); k2 = torch.full_like(k1, 7.0); v2 = torch.full_like(v1, 7.0)
    kf2, vf2 = to_dev(kf, dt), to_dev(vf, dt)
    qb.qcf_recompute_qkv_scatter(desc, dx, T, i32(rows), M, dw, i32(pos), q2, k2, v2, i32(dst), kf2, vf2, T)
    torch.cuda.synchronize()
    for a, b, name in ((q1, q2, "q"), (k1, k2, "k"), (v1, v2, "v"), (kf1, kf2, "k_fused"), (vf1, vf2, "v_fused")):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), name
    rq, rk, rv = orc.recompute_qkv(x[rows], w, pos, H, Hkv, D, sh.rope_base, sh.rope_style)
    ok = (dst >= 0) & (dst < T)
    ek, ev = orc.scatter(kf, vf, rk[ok], rv[ok], dst[ok])
    assert_close(to_np(kf2), ek, sh.dtype, "k_fused vs oracle")
    assert_close(to_np(vf2), ev, sh.dtype, "v_fused vs oracle")
    untouched = np.setdiff1d(np.arange(T), dst[ok])
    assert np.array_equal(to_np(kf2)[untouched], kf[untouched]) and np.array_equal(to_np(vf2)[untouched], vf[untouched])
    assert_close(to_np(q2), rq, sh.dtype, "q")


# ------------------------------------------------------------------ attn

def _attn_case(sh, T_list, N_list, seed, pos0=None, probe_rows=0, q_std=1.0):
    rng = np.random.default_rng(seed)
    dt = inputs.torch_dtype(sh.dtype)
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    B = len(T_list)
    ks = [rnd(rng, (T, Hkv, D), sh.dtype) for T in T_list]
    vs = [rnd(rng, (T, Hkv, D), sh.dtype) for T in T_list]
    p0 = [0] * B if pos0 is None else pos0
    qs, poss = [], []
    for b in range(B):
        idx = np.sort(rng.choice(T_list[b], size=N_list[b], replace=False)) if N_list[b] else np.zeros(0, np.int64)
        pos = idx + p0[b]
        if probe_rows and b == 0:                  # rows after the context see every token
            pos = np.concatenate([pos, T_list[b] + p0[b] + np.arange(probe_rows)])
        poss.append(pos.astype(np.int32))
        qs.append(rnd(rng, (len(pos), H, D), sh.dtype, std=q_std))
    n_rows = [len(p) for p in poss]
    ctx_off = np.concatenate([[0], np.cumsum(T_list)])
    sel_off = np.concatenate([[0], np.cumsum(n_rows)])
    total_sel = int(sel_off[-1])
    o = torch.full((max(total_sel, 1), H, D), 9.0, dtype=dt, device=DEV)
    lse = torch.full((max(total_sel, 1), H), 9.0, dtype=torch.float32, device=DEV)
    qb.qcf_recompute_attn(qb.make_desc(sh), B, to_dev(np.concatenate(qs), dt), i32(np.concatenate(poss)), i64(sel_off),
                          total_sel, to_dev(np.concatenate(ks), dt), to_dev(np.concatenate(vs), dt), i64(ctx_off),
                          int(ctx_off[-1]), None if pos0 is None else i32(pos0), o, lse)
    torch.cuda.synchronize()
    go, gl = to_np(o), to_np(lse)
    for b in range(B):
        ro, rl = orc.recompute_attn(qs[b], poss[b], ks[b], vs[b], ctx_pos0=p0[b])
        sl = slice(sel_off[b], sel_off[b + 1])
        assert_close(go[sl], ro, sh.dtype, f"o request {b}")
        fin = np.isfinite(rl)
        assert np.array_equal(np.isfinite(gl[sl]), fin)
        assert max_abs(gl[sl][fin], rl[fin]) < 2e-3, "log-sum-exp"


@pytest.mark.parametrize("sh", [shape_f32(), shape_bf16(), shape_bf16(H=32, Hkv=8, d_model=1024),
                                shape_bf16(H=16, Hkv=2), shape_bf16(H=2, Hkv=2), shape_bf16(D=64)],
                         ids=["f32", "bf16-g4", "bf16-llama", "bf16-g8", "bf16-mha", "bf16-d64-generic"])
def test_attn_single_request(sh):
    say(f"attn {sh}")
    _attn_case(sh, [700], [105], seed=40)


def test_attn_ragged_batch_and_offsets():
    sh = shape_bf16()
    _attn_case(sh, [300, 1, 64, 1025], [45, 1, 10, 150], seed=41)
    _attn_case(sh, [300, 500], [45, 0], seed=42, pos0=[5, 100])
    _attn_case(shape_f32(), [300, 90], [45, 14], seed=43, pos0=[5, 0])


def test_attn_all_rows_and_probe_rows():
    sh = shape_bf16()
    _attn_case(sh, [257], [257], seed=44)                 # ratio 1: dense causal attention
    _attn_case(sh, [200], [30], seed=45, probe_rows=7)    # rows positioned after the context


def test_attn_row_before_context_sees_nothing():
    sh = shape_bf16()
    rng = np.random.default_rng(46)
    dt = torch.bfloat16
    k, v = rnd(rng, (50, 2, 128), "bf16"), rnd(rng, (50, 2, 128), "bf16")
    q = rnd(rng, (2, 8, 128), "bf16")
    o = torch.full((2, 8, 128), 9.0, dtype=dt, device=DEV)
    lse = torch.zeros((2, 8), dtype=torch.float32, device=DEV)
    qb.qcf_recompute_attn(qb.make_desc(sh), 1, to_dev(q, dt), i32([3, 12]), i64([0, 2]), 2, to_dev(k, dt), to_dev(v, dt),
                          i64([0, 50]), 50, i32([10]), o, lse)
    torch.cuda.synchronize()
    ro, rl = orc.recompute_attn(q, np.array([3, 12]), k, v, ctx_pos0=10)
    assert torch.count_nonzero(o[0]).item() == 0 and torch.isinf(lse[0]).all()
    assert_close(to_np(o), ro, "bf16", "o")


def test_attn_rows_in_any_order_and_repeated():
    # the call does not need ascending positions: shuffled rows, the same position twice
    sh = shape_bf16()
    rng = np.random.default_rng(47)
    T, H, Hkv, D = 900, sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    k, v = rnd(rng, (T, Hkv, D), "bf16"), rnd(rng, (T, Hkv, D), "bf16")
    pos = rng.permutation(T)[:130].astype(np.int32)
    pos[7] = pos[3]
    q = rnd(rng, (len(pos), H, D), "bf16")
    o = torch.full((len(pos), H, D), 9.0, dtype=torch.bfloat16, device=DEV)
    qb.qcf_recompute_attn(qb.make_desc(sh), 1, to_dev(q, torch.bfloat16), i32(pos), i64([0, len(pos)]), len(pos),
                          to_dev(k, torch.bfloat16), to_dev(v, torch.bfloat16), i64([0, T]), T, None, o, None)
    torch.cuda.synchronize()
    ro, _ = orc.recompute_attn(q, pos, k, v)
    assert_close(to_np(o), ro, "bf16", "o")


@pytest.mark.parametrize("seed", range(8))
def test_attn_random_geometry(seed):
    # seeded sweep over head grouping, batch, lengths, row counts and position offsets (MFMA and generic paths)
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 3, 4, 8, 16]))
    sh = shape_bf16(H=Hkv * G, Hkv=Hkv)
    B = int(rng.integers(1, 4))
    T_list = [int(rng.integers(1, 1400)) for _ in range(B)]
    N_list = [int(rng.integers(0, min(T, 160) + 1)) for T in T_list]
    pos0 = [int(rng.integers(0, 50)) for _ in range(B)]
    say(f"attn random: Hkv={Hkv} G={G} T={T_list} N={N_list} pos0={pos0}")
    _attn_case(sh, T_list, N_list, seed=2000 + seed, pos0=pos0, probe_rows=int(rng.integers(0, 5)))


@pytest.mark.parametrize("seed", range(6))
def test_score_random_geometry(seed):
    rng = np.random.default_rng(3000 + seed)
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 8]))
    sh = shape_bf16(H=Hkv * G, Hkv=Hkv)
    B = int(rng.integers(1, 4))
    T_list = [int(rng.integers(1, 1500)) for _ in range(B)]
    R_list = [int(rng.integers(0, 70)) for _ in range(B)]
    limit = None
    if seed % 2:
        limit = [rng.integers(0, T + 1, size=R).astype(np.int32) for T, R in zip(T_list, R_list)]
    say(f"score random: Hkv={Hkv} G={G} T={T_list} R={R_list} limit={'yes' if limit else 'no'}")
    _score_case(sh, T_list, R_list, seed=4000 + seed, limit=limit)


@pytest.mark.parametrize("seed", range(6))
def test_qkv_random_geometry(seed):
    # seeded sweep over row counts, model widths (multiples of 64 take the MFMA tilings, others the generic
    # kernel), head counts and gather on/off
    rng = np.random.default_rng(600 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4]))
    d_model = int(rng.choice([64, 192, 520, 1024, 2048]))
    sh = shape_bf16(d_model=d_model, H=Hkv * G, Hkv=Hkv, style=int(seed % 2))
    M = int(rng.integers(1, 900))
    x_rows = M + int(rng.integers(0, 300))
    say(f"qkv random: d_model={d_model} H={Hkv * G}/{Hkv} M={M} x_rows={x_rows}")
    _qkv_case(sh, M, x_rows, seed=700 + seed, gather=bool(seed % 3))


@pytest.mark.parametrize("q_std", [0.05, 4.0, 12.0], ids=["flat", "peaky", "one-hot"])
def test_attn_logit_range(q_std):
    # nearly uniform rows, and rows whose logits span hundreds of units: the running reference point of the
    # softmax moves many times along a row (its lazy update must stay exact)
    _attn_case(shape_bf16(), [1500], [140], seed=48, q_std=q_std)
    _attn_case(shape_f32(), [400], [40], seed=49, q_std=q_std)


@pytest.mark.parametrize("q_std", [0.05, 4.0], ids=["flat", "peaky"])
def test_score_logit_range(q_std):
    # nearly uniform softmax rows, and rows dominated by a handful of tokens (partial maxima that differ by
    # hundreds of units between tiles)
    _score_case(shape_bf16(H=8, Hkv=2), [1300], [21], seed=17, q_std=q_std)
    _score_case(shape_f32(), [300], [6], seed=18, q_std=q_std)


def test_attn_more_row_blocks_than_the_planner_holds():
    # 4200 row blocks (G = 16: 8 selected rows per block) exceed the split planner's table, so the launch must stay
    # unsplit; positions repeat and are unsorted; sampled rows against the oracle
    sh = shape_bf16(H=16, Hkv=1)
    rng = np.random.default_rng(50)
    T, N, H, D = 100, 4200 * 8, 16, 128
    k, v = rnd(rng, (T, 1, D), "bf16"), rnd(rng, (T, 1, D), "bf16")
    pos = rng.integers(0, T, size=N).astype(np.int32)
    q = rnd(rng, (N, H, D), "bf16")
    o = torch.full((N, H, D), 9.0, dtype=torch.bfloat16, device=DEV)
    qb.qcf_recompute_attn(qb.make_desc(sh), 1, to_dev(q, torch.bfloat16), i32(pos), i64([0, N]), N,
                          to_dev(k, torch.bfloat16), to_dev(v, torch.bfloat16), i64([0, T]), T, None, o, None)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, N - 1], rng.choice(N, size=300, replace=False)]))
    ro, _ = orc.recompute_attn(q[rows], pos[rows], k, v)
    assert_close(to_np(o[torch.from_numpy(rows).to(DEV)]), ro, "bf16", "o (sampled rows)")
