"""Two decoder layers chained on the GPU (critical layer with scoring and selection, then a second layer that
reuses the selection), user-query rows included, against the same chain of oracle steps with the storage
rounding of the element type after every stage."""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import qcf_oracle as orc
from paper_2604_08585_amd import binding as qb
from paper_2604_08585_amd import inputs, pipeline
from gpu_util import DEV, SCORE_REL, assert_close, assert_indices_match, i32, i64, quantizer, to_dev, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def rnd(rng, shp, std=1.0):
    return inputs.round_to_dtype(rng.standard_normal(shp).astype(np.float32) * std, "bf16")


def make_layer(rng, sh, F, lens):
    dm, hd = sh.d_model, sh.n_q_heads * sh.head_dim
    one = lambda n: inputs.round_to_dtype((1.0 + 0.1 * rng.standard_normal(n)).astype(np.float32), "bf16")
    return dict(g1=one(dm), w_qkv=rnd(rng, (sh.qkv_rows, dm), 1 / math.sqrt(dm)), w_o=rnd(rng, (dm, hd), 0.5 / math.sqrt(hd)),
                g2=one(dm), w_gu=rnd(rng, (2 * F, dm), 1 / math.sqrt(dm)), w_dn=rnd(rng, (dm, F), 0.5 / math.sqrt(F)),
                k_chunks=[rnd(rng, (n, sh.n_kv_heads, sh.head_dim)) for n in lens],
                v_chunks=[rnd(rng, (n, sh.n_kv_heads, sh.head_dim)) for n in lens])


def oracle_layer(sh, lw, lens, h_rows, rows, h_ctx_all, T, R, ratio, sel=None):
    """One layer in oracle steps.  Layer with sel=None is the critical one: h_ctx_all holds the hidden states of
    all context tokens followed by the query rows, and the selection is made here."""
    qz = quantizer("bf16")
    H, Hkv, D, base = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.rope_base
    dst = np.concatenate([[0], np.cumsum(lens)])[:-1]
    kf, vf = orc.rerope(lw["k_chunks"], lw["v_chunks"], list(dst), base)
    kf, vf = qz(kf), qz(vf)
    kf = np.concatenate([kf, np.zeros((R, Hkv, D))]); vf = np.concatenate([vf, np.zeros((R, Hkv, D))])
    out = {}
    if sel is None:
        x_all = qz(orc.rmsnorm(h_ctx_all, lw["g1"], 1e-5))
        qp, _, _ = orc.recompute_qkv(x_all[T:], lw["w_qkv"], T + np.arange(R), H, Hkv, D, base)
        out["score"] = orc.score(qz(qp), kf[:T])
        out["x_all"] = x_all
        return out, kf, vf
    x = qz(orc.rmsnorm(h_rows, lw["g1"], 1e-5))
    q, k, v = orc.recompute_qkv(x, lw["w_qkv"], rows, H, Hkv, D, base)
    kf, vf = orc.scatter(kf, vf, qz(k), qz(v), rows)
    o, _ = orc.recompute_attn(qz(q), rows, kf, vf)
    out["h"] = orc.layer_tail(h_rows, qz(o), lw["w_o"], lw["g2"], lw["w_gu"], lw["w_dn"], 1e-5, quantize=qz)
    return out, kf, vf


def gpu_rerope(sh, desc, lw, lens, T, R):
    """Fused K/V of the layer with R extra (zero) rows for the query tokens."""
    dt = torch.bfloat16
    Hkv, D = sh.n_kv_heads, sh.head_dim
    kf = torch.zeros((T + R, Hkv, D), dtype=dt, device=DEV)
    vf = torch.zeros((T + R, Hkv, D), dtype=dt, device=DEV)
    keep = [(to_dev(k, dt), to_dev(v, dt)) for k, v in zip(lw["k_chunks"], lw["v_chunks"])]
    table = (qb.ChunkDesc * len(lens))()
    row = 0
    for c, n in enumerate(lens):
        table[c] = qb.ChunkDesc(keep[c][0].data_ptr(), keep[c][1].data_ptr(), n, 0, row, row)
        row += n
    tab_dev = torch.frombuffer(bytearray(bytes(table)), dtype=torch.uint8).to(DEV)
    qb.qcf_rerope(desc, tab_dev, len(lens), T, kf, vf)
    torch.cuda.synchronize()          # the chunk caches and the table go out of scope here
    return kf, vf


def gpu_layer(sh, desc, lw, lens, h_rows_dev, rows, T, R):
    """rerope -> qkv on rmsnorm(h) of the rows -> scatter -> attn -> rest of the block, on the GPU."""
    dt = torch.bfloat16
    H, Hkv, D, dm = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.d_model
    M = len(rows)
    kf, vf = gpu_rerope(sh, desc, lw, lens, T, R)
    x = torch.empty((M, dm), dtype=dt, device=DEV)
    qb.qcf_rmsnorm(desc, h_rows_dev, to_dev(lw["g1"], dt), 1e-5, M, dm, x)
    q = torch.empty((M, H, D), dtype=dt, device=DEV)
    k = torch.empty((M, Hkv, D), dtype=dt, device=DEV)
    v = torch.empty((M, Hkv, D), dtype=dt, device=DEV)
    r32 = i32(rows)
    qb.qcf_recompute_qkv(desc, x, M, None, M, to_dev(lw["w_qkv"], dt), r32, q, k, v)
    qb.qcf_scatter(desc, k, v, r32, M, kf, vf, T + R)
    o = torch.empty((M, H, D), dtype=dt, device=DEV)
    qb.qcf_recompute_attn(desc, 1, q, r32, i64([0, M]), M, kf, vf, i64([0, T + R]), T + R, None, o, None)
    tw = pipeline.TailWeights(to_dev(lw["w_o"], dt), to_dev(lw["g2"], dt), to_dev(lw["w_gu"], dt),
                              to_dev(lw["w_dn"], dt), 1e-5)
    return pipeline.layer_tail(desc, h_rows_dev, o, tw), kf, vf


def test_two_layer_chain_with_query_rows():
    rng = np.random.default_rng(50)
    sh = inputs.LayerShape(512, 8, 2, 128, 500000.0, "bf16", 0)
    desc = qb.make_desc(sh)
    dt = torch.bfloat16
    F, lens, R, ratio = 1408, [200, 150, 250], 16, 0.2
    T = sum(lens)
    N = orc.select_count(T, ratio)
    layers = [make_layer(rng, sh, F, lens) for _ in range(2)]
    h_all = rnd(rng, (T + R, sh.d_model), 0.7)                    # layer-0 input: context tokens, then query rows
    say(f"two-layer chain: T={T} R={R} N={N}")

    # critical layer, analysis: probe rows = the query rows; scored against the re-rotated layer-0 keys
    ref0, _, _ = oracle_layer(sh, layers[0], lens, None, None, h_all, T, R, ratio)
    x_all = torch.empty((T + R, sh.d_model), dtype=dt, device=DEV)
    qb.qcf_rmsnorm(desc, to_dev(h_all, dt), to_dev(layers[0]["g1"], dt), 1e-5, T + R, sh.d_model, x_all)
    qp = torch.empty((R, sh.n_q_heads, sh.head_dim), dtype=dt, device=DEV)
    qb.qcf_recompute_qkv(desc, x_all[T:], R, None, R, to_dev(layers[0]["w_qkv"], dt), i32(T + np.arange(R)), qp, None, None)
    kf0, _ = gpu_rerope(sh, desc, layers[0], lens, T, R)
    score = torch.empty(T, dtype=torch.float32, device=DEV)
    qb.qcf_score(desc, 1, qp, i64([0, R]), R, kf0[:T].contiguous(), i64([0, T]), T, None, score)
    sel = torch.empty(N, dtype=torch.int32, device=DEV)
    qb.qcf_select(1, score, i64([0, T]), T, i64([0, N]), N, None, sel, None, None)
    torch.cuda.synchronize()
    g = to_np(score)
    assert np.all(np.abs(g - ref0["score"]) <= SCORE_REL * ref0["score"] + 1e-12)
    sel_np = sel.cpu().numpy().astype(np.int64)
    assert_indices_match(sel_np, ref0["score"], N, "critical layer")

    # reconstruction through two layers on the GPU's index set, query rows appended at positions T .. T+R-1
    rows = np.concatenate([sel_np, T + np.arange(R)])
    h_rows = h_all[rows]
    h_gpu = to_dev(h_rows, dt)
    h_ref = h_rows.astype(np.float64)
    for l, lw in enumerate(layers):
        h_gpu, kf, vf = gpu_layer(sh, desc, lw, lens, h_gpu, rows, T, R)
        out, rkf, rvf = oracle_layer(sh, lw, lens, h_ref, rows, None, T, R, ratio, sel=sel_np)
        torch.cuda.synchronize()
        h_ref = out["h"]
        got = to_np(h_gpu)
        err = np.abs(got - h_ref)
        say(f"  layer {l}: max abs err hidden {err.max():.3e}, fused K {np.abs(to_np(kf) - rkf).max():.3e}")
        assert np.abs(to_np(kf) - rkf).max() <= 2e-2 and np.abs(to_np(vf) - rvf).max() <= 2e-2
        # one element-type rounding step may differ per stage; it must not grow through the chain
        assert np.all(err <= 2e-2 + 2.0 ** -7 * np.abs(h_ref)), f"layer {l}"
        assert np.mean(err) < 2e-3


def test_chunk_caches_streamed_from_the_host_give_the_same_layers():
    """Layers whose chunk caches arrive over a copy stream (double-buffered): every streamed layer's patched K/V
    and attention rows against the oracle run on that layer's host caches (rerope -> qkv -> scatter -> attn on
    the critical layer's selection), and bit-identical to the same layers run one after the other with every
    copy awaited."""
    wl = inputs.make_config(1, orc.PlantOps(), scale=0.25)
    sh, req = wl.shape, wl.requests[0]
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    qz = quantizer(sh.dtype)
    L = pipeline.upload(wl, DEV)
    pipeline.enqueue_layer(L)                                   # critical layer: fixes the selection
    torch.cuda.synchronize()
    lens = [c.length for r in wl.requests for c in r.chunks]
    n_layers = 5
    host = pipeline.host_chunk_caches(L, seed=3, n_layers=n_layers)
    st = pipeline.ChunkStreamer(L, lens, host)
    results = {}
    for mode in (False, True):
        outs = []
        st.run(n_layers, after_layer=lambda i: outs.append((L.k_fused.clone(), L.v_fused.clone(), L.o_sel.clone())),
               overlap=mode)
        torch.cuda.synchronize()
        results[mode] = outs
    for i in range(n_layers):
        for j, what in enumerate(("fused K", "fused V", "O rows")):
            assert torch.equal(results[True][i][j], results[False][i][j]), f"{what}, layer {i}"

    # oracle on every layer's host caches, with the selection the critical layer made on the GPU
    n = L.total_sel
    idx = L.sel_idx[:n].cpu().numpy().astype(np.int64)
    assert n == orc.select_count(req.T, wl.ratio) and np.all(np.diff(idx) > 0)
    bounds = np.concatenate([[0], np.cumsum(lens)])
    q_s, k_s, v_s = orc.recompute_qkv(req.x_ctx[idx], wl.w_qkv, idx, H, Hkv, D, sh.rope_base, sh.rope_style)
    q_s, k_s, v_s = qz(q_s), qz(k_s), qz(v_s)
    for i in range(n_layers):
        hk, hv = to_np(host[i][0]), to_np(host[i][1])
        kc = [hk[bounds[c]:bounds[c + 1]] for c in range(len(lens))]
        vc = [hv[bounds[c]:bounds[c + 1]] for c in range(len(lens))]
        kf, vf = orc.rerope(kc, vc, [p - c.src_pos0 for p, c in zip(req.dst_pos0, req.chunks)], sh.rope_base,
                            sh.rope_style)
        kp, vp = orc.scatter(qz(kf), qz(vf), k_s, v_s, idx)
        o_ref, _ = orc.recompute_attn(q_s, idx, kp, vp)
        gk, gv, go = (to_np(t) for t in results[True][i])
        ek = assert_close(gk[:req.T], kp, sh.dtype, f"patched K, streamed layer {i}")
        ev = assert_close(gv[:req.T], vp, sh.dtype, f"patched V, streamed layer {i}")
        eo = assert_close(go[:n], qz(o_ref), sh.dtype, f"O rows, streamed layer {i}")
        say(f"  streamed layer {i}: max abs err K {ek:.3e} V {ev:.3e} O {eo:.3e}")
    # layer 0 streams the layer's own caches: the same result as the resident path
    pipeline.enqueue_layer(L, critical=False)
    torch.cuda.synchronize()
    assert torch.equal(results[True][0][2], L.o_sel)
    assert not torch.equal(results[True][1][2], results[True][0][2])     # other layers really hold other caches
