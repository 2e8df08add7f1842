"""GPU parity of the rest-of-the-layer calls (linear map with residual, RMSNorm, gated SiLU) and of the
user-query rows run as extra recomputed rows, against the CPU oracle on identical inputs."""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import qcf_oracle as orc
from paper_2604_08585_amd import binding as qb
from paper_2604_08585_amd import inputs, pipeline
from gpu_util import DEV, assert_close, i32, i64, quantizer, to_dev, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def shape(dtype):
    return inputs.LayerShape(256, 4, 2, 64, 10000.0, dtype, 0)       # only the dtype matters for these calls


def rnd(rng, shp, dtype, std=1.0):
    return inputs.round_to_dtype(rng.standard_normal(shp).astype(np.float32) * std, dtype)


def tight(got, ref, dtype, what):
    """One rounding of the stored element type on top of fp32 accumulation."""
    rel, ab = (2.0 ** -8, 2e-4) if dtype == "bf16" else (2e-6, 2e-6)
    bad = np.abs(got - ref) > rel * np.abs(ref) + ab
    assert not bad.any(), f"{what}: {bad.sum()} elements off, worst {np.abs(got - ref).max():.3e}"


@pytest.mark.parametrize("dtype,M,K,N,res", [
    ("bf16", 77, 256, 256, "none"), ("bf16", 77, 256, 256, "separate"), ("bf16", 130, 512, 384, "alias"),
    ("bf16", 256 * 4 + 19, 512, 6144, "separate"),     # enough 256-row tiles for the load/compute-split kernel
    ("bf16", 256 * 4 + 19, 1024, 6144, "none"),
    ("bf16", 33, 72, 40, "separate"),                   # shapes the MFMA tiling does not cover
    ("f32", 50, 40, 24, "alias"), ("f32", 70, 256, 128, "none")])
def test_linear(dtype, M, K, N, res):
    say(f"linear {dtype} M={M} K={K} N={N} residual={res}")
    rng = np.random.default_rng(40)
    dt = inputs.torch_dtype(dtype)
    x, w = rnd(rng, (M, K), dtype), rnd(rng, (N, K), dtype, std=1 / math.sqrt(K))
    r = rnd(rng, (M, N), dtype) if res != "none" else None
    out = torch.full((M, N), 7.0, dtype=dt, device=DEV)
    r_dev = None
    if res == "separate":
        r_dev = to_dev(r, dt)
    elif res == "alias":
        out.copy_(to_dev(r, dt))
        r_dev = out
    qb.qcf_linear(qb.make_desc(shape(dtype)), to_dev(x, dt), M, K, to_dev(w, dt), N, r_dev, out)
    torch.cuda.synchronize()
    ref = orc.linear(x, w, r)
    assert_close(to_np(out), ref, dtype, "linear")
    tight(to_np(out), ref, dtype, "linear")


@pytest.mark.parametrize("dtype,M,cols", [("f32", 9, 256), ("bf16", 300, 4096), ("bf16", 5, 16384), ("bf16", 3, 24)])
def test_rmsnorm(dtype, M, cols):
    say(f"rmsnorm {dtype} M={M} cols={cols}")
    rng = np.random.default_rng(41)
    dt = inputs.torch_dtype(dtype)
    # outputs stay below 8, where a bf16 half-ulp (0.0156) is inside the 2e-2 bar
    x = rnd(rng, (M, cols), dtype, std=1.7)
    g = inputs.round_to_dtype((1.0 + 0.1 * rng.standard_normal(cols)).astype(np.float32), dtype)
    xd = to_dev(x, dt)
    out = torch.empty_like(xd)
    desc = qb.make_desc(shape(dtype))
    qb.qcf_rmsnorm(desc, xd, to_dev(g, dt), 1e-5, M, cols, out)
    qb.qcf_rmsnorm(desc, xd, to_dev(g, dt), 1e-5, M, cols, xd)          # in place
    torch.cuda.synchronize()
    ref = orc.rmsnorm(x, g, 1e-5)
    assert_close(to_np(out), ref, dtype, "rmsnorm")
    tight(to_np(out), ref, dtype, "rmsnorm")
    assert torch.equal(out, xd)


@pytest.mark.parametrize("dtype,M,F", [("f32", 7, 40), ("bf16", 300, 2816), ("bf16", 2, 8)])
def test_swiglu(dtype, M, F):
    say(f"swiglu {dtype} M={M} F={F}")
    rng = np.random.default_rng(42)
    dt = inputs.torch_dtype(dtype)
    gu = rnd(rng, (M, 2 * F), dtype, std=2.0)
    out = torch.empty((M, F), dtype=dt, device=DEV)
    qb.qcf_swiglu(qb.make_desc(shape(dtype)), to_dev(gu, dt), M, F, out)
    torch.cuda.synchronize()
    ref = orc.swiglu(gu)
    small = np.abs(ref) < 8.0                     # above 8 a bf16 half-ulp alone exceeds the absolute bar
    assert_close(to_np(out)[small], ref[small], dtype, "swiglu")
    tight(to_np(out), ref, dtype, "swiglu")


@pytest.mark.parametrize("dtype,M,dm,hd,F", [("f32", 40, 256, 256, 344), ("bf16", 615, 1024, 1024, 2816)])
def test_layer_tail_chain(dtype, M, dm, hd, F):
    """The five calls chained (each stage stores its result in the element type) against the oracle's block
    with the same storage rounding after every stage."""
    say(f"layer tail {dtype} M={M} d_model={dm} F={F}")
    rng = np.random.default_rng(43)
    dt = inputs.torch_dtype(dtype)
    H, d = hd // 64, 64
    h_in, o = rnd(rng, (M, dm), dtype, std=0.5), rnd(rng, (M, H, d), dtype)
    w_o = rnd(rng, (dm, hd), dtype, std=0.5 / math.sqrt(hd))
    g = rnd(rng, (dm,), dtype, std=0.2) + inputs.round_to_dtype(np.ones(dm, np.float32), dtype)
    g = inputs.round_to_dtype(g.astype(np.float32), dtype)
    w_gu = rnd(rng, (2 * F, dm), dtype, std=1 / math.sqrt(dm))
    w_dn = rnd(rng, (dm, F), dtype, std=0.5 / math.sqrt(F))
    tw = pipeline.TailWeights(to_dev(w_o, dt), to_dev(g, dt), to_dev(w_gu, dt), to_dev(w_dn, dt), 1e-5)
    out = pipeline.layer_tail(qb.make_desc(shape(dtype)), to_dev(h_in, dt), to_dev(o, dt), tw)
    torch.cuda.synchronize()
    ref = orc.layer_tail(h_in, o, w_o, g, w_gu, w_dn, 1e-5, quantize=quantizer(dtype))
    assert np.abs(ref).max() < 8.0                        # the bf16 bar is only meaningful below 8
    err = assert_close(to_np(out), ref, dtype, "layer tail")
    say(f"  max abs err {err:.3e}")


def test_query_rows_run_as_extra_recomputed_rows():
    """The R user-query rows (positions T .. T+R-1) go through the same projection, scatter (appended to the
    fused cache) and attention calls as the selected context rows."""
    rng = np.random.default_rng(44)
    sh = inputs.LayerShape(512, 8, 2, 128, 500000.0, "bf16", 0)
    dt = inputs.torch_dtype(sh.dtype)
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    T, R, N = 700, 24, 90
    kf, vf = rnd(rng, (T + R, Hkv, D), "bf16"), rnd(rng, (T + R, Hkv, D), "bf16")      # rows T.. are placeholders
    x_ctx, x_q = rnd(rng, (T, sh.d_model), "bf16"), rnd(rng, (R, sh.d_model), "bf16")
    w = rnd(rng, (sh.qkv_rows, sh.d_model), "bf16", std=1 / math.sqrt(sh.d_model))
    sel = np.sort(rng.choice(T, size=N, replace=False))
    rows = np.concatenate([sel, T + np.arange(R)]).astype(np.int32)                    # fused rows == positions
    x_all = np.concatenate([x_ctx, x_q])
    M = N + R
    desc = qb.make_desc(sh)
    q = torch.empty((M, H, D), dtype=dt, device=DEV)
    k = torch.empty((M, Hkv, D), dtype=dt, device=DEV)
    v = torch.empty((M, Hkv, D), dtype=dt, device=DEV)
    qb.qcf_recompute_qkv(desc, to_dev(x_all, dt), T + R, i32(rows), M, to_dev(w, dt), i32(rows), q, k, v)
    dk, dv = to_dev(kf, dt), to_dev(vf, dt)
    qb.qcf_scatter(desc, k, v, i32(rows), M, dk, dv, T + R)
    o = torch.empty((M, H, D), dtype=dt, device=DEV)
    qb.qcf_recompute_attn(desc, 1, q, i32(rows), i64([0, M]), M, dk, dv, i64([0, T + R]), T + R, None, o, None)
    torch.cuda.synchronize()
    qz = quantizer("bf16")
    rq, rk, rv = orc.recompute_qkv(x_all[rows], w, rows, H, Hkv, D, sh.rope_base)
    rkf, rvf = orc.scatter(kf, vf, qz(rk), qz(rv), rows)
    ro, _ = orc.recompute_attn(qz(rq), rows, rkf, rvf)
    assert_close(to_np(o), ro, "bf16", "O of context + query rows")
    assert_close(to_np(dk), rkf, "bf16", "fused K with query rows appended")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_anchor_extraction(dtype):
    """Key norm, per-chunk Top-N by norm and the gather of the anchor rows against the oracle."""
    rng = np.random.default_rng(45)
    sh = (inputs.LayerShape(256, 4, 2, 64, 10000.0, "f32", 0) if dtype == "f32"
          else inputs.LayerShape(4096, 32, 8, 128, 500000.0, "bf16", 0))
    dt = inputs.torch_dtype(dtype)
    lens = [300, 1, 517, 64, 1000]
    n_anchor = [12, 1, 21, 0, 40]
    ks = [rnd(rng, (n, sh.n_kv_heads, sh.head_dim), dtype) for n in lens]
    vs = [rnd(rng, (n, sh.n_kv_heads, sh.head_dim), dtype) for n in lens]
    say(f"anchors {dtype}: chunks {lens}, anchors {n_anchor}")
    desc = qb.make_desc(sh)
    k_all, v_all = to_dev(np.concatenate(ks), dt), to_dev(np.concatenate(vs), dt)
    rows, ak, av = pipeline.extract_anchors(desc, k_all, v_all, lens, n_anchor)
    norm = torch.empty(sum(lens), dtype=torch.float32, device=DEV)
    qb.qcf_key_norm(desc, k_all, sum(lens), norm)
    torch.cuda.synchronize()
    ref_norm = np.concatenate([orc.key_norm(k) for k in ks])
    assert np.all(np.abs(to_np(norm) - ref_norm) <= 2e-6 * ref_norm)
    got = rows.cpu().numpy().astype(np.int64)
    off, pos = 0, 0
    from gpu_util import assert_indices_match
    for c, n in enumerate(lens):
        na = n_anchor[c]
        mine = got[pos:pos + na] - off
        # exact indices unless two norms are closer than the fp32 rounding of the norm
        assert_indices_match(mine, orc.key_norm(ks[c]), na, f"chunk {c}")
        assert np.array_equal(to_np(ak[pos:pos + na]), ks[c][mine]) and np.array_equal(to_np(av[pos:pos + na]), vs[c][mine])
        off += n
        pos += na
    assert pos == len(got)
    # an index outside the source gives a zero row
    bad = i32([5, -1, sum(lens), 7])
    ko = torch.full((4, sh.n_kv_heads, sh.head_dim), 3.0, dtype=dt, device=DEV)
    qb.qcf_gather(desc, k_all, None, bad, 4, sum(lens), ko, None)
    torch.cuda.synchronize()
    assert torch.equal(ko[0], k_all[5]) and torch.equal(ko[3], k_all[7]) and float(ko[1:3].abs().max()) == 0.0
