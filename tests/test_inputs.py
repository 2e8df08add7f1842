"""The seeded workload generators: structure, determinism, dtype rounding."""
import numpy as np
import pytest

from oracle import qcf_oracle as orc
from paper_2604_08585_amd import inputs


def test_ragged_lengths_recipe():
    rng = np.random.default_rng(0)
    lens = inputs.ragged_lengths(rng, 16, 256, 768, 8192)
    assert len(lens) == 16 and sum(lens) == 8192
    assert min(lens) >= 256 and max(lens) <= 768
    assert len(set(lens)) > 4


def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -3.14159], dtype=np.float32)
    r = inputs.round_to_dtype(a, "bf16")
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -6 and r[3] == 1.0 + 2 ** -7
    assert (r.view(np.uint32) & 0xFFFF == 0).all()
    assert inputs.round_to_dtype(a, "f32").tobytes() == a.tobytes()


def test_config0_shapes_and_determinism():
    ops = orc.PlantOps()
    a = inputs.make_config(0, ops)
    b = inputs.make_config(0, ops)
    sh, req = a.shape, a.requests[0]
    assert (sh.d_model, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype) == (256, 4, 2, 64, "f32")
    assert req.chunk_lens == [128] * 4 and req.R == 20 and req.T == 512
    assert a.w_qkv.shape == (512, 256) and req.x_ctx.shape == (512, 256)
    assert req.q_probe.shape == (20, 4, 64) and len(req.planted) == 32
    assert abs(a.w_qkv.std() - 1 / 16) < 0.002
    for ca, cb in zip(a.requests[0].chunks, b.requests[0].chunks):
        assert np.array_equal(ca.k, cb.k) and np.array_equal(ca.v, cb.v)
    assert np.array_equal(a.requests[0].q_probe, b.requests[0].q_probe)


def test_config2_scaled_structure():
    wl = inputs.make_raw(2, scale=1 / 16)
    req = wl.requests[0]
    assert len(req.chunks) == 16 and req.T == 512 and req.R == 80
    assert min(req.chunk_lens) >= 16 and max(req.chunk_lens) <= 48
    assert req.dst_pos0[0] == 0 and req.dst_pos0[-1] == 512 - req.chunk_lens[-1]
    v = req.chunks[0].k
    assert (v.view(np.uint32) & 0xFFFF == 0).all()      # bf16-representable


def test_config4_shares_chunks_at_different_offsets():
    wl = inputs.make_raw(4, scale=1 / 64, batch=6,
                         shape=inputs.LayerShape(64, 4, 2, 16, 10000.0, "bf16"))
    seen = {}
    shared_slots = total = 0
    moved = False
    for req in wl.requests:
        assert 4 <= len(req.chunks) <= 32 and 16 + 8 <= req.R <= 64 + 8
        uids = [c.uid for c in req.chunks]
        assert len(set(uids)) == len(uids)
        for c, p0 in zip(req.chunks, req.dst_pos0):
            total += 1
            if c.uid < 64:
                shared_slots += 1
                if c.uid in seen and seen[c.uid] != p0:
                    moved = True
                seen[c.uid] = p0
    assert 0.5 < shared_slots / total < 0.9 and moved


def test_planting_never_touches_the_shared_originals():
    ops = orc.PlantOps()
    raw = inputs.make_raw(1, scale=1 / 16, shape=inputs.LayerShape(64, 4, 2, 16, 10000.0, "bf16"))
    before = [c.k.copy() for c in raw.requests[0].chunks]
    originals = list(raw.requests[0].chunks)
    wl = inputs.assemble(raw, ops, plant_frac=0.1)
    for c, b in zip(originals, before):
        assert np.array_equal(c.k, b)
    assert len(wl.requests[0].planted) == 8 * round(0.1 * 32)
    inputs.assert_bf16_headroom(wl)
