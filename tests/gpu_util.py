"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

from oracle import qcf_oracle as orc
from paper_2604_08585_amd import binding as qb
from paper_2604_08585_amd import inputs

DEV = torch.device("cuda:0")

# the bar: max-abs 2e-2 for bf16 outputs, 1e-4 for fp32 outputs; scores are fp32 of magnitude
# ~1/T, so they must also agree to 1e-3 relative
TOL = {"bf16": 2e-2, "f32": 1e-4}
SCORE_REL = 1e-3


def to_dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device=DEV, dtype=dtype)


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def quantizer(dtype):
    return lambda a: inputs.round_to_dtype(np.asarray(a, dtype=np.float64), dtype).astype(np.float64)


def i64(v):
    return torch.tensor(list(v), dtype=torch.int64, device=DEV)


def i32(v):
    return torch.tensor(np.asarray(v, dtype=np.int32), dtype=torch.int32, device=DEV)


def max_abs(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.abs(a - b).max()) if a.size else 0.0


def assert_close(got, ref, dtype, what):
    err = max_abs(got, ref)
    assert err <= TOL[dtype], f"{what}: max abs error {err:.3e} > {TOL[dtype]}"
    return err


def assert_indices_match(got, ref_scores, n, what=""):
    """Bit-exact selected indices, except where the oracle's score margin to the Top-N threshold is
    below 1e-3 (relative to the threshold): |S| = N exactly, ascending, and every index in the
    symmetric difference with the oracle's set lies inside that band."""
    got = np.asarray(got, dtype=np.int64)
    ref = orc.select(ref_scores, n)
    assert got.shape == (n,), f"{what}: {got.shape} != ({n},)"
    assert np.all(np.diff(got) > 0), f"{what}: not strictly ascending"
    if n == 0 or np.array_equal(got, ref):
        return 0
    tau = np.sort(np.asarray(ref_scores, dtype=np.float64))[::-1][n - 1]
    diff = np.setxor1d(got, ref)
    margin = np.abs(np.asarray(ref_scores, dtype=np.float64)[diff] - tau)
    assert np.all(margin <= 1e-3 * abs(tau)), f"{what}: indices {diff} differ outside the threshold band"
    return len(diff)


def layer_desc(shape):
    return qb.make_desc(shape)


def run_rerope(shape, chunks, dst_rows, dst_pos0, total_rows, src_pos0=None, with_v=True, prefill=None):
    """chunks: list of (k, v) float arrays holding dtype-representable values."""
    dt = inputs.torch_dtype(shape.dtype)
    desc = qb.make_desc(shape)
    cds, keep = [], []
    for i, (k, v) in enumerate(chunks):
        kt, vt = to_dev(k, dt), to_dev(v, dt)
        keep.append((kt, vt))
        cds.append(dict(k=kt, v=vt, src_pos0=0 if src_pos0 is None else src_pos0[i], dst_row=dst_rows[i],
                        dst_pos0=dst_pos0[i]))
    table = qb.chunk_table(cds, DEV)
    Hkv, D = shape.n_kv_heads, shape.head_dim
    if prefill is None:
        kf = torch.zeros(max(total_rows, 1), Hkv, D, dtype=dt, device=DEV)
        vf = torch.zeros(max(total_rows, 1), Hkv, D, dtype=dt, device=DEV)
    else:
        kf, vf = to_dev(prefill[0], dt), to_dev(prefill[1], dt)
    qb.qcf_rerope(desc, table, len(cds), total_rows, kf, vf if with_v else None)
    torch.cuda.synchronize()
    return kf[:total_rows], vf[:total_rows]
