"""qcf_score_static (scoring on the library's built-in scratch buffer, for callers that cannot allocate)
against qcf_score on the same inputs, through the C ABI: two calls in a row, the second on a smaller input,
plus the host-side rejection of a problem that does not fit the built-in buffer."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_08585_amd import binding as qb
from paper_2604_08585_amd import inputs
from gpu_util import DEV, SCORE_REL, i64


def _case(seed, T, R, dtype, H=32, Hkv=8, D=128):
    sh = inputs.LayerShape(512, H, Hkv, D, 500000.0, dtype)
    g = torch.Generator(device="cpu").manual_seed(seed)
    dt = inputs.torch_dtype(dtype)
    q = torch.randn((R, H, D), generator=g).to(dt).to(DEV)
    k = torch.randn((T, Hkv, D), generator=g).to(dt).to(DEV)
    return sh, q, k


def _both(sh, q, k, limit=None):
    desc = qb.make_desc(sh)
    R, T = q.shape[0], k.shape[0]
    ref = torch.full((T,), -1.0, dtype=torch.float32, device=DEV)
    got = torch.full((T,), -2.0, dtype=torch.float32, device=DEV)
    qb.qcf_score(desc, 1, q, i64([0, R]), R, k, i64([0, T]), T, limit, ref)
    qb.qcf_score_static(desc, 1, q, i64([0, R]), R, k, i64([0, T]), T, limit, got)
    torch.cuda.synchronize()
    return ref.cpu().numpy().astype(np.float64), got.cpu().numpy().astype(np.float64)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_scoring_matches_the_workspace_entry_point(dtype):
    """Two calls in a row share the built-in buffer; the second is smaller, so stale contents of the first
    (partials of tiles that no longer exist) must not leak into it."""
    shapes = [(2000, 48), (700, 20)] if dtype == "bf16" else [(600, 12), (130, 5)]
    H, Hkv, D = (32, 8, 128) if dtype == "bf16" else (4, 2, 64)
    for call, (T, R) in enumerate(shapes):
        print(f"qcf_score_static {dtype} call {call}: T={T} R={R}", flush=True)
        sh, q, k = _case(10 + call, T, R, dtype, H, Hkv, D)
        ref, got = _both(sh, q, k)
        assert np.all(np.isfinite(got)) and abs(got.sum() - 1.0) < 1e-4
        assert np.all(np.abs(got - ref) <= SCORE_REL * ref + 1e-12), f"call {call}"
        assert np.array_equal(got, ref), f"call {call}: same kernels, same order of operations"
    # a limited-row call right after, again on the shared buffer
    sh, q, k = _case(12, shapes[1][0], shapes[1][1], dtype, H, Hkv, D)
    limit = torch.randint(0, shapes[1][0] + 1, (shapes[1][1],), dtype=torch.int32).to(DEV)
    ref, got = _both(sh, q, k, limit)
    assert np.array_equal(got, ref)


@pytest.mark.gpu
def test_static_scratch_scoring_rejects_what_does_not_fit():
    lib = qb.load_library()
    sh = inputs.LayerShape(4096, 32, 8, 128, 500000.0, "bf16")
    desc = qb.make_desc(sh)
    fake = 0x1000            # aligned, never dereferenced: the size check fails on the host
    big_T, big_R = 1 << 20, 4096
    assert lib.qcf_score_workspace_bytes(C.byref(desc), 1, big_R, big_T) > (16 << 20)
    st = lib.qcf_score_static(C.byref(desc), 1, fake, fake, big_R, fake, fake, big_T, None, fake, None)
    assert st == 3 and b"built-in buffer" in lib.qcf_last_error()
    # empty work is fine and touches nothing
    assert lib.qcf_score_static(C.byref(desc), 0, None, None, 0, None, None, 0, None, None, None) == 0
