"""The C-ABI library: it loads, exports every symbol the header declares, and rejects bad
arguments on the host without launching anything (no GPU needed for any of this)."""
import ctypes as C
import os
import re

import pytest

from paper_2604_08585_amd import binding as qb
from paper_2604_08585_amd.inputs import LayerShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qcf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qcf_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = qb.load_library()
    names = declared_symbols()
    assert len(names) == 24 and set(names) == set(qb.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.qcf_version() >= 100
    assert lib.qcf_status_string(0) == b"QCF_OK"
    assert lib.qcf_status_string(3) == b"QCF_ERR_WORKSPACE_TOO_SMALL"


def test_struct_layouts_match_the_header():
    assert C.sizeof(qb.LayerDesc) == 32
    assert C.sizeof(qb.ChunkDesc) == 40
    assert qb.ChunkDesc.dst_row.offset == 24 and qb.LayerDesc.rope_base.offset == 16


def test_select_count_helper():
    assert qb.qcf_select_count(8192, 0.15) == 1229
    assert qb.qcf_select_count(8192, 0.05) == 410
    assert qb.qcf_select_count(8192, 0.30) == 2458
    assert qb.qcf_select_count(100, 0.07) == 7
    assert qb.qcf_select_count(100, 0.0) == 0 and qb.qcf_select_count(100, 1.5) == 100
    assert qb.qcf_select_count(0, 0.5) == 0


def _desc(**kw):
    base = dict(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rope_base=10000.0, dtype="f32")
    base.update(kw)
    return qb.make_desc(LayerShape(**base))


def test_bad_arguments_are_rejected_on_the_host():
    lib = qb.load_library()
    fake = 0x1000          # aligned, never dereferenced: validation fails before any launch
    d = _desc()
    # unsupported head_dim / dtype / bad heads
    assert lib.qcf_rerope(C.byref(_desc(head_dim=96)), fake, 1, 8, fake, fake, fake, 1 << 20, None) == 2
    assert b"head_dim" in lib.qcf_last_error()
    bad = _desc(); bad.dtype = 5
    assert lib.qcf_scatter(C.byref(bad), fake, fake, fake, 4, fake, fake, 8, None) == 2
    assert lib.qcf_scatter(C.byref(_desc(n_q_heads=5)), fake, fake, fake, 4, fake, fake, 8, None) == 1
    # null / misaligned pointers
    assert lib.qcf_rerope(C.byref(d), fake, 1, 8, None, fake, fake, 1 << 20, None) == 1
    assert lib.qcf_rerope(C.byref(d), fake, 1, 8, fake + 4, fake, fake, 1 << 20, None) == 1
    assert b"aligned" in lib.qcf_last_error()
    assert lib.qcf_rerope(None, fake, 1, 8, fake, fake, fake, 1 << 20, None) == 1
    # workspace too small / missing
    need = lib.qcf_rerope_workspace_bytes(C.byref(d), 4, 512)
    assert need > 0
    assert lib.qcf_rerope(C.byref(d), fake, 4, 512, fake, fake, fake, need - 1, None) == 3
    assert lib.qcf_rerope(C.byref(d), fake, 4, 512, fake, fake, None, 0, None) == 3
    need_s = lib.qcf_score_workspace_bytes(C.byref(d), 1, 20, 512)
    assert lib.qcf_score(C.byref(d), 1, fake, fake, 20, fake, fake, 512, None, fake, fake, need_s - 1, None) == 3
    # negative sizes, inconsistent totals
    assert lib.qcf_select(1, fake, fake, 10, fake, 11, None, fake, None, None, None, 0, None) == 1
    assert lib.qcf_recompute_qkv(C.byref(d), fake, -1, None, 4, fake, fake, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.qcf_recompute_qkv(C.byref(d), fake, 2, None, 4, fake, fake, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.qcf_scatter(C.byref(d), fake, fake, fake, 4, fake, None, 8, None) == 1
    # a gather table over an empty x (an index outside x falls back to row 0, which must exist)
    assert lib.qcf_recompute_qkv(C.byref(d), fake, 0, fake, 4, fake, fake, fake, fake, fake, fake, 1 << 20, None) == 1
    assert b"no rows" in lib.qcf_last_error()
    # the one-call form of projection + write-back needs the K/V outputs and the cache
    assert lib.qcf_recompute_qkv_scatter(C.byref(d), fake, 8, fake, 4, fake, fake, fake, None, fake, fake, fake, fake, 8,
                                         fake, 1 << 20, None) == 1
    assert b"k_out" in lib.qcf_last_error()
    assert lib.qcf_recompute_qkv_scatter(C.byref(d), fake, 8, fake, 4, fake, fake, fake, fake, fake, None, fake, fake, 8,
                                         fake, 1 << 20, None) == 1
    assert lib.qcf_recompute_qkv_scatter(C.byref(d), fake, 8, fake, 4, fake, fake, fake, fake, fake, fake, fake, None, 8,
                                         fake, 1 << 20, None) == 1
    assert lib.qcf_recompute_qkv_scatter(C.byref(d), None, 0, None, 0, None, None, None, None, None, None, None, None, 0,
                                         None, 0, None) == 0
    # rest-of-the-layer calls: sizes must be multiples of 8, the f32 / odd-shape path needs its workspace
    assert lib.qcf_linear(C.byref(d), fake, 4, 20, fake, 64, None, fake, None, 0, None) == 1
    assert lib.qcf_linear(C.byref(d), fake, 4, 64, fake, 128, None, None, None, 0, None) == 1
    assert lib.qcf_linear_workspace_bytes(C.byref(_desc(dtype="bf16")), 4, 64, 128) == 0   # MFMA-shaped bf16: none
    need_l = lib.qcf_linear_workspace_bytes(C.byref(d), 4, 24, 40)
    assert need_l >= 4 * 40 * 4
    assert lib.qcf_linear(C.byref(d), fake, 4, 24, fake, 40, None, fake, fake, need_l - 1, None) == 3
    assert lib.qcf_rmsnorm(C.byref(d), fake, fake, 1e-5, 4, 100, fake, None) == 1
    assert lib.qcf_rmsnorm(C.byref(d), fake, fake, -1.0, 4, 64, fake, None) == 1
    assert lib.qcf_swiglu(C.byref(d), fake, 4, 12, fake, None) == 1
    assert lib.qcf_swiglu(C.byref(bad), fake, 4, 16, fake, None) == 2
    assert lib.qcf_key_norm(C.byref(d), None, 4, fake, None) == 1
    assert lib.qcf_gather(C.byref(d), fake, fake, fake, 4, 10, fake, None, None) == 1


def test_empty_work_is_ok_and_launches_nothing():
    lib = qb.load_library()
    d = _desc()
    assert lib.qcf_rerope(C.byref(d), None, 0, 0, None, None, None, 0, None) == 0
    assert lib.qcf_score(C.byref(d), 0, None, None, 0, None, None, 0, None, None, None, 0, None) == 0
    assert lib.qcf_select(1, None, None, 10, None, 0, None, None, None, None, None, 0, None) == 0
    assert lib.qcf_recompute_qkv(C.byref(d), None, 0, None, 0, None, None, None, None, None, None, 0, None) == 0
    assert lib.qcf_scatter(C.byref(d), None, None, None, 0, None, None, 10, None) == 0
    assert lib.qcf_recompute_attn(C.byref(d), 1, None, None, None, 0, None, None, None, 10, None, None, None,
                                  None, 0, None) == 0
    assert lib.qcf_linear(C.byref(d), None, 0, 64, None, 128, None, None, None, 0, None) == 0
    assert lib.qcf_rmsnorm(C.byref(d), None, None, 1e-5, 0, 64, None, None) == 0
    assert lib.qcf_swiglu(C.byref(d), None, 0, 64, None, None) == 0
    assert lib.qcf_key_norm(C.byref(d), None, 0, None, None) == 0
    assert lib.qcf_gather(C.byref(d), None, None, None, 0, 10, None, None, None) == 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(qb, "_lib", None)
    monkeypatch.setattr(qb, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(qb.QcfError):
        qb.load_library()
