"""ctypes binding of libqcf.so: the same calls as include/qcf.h, taking torch CUDA
tensors.  Argument marshalling only - every step runs in the library's HIP kernels.  There is
no fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

from .inputs import LayerShape

_HERE = os.path.dirname(os.path.abspath(__file__))
# QCF_LIB_PATH lets a developer load another build of the same library (A/B comparisons)
LIB_PATH = os.environ.get("QCF_LIB_PATH") or os.path.join(_HERE, "libqcf.so")

EXPORTS = [
    "qcf_status_string", "qcf_last_error", "qcf_version", "qcf_select_count",
    "qcf_rerope_workspace_bytes", "qcf_rerope",
    "qcf_score_workspace_bytes", "qcf_score", "qcf_score_accumulate", "qcf_score_static",
    "qcf_select_workspace_bytes", "qcf_select",
    "qcf_recompute_qkv_workspace_bytes", "qcf_recompute_qkv", "qcf_recompute_qkv_scatter",
    "qcf_scatter",
    "qcf_recompute_attn_workspace_bytes", "qcf_recompute_attn",
    "qcf_linear_workspace_bytes", "qcf_linear", "qcf_rmsnorm", "qcf_swiglu",
    "qcf_key_norm", "qcf_gather",
]


class QcfError(RuntimeError):
    pass


class LayerDesc(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("rope_base", C.c_double), ("rope_style", C.c_int32),
                ("dtype", C.c_int32)]


class ChunkDesc(C.Structure):
    _fields_ = [("k_src", C.c_void_p), ("v_src", C.c_void_p), ("len", C.c_int32),
                ("src_pos0", C.c_int32), ("dst_row", C.c_int64), ("dst_pos0", C.c_int32),
                ("reserved", C.c_int32)]


_lib = None


def load_library() -> C.CDLL:
    """Load the HIP library built in-tree; fail loudly when it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise QcfError(f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; "
                       f"g.build()'` from the repository root (hipcc, gfx950). There is no CPU fallback.")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, sz, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_double
    dp = C.POINTER(LayerDesc)
    lib.qcf_status_string.restype = C.c_char_p
    lib.qcf_status_string.argtypes = [C.c_int]
    lib.qcf_last_error.restype = C.c_char_p
    lib.qcf_last_error.argtypes = []
    lib.qcf_version.restype = i32
    lib.qcf_select_count.restype = i64
    lib.qcf_select_count.argtypes = [i64, dbl]
    lib.qcf_rerope_workspace_bytes.restype = sz
    lib.qcf_rerope_workspace_bytes.argtypes = [dp, i32, i64]
    lib.qcf_rerope.restype = C.c_int
    lib.qcf_rerope.argtypes = [dp, vp, i32, i64, vp, vp, vp, sz, vp]
    lib.qcf_score_workspace_bytes.restype = sz
    lib.qcf_score_workspace_bytes.argtypes = [dp, i32, i64, i64]
    lib.qcf_score.restype = C.c_int
    lib.qcf_score.argtypes = [dp, i32, vp, vp, i64, vp, vp, i64, vp, vp, vp, sz, vp]
    lib.qcf_score_accumulate.restype = C.c_int
    lib.qcf_score_accumulate.argtypes = [dp, i32, vp, vp, i64, vp, vp, i64, vp, C.c_float, C.c_float, vp, vp, sz, vp]
    lib.qcf_score_static.restype = C.c_int
    lib.qcf_score_static.argtypes = [dp, i32, vp, vp, i64, vp, vp, i64, vp, vp, vp]
    lib.qcf_select_workspace_bytes.restype = sz
    lib.qcf_select_workspace_bytes.argtypes = [i32, i64]
    lib.qcf_select.restype = C.c_int
    lib.qcf_select.argtypes = [i32, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.qcf_recompute_qkv_workspace_bytes.restype = sz
    lib.qcf_recompute_qkv_workspace_bytes.argtypes = [dp, i64]
    lib.qcf_recompute_qkv.restype = C.c_int
    lib.qcf_recompute_qkv.argtypes = [dp, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.qcf_recompute_qkv_scatter.restype = C.c_int
    lib.qcf_recompute_qkv_scatter.argtypes = [dp, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    lib.qcf_scatter.restype = C.c_int
    lib.qcf_scatter.argtypes = [dp, vp, vp, vp, i64, vp, vp, i64, vp]
    lib.qcf_recompute_attn_workspace_bytes.restype = sz
    lib.qcf_recompute_attn_workspace_bytes.argtypes = [dp, i32, i64, i64]
    lib.qcf_recompute_attn.restype = C.c_int
    lib.qcf_recompute_attn.argtypes = [dp, i32, vp, vp, vp, i64, vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.qcf_linear_workspace_bytes.restype = sz
    lib.qcf_linear_workspace_bytes.argtypes = [dp, i64, i32, i32]
    lib.qcf_linear.restype = C.c_int
    lib.qcf_linear.argtypes = [dp, vp, i64, i32, vp, i32, vp, vp, vp, sz, vp]
    lib.qcf_rmsnorm.restype = C.c_int
    lib.qcf_rmsnorm.argtypes = [dp, vp, vp, dbl, i64, i32, vp, vp]
    lib.qcf_swiglu.restype = C.c_int
    lib.qcf_swiglu.argtypes = [dp, vp, i64, i32, vp, vp]
    lib.qcf_key_norm.restype = C.c_int
    lib.qcf_key_norm.argtypes = [dp, vp, i64, vp, vp]
    lib.qcf_gather.restype = C.c_int
    lib.qcf_gather.argtypes = [dp, vp, vp, vp, i64, i64, vp, vp, vp]
    _lib = lib
    return lib


def make_desc(shape: LayerShape) -> LayerDesc:
    return LayerDesc(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                     float(shape.rope_base), int(shape.rope_style), 1 if shape.dtype == "bf16" else 0)


def _check(status: int) -> None:
    if status != 0:
        lib = load_library()
        raise QcfError(f"{lib.qcf_status_string(status).decode()}: {lib.qcf_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise QcfError("tensors handed to the library must be contiguous CUDA tensors")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _ws_args(ws: Optional[torch.Tensor]):
    return (None, 0) if ws is None else (ws.data_ptr(), ws.numel())


def chunk_table(chunks: Sequence[dict], device) -> torch.Tensor:
    """Device array of qcf_chunk from dicts with keys k, v (tensors or None), src_pos0, dst_row,
    dst_pos0.  Keep the returned tensor (and the chunk tensors) alive while calls are in flight."""
    arr = (ChunkDesc * len(chunks))()
    for i, ch in enumerate(chunks):
        arr[i] = ChunkDesc(_ptr(ch["k"]), _ptr(ch.get("v")), int(ch["k"].shape[0]), int(ch.get("src_pos0", 0)),
                           int(ch["dst_row"]), int(ch["dst_pos0"]), 0)
    raw = bytes(arr)
    host = torch.frombuffer(bytearray(raw), dtype=torch.uint8) if raw else torch.zeros(0, dtype=torch.uint8)
    return host.to(device)


def qcf_select_count(T: int, ratio: float) -> int:
    return int(load_library().qcf_select_count(int(T), float(ratio)))


def qcf_rerope_workspace_bytes(desc: LayerDesc, n_chunks: int, total_rows: int) -> int:
    return int(load_library().qcf_rerope_workspace_bytes(C.byref(desc), n_chunks, total_rows))


def qcf_rerope(desc: LayerDesc, chunks_dev: torch.Tensor, n_chunks: int, total_rows: int,
               k_fused: torch.Tensor, v_fused: Optional[torch.Tensor],
               workspace: Optional[torch.Tensor] = None) -> None:
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_rerope_workspace_bytes(desc, n_chunks, total_rows), k_fused.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_rerope(C.byref(desc), _ptr(chunks_dev), n_chunks, total_rows, _ptr(k_fused), _ptr(v_fused),
                          wp, wn, _stream()))


def qcf_score_workspace_bytes(desc: LayerDesc, B: int, total_probe: int, total_ctx: int) -> int:
    return int(load_library().qcf_score_workspace_bytes(C.byref(desc), B, total_probe, total_ctx))


def qcf_score(desc: LayerDesc, B: int, q_probe: torch.Tensor, probe_off: torch.Tensor, total_probe: int,
              k_fused: torch.Tensor, ctx_off: torch.Tensor, total_ctx: int,
              probe_limit: Optional[torch.Tensor], score: torch.Tensor,
              workspace: Optional[torch.Tensor] = None) -> None:
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_score_workspace_bytes(desc, B, total_probe, total_ctx), score.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_score(C.byref(desc), B, _ptr(q_probe), _ptr(probe_off), total_probe, _ptr(k_fused),
                         _ptr(ctx_off), total_ctx, _ptr(probe_limit), _ptr(score), wp, wn, _stream()))


def qcf_score_accumulate(desc: LayerDesc, B: int, q_probe: torch.Tensor, probe_off: torch.Tensor, total_probe: int,
                         k_fused: torch.Tensor, ctx_off: torch.Tensor, total_ctx: int,
                         probe_limit: Optional[torch.Tensor], alpha: float, beta: float, score: torch.Tensor,
                         workspace: Optional[torch.Tensor] = None) -> None:
    """score = beta * score + alpha * (mean attention of this layer's probe rows over its keys)."""
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_score_workspace_bytes(desc, B, total_probe, total_ctx), score.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_score_accumulate(C.byref(desc), B, _ptr(q_probe), _ptr(probe_off), total_probe, _ptr(k_fused),
                                    _ptr(ctx_off), total_ctx, _ptr(probe_limit), float(alpha), float(beta),
                                    _ptr(score), wp, wn, _stream()))


def qcf_score_static(desc: LayerDesc, B: int, q_probe: torch.Tensor, probe_off: torch.Tensor, total_probe: int,
                     k_fused: torch.Tensor, ctx_off: torch.Tensor, total_ctx: int,
                     probe_limit: Optional[torch.Tensor], score: torch.Tensor) -> None:
    """qcf_score on the library's built-in scratch buffer: no workspace, no allocation."""
    _check(load_library().qcf_score_static(C.byref(desc), B, _ptr(q_probe), _ptr(probe_off), total_probe,
                                           _ptr(k_fused), _ptr(ctx_off), total_ctx, _ptr(probe_limit), _ptr(score),
                                           _stream()))


def qcf_select_workspace_bytes(B: int, total_ctx: int) -> int:
    return int(load_library().qcf_select_workspace_bytes(B, total_ctx))


def qcf_select(B: int, score: torch.Tensor, ctx_off: torch.Tensor, total_ctx: int, sel_off: torch.Tensor,
               total_sel: int, ctx_pos0: Optional[torch.Tensor], sel_idx: torch.Tensor,
               sel_row: Optional[torch.Tensor], sel_pos: Optional[torch.Tensor],
               workspace: Optional[torch.Tensor] = None) -> None:
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_select_workspace_bytes(B, total_ctx), score.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_select(B, _ptr(score), _ptr(ctx_off), total_ctx, _ptr(sel_off), total_sel, _ptr(ctx_pos0),
                          _ptr(sel_idx), _ptr(sel_row), _ptr(sel_pos), wp, wn, _stream()))


def qcf_recompute_qkv_workspace_bytes(desc: LayerDesc, M: int) -> int:
    return int(load_library().qcf_recompute_qkv_workspace_bytes(C.byref(desc), M))


def qcf_recompute_qkv(desc: LayerDesc, x: torch.Tensor, x_rows: int, x_gather: Optional[torch.Tensor], M: int,
                      w_qkv: torch.Tensor, pos: torch.Tensor, q_out: Optional[torch.Tensor],
                      k_out: Optional[torch.Tensor], v_out: Optional[torch.Tensor],
                      workspace: Optional[torch.Tensor] = None) -> None:
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_recompute_qkv_workspace_bytes(desc, M), x.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_recompute_qkv(C.byref(desc), _ptr(x), x_rows, _ptr(x_gather), M, _ptr(w_qkv), _ptr(pos),
                                 _ptr(q_out), _ptr(k_out), _ptr(v_out), wp, wn, _stream()))


def qcf_recompute_qkv_scatter(desc: LayerDesc, x: torch.Tensor, x_rows: int, x_gather: Optional[torch.Tensor],
                              M: int, w_qkv: torch.Tensor, pos: torch.Tensor, q_out: Optional[torch.Tensor],
                              k_out: torch.Tensor, v_out: torch.Tensor, dst_rows: torch.Tensor,
                              k_fused: torch.Tensor, v_fused: torch.Tensor, total_rows: int,
                              workspace: Optional[torch.Tensor] = None) -> None:
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_recompute_qkv_workspace_bytes(desc, M), x.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_recompute_qkv_scatter(C.byref(desc), _ptr(x), x_rows, _ptr(x_gather), M, _ptr(w_qkv), _ptr(pos),
                                         _ptr(q_out), _ptr(k_out), _ptr(v_out), _ptr(dst_rows), _ptr(k_fused),
                                         _ptr(v_fused), total_rows, wp, wn, _stream()))


def qcf_scatter(desc: LayerDesc, k_new: torch.Tensor, v_new: Optional[torch.Tensor], dst_rows: torch.Tensor,
                M: int, k_fused: torch.Tensor, v_fused: Optional[torch.Tensor], total_rows: int) -> None:
    lib = load_library()
    _check(lib.qcf_scatter(C.byref(desc), _ptr(k_new), _ptr(v_new), _ptr(dst_rows), M, _ptr(k_fused),
                           _ptr(v_fused), total_rows, _stream()))


def qcf_recompute_attn_workspace_bytes(desc: LayerDesc, B: int, total_sel: int, total_ctx: int) -> int:
    return int(load_library().qcf_recompute_attn_workspace_bytes(C.byref(desc), B, total_sel, total_ctx))


def qcf_recompute_attn(desc: LayerDesc, B: int, q_sel: torch.Tensor, sel_pos: torch.Tensor,
                       sel_off: torch.Tensor, total_sel: int, k_fused: torch.Tensor, v_fused: torch.Tensor,
                       ctx_off: torch.Tensor, total_ctx: int, ctx_pos0: Optional[torch.Tensor],
                       o_out: torch.Tensor, lse_out: Optional[torch.Tensor],
                       workspace: Optional[torch.Tensor] = None) -> None:
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_recompute_attn_workspace_bytes(desc, B, total_sel, total_ctx), q_sel.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_recompute_attn(C.byref(desc), B, _ptr(q_sel), _ptr(sel_pos), _ptr(sel_off), total_sel,
                                  _ptr(k_fused), _ptr(v_fused), _ptr(ctx_off), total_ctx, _ptr(ctx_pos0),
                                  _ptr(o_out), _ptr(lse_out), wp, wn, _stream()))


def qcf_linear_workspace_bytes(desc: LayerDesc, M: int, K: int, N: int) -> int:
    return int(load_library().qcf_linear_workspace_bytes(C.byref(desc), M, K, N))


def qcf_linear(desc: LayerDesc, x: torch.Tensor, M: int, K: int, w: torch.Tensor, N: int,
               residual: Optional[torch.Tensor], out: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> None:
    lib = load_library()
    if workspace is None:
        workspace = _workspace(qcf_linear_workspace_bytes(desc, M, K, N), x.device)
    wp, wn = _ws_args(workspace)
    _check(lib.qcf_linear(C.byref(desc), _ptr(x), M, K, _ptr(w), N, _ptr(residual), _ptr(out), wp, wn, _stream()))


def qcf_rmsnorm(desc: LayerDesc, x: torch.Tensor, weight: torch.Tensor, eps: float, M: int, cols: int,
                out: torch.Tensor) -> None:
    _check(load_library().qcf_rmsnorm(C.byref(desc), _ptr(x), _ptr(weight), float(eps), M, cols, _ptr(out), _stream()))


def qcf_swiglu(desc: LayerDesc, gate_up: torch.Tensor, M: int, F: int, out: torch.Tensor) -> None:
    _check(load_library().qcf_swiglu(C.byref(desc), _ptr(gate_up), M, F, _ptr(out), _stream()))


def qcf_key_norm(desc: LayerDesc, k: torch.Tensor, rows: int, norm: torch.Tensor) -> None:
    _check(load_library().qcf_key_norm(C.byref(desc), _ptr(k), rows, _ptr(norm), _stream()))


def qcf_gather(desc: LayerDesc, k_src: torch.Tensor, v_src: Optional[torch.Tensor], src_rows: torch.Tensor, M: int,
               total_rows: int, k_out: torch.Tensor, v_out: Optional[torch.Tensor]) -> None:
    _check(load_library().qcf_gather(C.byref(desc), _ptr(k_src), _ptr(v_src), _ptr(src_rows), M, total_rows,
                                     _ptr(k_out), _ptr(v_out), _stream()))
