"""One fused layer = the library calls of the path in order, on buffers allocated once.

Marshalling only: this module allocates device buffers through torch, builds the small
offset tables, and enqueues the calls of binding.py on the current stream.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as qb
from .inputs import Workload, torch_dtype


@dataclasses.dataclass
class DeviceLayer:
    desc: qb.LayerDesc
    B: int
    total_ctx: int
    total_probe: int
    total_sel: int
    n_chunks: int
    ctx_lens: List[int]
    sel_counts: List[int]
    chunk_tensors: list            # keeps the chunk caches alive
    chunks_dev: torch.Tensor
    ctx_off: torch.Tensor
    probe_off: torch.Tensor
    sel_off: torch.Tensor
    q_probe: torch.Tensor
    x_ctx: torch.Tensor
    w_qkv: torch.Tensor
    k_fused: torch.Tensor
    v_fused: torch.Tensor
    score: torch.Tensor
    sel_idx: torch.Tensor
    sel_row: torch.Tensor
    sel_pos: torch.Tensor
    q_sel: torch.Tensor
    k_sel: torch.Tensor
    v_sel: torch.Tensor
    o_sel: torch.Tensor
    lse: torch.Tensor
    ws_rerope: Optional[torch.Tensor]
    ws_score: Optional[torch.Tensor]
    ws_select: Optional[torch.Tensor]
    ws_qkv: Optional[torch.Tensor]
    ws_attn: Optional[torch.Tensor]


def _ws(nbytes: int, device) -> Optional[torch.Tensor]:
    return torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes else None


def upload(wl: Workload, device, ratio: Optional[float] = None, shared_chunks: Optional[dict] = None) -> DeviceLayer:
    """Copy a workload to the device and allocate every buffer the layer needs.
    `shared_chunks` (uid -> (k, v) tensors) lets several layers or requests share chunk caches."""
    sh = wl.shape
    dt = torch_dtype(sh.dtype)
    desc = qb.make_desc(sh)
    ratio = wl.ratio if ratio is None else ratio
    cache = {} if shared_chunks is None else shared_chunks

    def dev_t(a: np.ndarray, dtype=dt) -> torch.Tensor:
        return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype)

    chunk_dicts, keep = [], []
    ctx_off, probe_off, sel_off = [0], [0], [0]
    row = 0
    for req in wl.requests:
        for ch, pos0 in zip(req.chunks, req.dst_pos0):
            key = ch.uid if ch.uid >= 0 else id(ch)
            if key not in cache or cache[key][2] is not ch.k:
                cache[key] = (dev_t(ch.k), dev_t(ch.v), ch.k)
            kt, vt, _ = cache[key]
            keep.append((kt, vt))
            chunk_dicts.append(dict(k=kt, v=vt, src_pos0=ch.src_pos0, dst_row=row, dst_pos0=pos0))
            row += ch.length
        ctx_off.append(row)
        probe_off.append(probe_off[-1] + req.R)
        sel_off.append(sel_off[-1] + qb.qcf_select_count(req.T, ratio))
    B = len(wl.requests)
    total_ctx, total_probe, total_sel = ctx_off[-1], probe_off[-1], sel_off[-1]
    H, Hkv, D = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    i64 = lambda v: torch.tensor(v, dtype=torch.int64, device=device)
    empty = lambda *s, dtype=dt: torch.empty(*s, dtype=dtype, device=device)
    q_probe = torch.cat([dev_t(r.q_probe) for r in wl.requests]) if total_probe else empty(0, H, D)
    x_ctx = torch.cat([dev_t(r.x_ctx) for r in wl.requests]) if total_ctx else empty(0, sh.d_model)
    n_sel = max(total_sel, 1)
    return DeviceLayer(
        desc=desc, B=B, total_ctx=total_ctx, total_probe=total_probe, total_sel=total_sel,
        n_chunks=len(chunk_dicts), ctx_lens=[r.T for r in wl.requests],
        sel_counts=[sel_off[i + 1] - sel_off[i] for i in range(B)],
        chunk_tensors=keep, chunks_dev=qb.chunk_table(chunk_dicts, device),
        ctx_off=i64(ctx_off), probe_off=i64(probe_off), sel_off=i64(sel_off),
        q_probe=q_probe, x_ctx=x_ctx, w_qkv=dev_t(wl.w_qkv),
        k_fused=empty(max(total_ctx, 1), Hkv, D), v_fused=empty(max(total_ctx, 1), Hkv, D),
        score=empty(max(total_ctx, 1), dtype=torch.float32),
        sel_idx=empty(n_sel, dtype=torch.int32), sel_row=empty(n_sel, dtype=torch.int32),
        sel_pos=empty(n_sel, dtype=torch.int32),
        q_sel=empty(n_sel, H, D), k_sel=empty(n_sel, Hkv, D), v_sel=empty(n_sel, Hkv, D),
        o_sel=empty(n_sel, H, D), lse=empty(n_sel, H, dtype=torch.float32),
        ws_rerope=_ws(qb.qcf_rerope_workspace_bytes(desc, len(chunk_dicts), total_ctx), device),
        ws_score=_ws(qb.qcf_score_workspace_bytes(desc, B, total_probe, total_ctx), device),
        ws_select=_ws(qb.qcf_select_workspace_bytes(B, total_ctx), device),
        ws_qkv=_ws(qb.qcf_recompute_qkv_workspace_bytes(desc, total_sel), device),
        ws_attn=_ws(qb.qcf_recompute_attn_workspace_bytes(desc, B, total_sel, total_ctx), device),
    )


def step_rerope(L: DeviceLayer) -> None:
    qb.qcf_rerope(L.desc, L.chunks_dev, L.n_chunks, L.total_ctx, L.k_fused, L.v_fused, L.ws_rerope)


def step_score(L: DeviceLayer) -> None:
    qb.qcf_score(L.desc, L.B, L.q_probe, L.probe_off, L.total_probe, L.k_fused, L.ctx_off, L.total_ctx,
                 None, L.score, L.ws_score)


def step_select(L: DeviceLayer) -> None:
    qb.qcf_select(L.B, L.score, L.ctx_off, L.total_ctx, L.sel_off, L.total_sel, None, L.sel_idx, L.sel_row,
                  L.sel_pos, L.ws_select)


def step_qkv(L: DeviceLayer) -> None:
    qb.qcf_recompute_qkv(L.desc, L.x_ctx, L.total_ctx, L.sel_row, L.total_sel, L.w_qkv, L.sel_pos,
                         L.q_sel, L.k_sel, L.v_sel, L.ws_qkv)


def step_qkv_scatter(L: DeviceLayer) -> None:
    """Projection and write-back in one call (same results as step_qkv followed by step_scatter)."""
    qb.qcf_recompute_qkv_scatter(L.desc, L.x_ctx, L.total_ctx, L.sel_row, L.total_sel, L.w_qkv, L.sel_pos,
                                 L.q_sel, L.k_sel, L.v_sel, L.sel_row, L.k_fused, L.v_fused, L.total_ctx, L.ws_qkv)


def step_scatter(L: DeviceLayer) -> None:
    qb.qcf_scatter(L.desc, L.k_sel, L.v_sel, L.sel_row, L.total_sel, L.k_fused, L.v_fused, L.total_ctx)


def step_attn(L: DeviceLayer) -> None:
    qb.qcf_recompute_attn(L.desc, L.B, L.q_sel, L.sel_pos, L.sel_off, L.total_sel, L.k_fused, L.v_fused,
                          L.ctx_off, L.total_ctx, None, L.o_sel, L.lse, L.ws_attn)


def score_over_layers(desc, probes: List[torch.Tensor], keys: List[torch.Tensor], probe_off: torch.Tensor,
                      ctx_off: torch.Tensor, weights: Optional[List[float]] = None) -> torch.Tensor:
    """Token scores summed over layers (the all-layer selector; one layer with bare-query probes is the last-layer
    selector): one qcf_score_accumulate call per layer into the same buffer.  probes[l] [total_probe, H, d] and
    keys[l] [total_ctx, H_kv, d] belong to layer l; weights default to the mean."""
    n = len(keys)
    w = [1.0 / n] * n if weights is None else list(weights)
    total_probe, total_ctx = int(probes[0].shape[0]), int(keys[0].shape[0])
    B = int(probe_off.numel()) - 1
    score = torch.empty(max(total_ctx, 1), dtype=torch.float32, device=keys[0].device)
    ws = _ws(qb.qcf_score_workspace_bytes(desc, B, total_probe, total_ctx), keys[0].device)
    for l in range(n):
        qb.qcf_score_accumulate(desc, B, probes[l], probe_off, total_probe, keys[l], ctx_off, total_ctx, None,
                                w[l], 0.0 if l == 0 else 1.0, score, ws)
    return score[:total_ctx]


STEPS = (("rerope", step_rerope), ("score", step_score), ("select", step_select),
         ("qkv", step_qkv), ("scatter", step_scatter), ("attn", step_attn))


# the same path with the projection and the write-back in one call
FUSED_STEPS = (("rerope", step_rerope), ("score", step_score), ("select", step_select),
               ("qkv_scatter", step_qkv_scatter), ("attn", step_attn))


def enqueue_layer(L: DeviceLayer, critical: bool = True, fused: bool = True) -> None:
    """rerope -> [score -> select at the critical layer] -> qkv -> scatter -> attn; with `fused` the projection
    writes the cache rows itself (qcf_recompute_qkv_scatter), otherwise qcf_scatter runs as a call of its own."""
    for name, fn in (FUSED_STEPS if fused else STEPS):
        if not critical and name in ("score", "select"):
            continue
        fn(L)


def fuse_layer(L: DeviceLayer, critical: bool = True) -> Dict[str, torch.Tensor]:
    enqueue_layer(L, critical)
    n = L.total_sel
    return dict(k_fused=L.k_fused[:L.total_ctx], v_fused=L.v_fused[:L.total_ctx], score=L.score[:L.total_ctx],
                sel_idx=L.sel_idx[:n], sel_row=L.sel_row[:n], sel_pos=L.sel_pos[:n], q_sel=L.q_sel[:n],
                k_sel=L.k_sel[:n], v_sel=L.v_sel[:n], o_sel=L.o_sel[:n], lse=L.lse[:n])


class HipPlantOps:
    """Backend for inputs.assemble() that borrows the two method operations of the planting
    recipe from the GPU library (used where the CPU oracle must not be: the benchmark)."""

    def __init__(self, device):
        self.device = device

    def project_qkv(self, shape, x, w_qkv, pos):
        dt = torch_dtype(shape.dtype)
        desc = qb.make_desc(shape)
        M = int(x.shape[0])
        xd = torch.from_numpy(np.ascontiguousarray(x)).to(device=self.device, dtype=dt)
        wd = torch.from_numpy(np.ascontiguousarray(w_qkv)).to(device=self.device, dtype=dt)
        pd = torch.from_numpy(np.asarray(pos, dtype=np.int32)).to(self.device)
        q = torch.empty(M, shape.n_q_heads, shape.head_dim, dtype=dt, device=self.device)
        k = torch.empty(M, shape.n_kv_heads, shape.head_dim, dtype=dt, device=self.device)
        v = torch.empty(M, shape.n_kv_heads, shape.head_dim, dtype=dt, device=self.device)
        qb.qcf_recompute_qkv(desc, xd, M, None, M, wd, pd, q, k, v)
        torch.cuda.synchronize()
        f = lambda t: t.float().cpu().numpy()
        return f(q), f(k), f(v)

    def shift_keys(self, shape, k_rows, delta):
        dt = torch_dtype(shape.dtype)
        desc = qb.make_desc(shape)
        n = int(k_rows.shape[0])
        # the planted target is not yet rounded to the storage dtype: shift it in fp32
        desc32 = qb.make_desc(dataclasses.replace(shape, dtype="f32"))
        kd = torch.from_numpy(np.ascontiguousarray(k_rows, dtype=np.float32)).to(self.device)
        table = qb.chunk_table([dict(k=kd, v=None, src_pos0=0, dst_row=0, dst_pos0=int(delta))], self.device)
        out = torch.empty_like(kd)
        qb.qcf_rerope(desc32, table, 1, n, out, None)
        torch.cuda.synchronize()
        return out.cpu().numpy()


# ------------------------------------------------------------------ rest of the layer

@dataclasses.dataclass
class TailWeights:
    """Device weights of the part of a pre-norm block that follows the attention."""
    w_o: torch.Tensor          # [d_model, H d]
    norm_weight: torch.Tensor  # [d_model]
    w_gate_up: torch.Tensor    # [2 F, d_model], gate rows then up rows
    w_down: torch.Tensor       # [d_model, F]
    eps: float


def layer_tail(desc, h_in: torch.Tensor, o_rows: torch.Tensor, tw: TailWeights) -> torch.Tensor:
    """Hidden states of the recomputed rows after the block: h1 = h_in + o w_o^T,
    h_out = h1 + (silu(n w_gate^T) * (n w_up^T)) w_down^T with n = rmsnorm(h1).  Five library calls."""
    M, dm = h_in.shape
    hd = tw.w_o.shape[1]
    F2 = tw.w_gate_up.shape[0]
    dt, dev = h_in.dtype, h_in.device
    h1 = torch.empty((M, dm), dtype=dt, device=dev)
    qb.qcf_linear(desc, o_rows.reshape(M, hd), M, hd, tw.w_o, dm, h_in, h1)
    n = torch.empty_like(h1)
    qb.qcf_rmsnorm(desc, h1, tw.norm_weight, tw.eps, M, dm, n)
    gu = torch.empty((M, F2), dtype=dt, device=dev)
    qb.qcf_linear(desc, n, M, dm, tw.w_gate_up, F2, None, gu)
    act = torch.empty((M, F2 // 2), dtype=dt, device=dev)
    qb.qcf_swiglu(desc, gu, M, F2 // 2, act)
    out = torch.empty_like(h1)
    qb.qcf_linear(desc, act, M, F2 // 2, tw.w_down, dm, h1, out)
    return out


# ------------------------------------------------------------------ anchor extraction (offline)

def extract_anchors(desc, k: torch.Tensor, v: torch.Tensor, chunk_lens: List[int], n_per_chunk: List[int]):
    """For chunks stored back to back in k / v [sum len, H_kv, d]: the n_c tokens of chunk c with the largest key
    norm.  Returns (rows into k / v, ascending inside each chunk; anchor K rows; anchor V rows).  Three library
    calls: key norm, Top-N per chunk (the selection kernel with one "request" per chunk), gather."""
    dev = k.device
    rows = int(sum(chunk_lens))
    n_per_chunk = [min(int(n), int(l)) for n, l in zip(n_per_chunk, chunk_lens)]
    total = int(sum(n_per_chunk))
    norm = torch.empty(max(rows, 1), dtype=torch.float32, device=dev)
    qb.qcf_key_norm(desc, k, rows, norm)
    ctx_off = torch.tensor(np.concatenate([[0], np.cumsum(chunk_lens)]), dtype=torch.int64, device=dev)
    sel_off = torch.tensor(np.concatenate([[0], np.cumsum(n_per_chunk)]), dtype=torch.int64, device=dev)
    idx = torch.empty(max(total, 1), dtype=torch.int32, device=dev)
    row = torch.empty(max(total, 1), dtype=torch.int32, device=dev)
    qb.qcf_select(len(chunk_lens), norm, ctx_off, rows, sel_off, total, None, idx, row, None)
    ak = torch.empty((max(total, 1),) + tuple(k.shape[1:]), dtype=k.dtype, device=dev)
    av = torch.empty_like(ak)
    qb.qcf_gather(desc, k, v, row, total, rows, ak, av)
    return row[:total], ak[:total], av[:total]


# ------------------------------------------------------------------ layer pipeline: chunk caches streamed from the host

class ChunkStreamer:
    """Per-layer loop in which the chunk caches of layer i+1 travel from pinned host memory to the device on a
    copy stream while layer i is reconstructed on the compute stream (Section 3.1 Phase 4 loads and recomputes
    "layer by layer" in a pipeline).  Two device staging buffers; the re-rotation is the only reader of a staging
    buffer, so a buffer is free again as soon as its layer's qcf_rerope has run.

    host_layers: one (k, v) pair of pinned host tensors [rows, H_kv, d] per layer, holding that layer's chunk
    caches back to back in the order of the layer's chunk table (as `host_chunk_caches` builds them)."""

    def __init__(self, L: DeviceLayer, chunk_lens: List[int], host_layers):
        self.L = L
        self.host = host_layers
        dev = L.k_fused.device
        rows = int(sum(chunk_lens))
        hk0 = host_layers[0][0]
        assert hk0.is_pinned() and tuple(hk0.shape[0:1]) == (rows,)
        self.stage = [(torch.empty_like(hk0, device=dev), torch.empty_like(hk0, device=dev)) for _ in range(2)]
        table = bytes(L.chunks_dev.cpu().numpy().tobytes())
        n = L.n_chunks
        self.tables = []
        row_bytes = hk0.shape[1] * hk0.shape[2] * hk0.element_size()
        for dk, dv in self.stage:
            t = (qb.ChunkDesc * n).from_buffer_copy(table)
            off = 0
            for c in range(n):
                t[c].k_src = dk.data_ptr() + off * row_bytes
                t[c].v_src = dv.data_ptr() + off * row_bytes
                off += chunk_lens[c]
            self.tables.append(torch.frombuffer(bytearray(bytes(t)), dtype=torch.uint8).to(dev))
        self.copy_stream = torch.cuda.Stream(device=dev)
        self.copied = [torch.cuda.Event() for _ in range(2)]
        self.consumed = [torch.cuda.Event() for _ in range(2)]

    def _prefetch(self, layer: int, first_use: bool) -> None:
        s = layer % 2
        with torch.cuda.stream(self.copy_stream):
            if not first_use:
                self.copy_stream.wait_event(self.consumed[s])      # the stage's previous layer has been re-rotated
            self.stage[s][0].copy_(self.host[layer][0], non_blocking=True)
            self.stage[s][1].copy_(self.host[layer][1], non_blocking=True)
            self.copied[s].record(self.copy_stream)

    def run(self, n_layers: int, after_layer=None, overlap: bool = True) -> None:
        """Reconstruction (rerope, qkv, scatter, attn) of n_layers layers on the current stream.  after_layer(i) is
        called after layer i has been enqueued (e.g. to copy results out).  overlap=False waits for every copy
        before computing and for every layer before the next copy (the serial reference)."""
        L = self.L
        cur = torch.cuda.current_stream()
        self._prefetch(0, True)
        for i in range(n_layers):
            s = i % 2
            cur.wait_event(self.copied[s])
            qb.qcf_rerope(L.desc, self.tables[s], L.n_chunks, L.total_ctx, L.k_fused, L.v_fused, L.ws_rerope)
            self.consumed[s].record(cur)
            if overlap and i + 1 < n_layers:
                self._prefetch(i + 1, i + 1 < 2)
            step_qkv(L)
            step_scatter(L)
            step_attn(L)
            if after_layer is not None:
                after_layer(i)
            if not overlap and i + 1 < n_layers:
                cur.synchronize()
                self._prefetch(i + 1, i + 1 < 2)
                self.copy_stream.synchronize()


def host_chunk_caches(L: DeviceLayer, seed: int, n_layers: int):
    """Pinned host copies of n_layers sets of chunk caches shaped like the layer's own (layer 0 = the layer's own
    caches, the others = seeded random values of the same shape and element type)."""
    ks = torch.cat([k for k, _ in L.chunk_tensors])
    vs = torch.cat([v for _, v in L.chunk_tensors])
    out = []
    g = torch.Generator().manual_seed(seed)
    for i in range(n_layers):
        hk = torch.empty(ks.shape, dtype=ks.dtype, pin_memory=True)
        hv = torch.empty(vs.shape, dtype=vs.dtype, pin_memory=True)
        if i == 0:
            hk.copy_(ks)
            hv.copy_(vs)
        else:
            hk.copy_(torch.randn(ks.shape, generator=g).to(ks.dtype))
            hv.copy_(torch.randn(vs.shape, generator=g).to(vs.dtype))
        out.append((hk, hv))
    return out
