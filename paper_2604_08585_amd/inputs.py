"""Seeded synthetic workloads for the per-layer KV-cache fusion path.

This module only draws random numbers, rounds them to the storage dtype and
lays out chunks.  It performs none of the method's arithmetic (no rotary
embedding, no projection, no attention, no ranking): the two operations the
planting recipe needs from the method (projecting probe rows to rotated query
vectors, and moving a key back to a chunk's local frame) are supplied by the
caller through a small backend object, so the CPU oracle and the GPU library
can each assemble a workload without sharing code.

The workloads stand in for RAG prompts (retrieved chunks prefilled
independently, then concatenated in front of a user query; Section 3.1 of the
paper): shapes follow 8B/70B-class decoder layers, values are Gaussian.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Protocol, Sequence, Tuple

import numpy as np
import torch


# --------------------------------------------------------------------------
# storage dtypes
# --------------------------------------------------------------------------

def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float array to the storage dtype; result is float32 holding
    exactly representable values (round-to-nearest-even for bf16)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a32
    if dtype == "bf16":
        t = torch.from_numpy(a32).to(torch.bfloat16).to(torch.float32)
        return t.numpy()
    raise ValueError(f"unknown dtype {dtype!r}")


def torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


# --------------------------------------------------------------------------
# descriptors
# --------------------------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class LayerShape:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    dtype: str            # "f32" | "bf16"
    rope_style: int = 0   # 0 = half-split pairs (i, i+d/2), 1 = interleaved (2i, 2i+1)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim


@dataclasses.dataclass
class Chunk:
    """One independently prefilled context chunk (read-only, may be shared)."""
    k: np.ndarray            # [len, H_kv, d] float32 holding dtype-rounded values
    v: np.ndarray            # [len, H_kv, d]
    src_pos0: int = 0        # local position of its first token when it was prefilled
    uid: int = -1            # identity of the chunk (shared chunks have the same uid)

    @property
    def length(self) -> int:
        return int(self.k.shape[0])


@dataclasses.dataclass
class Request:
    chunks: List[Chunk]
    x_ctx: np.ndarray        # [T, d_model] hidden states of the context tokens
    x_probe: np.ndarray      # [R, d_model] anchor rows first, then user-query rows
    n_q: int
    n_a: int
    q_probe: Optional[np.ndarray] = None   # [R, H, d], filled by assemble()
    planted: Optional[np.ndarray] = None   # fused-row indices of planted tokens

    @property
    def chunk_lens(self) -> List[int]:
        return [c.length for c in self.chunks]

    @property
    def T(self) -> int:
        return int(sum(self.chunk_lens))

    @property
    def R(self) -> int:
        return self.n_q + self.n_a

    @property
    def dst_pos0(self) -> List[int]:
        """Global position of each chunk's first token in the fused prompt."""
        out, acc = [], 0
        for n in self.chunk_lens:
            out.append(acc)
            acc += n
        return out


@dataclasses.dataclass
class Workload:
    name: str
    shape: LayerShape
    w_qkv: np.ndarray        # [(H + 2 H_kv) d, d_model]; rows: Q heads, K heads, V heads
    requests: List[Request]
    ratio: float
    seed: int


class PlantBackend(Protocol):
    """The two method operations the planting recipe borrows from its caller."""

    def project_qkv(self, shape: LayerShape, x: np.ndarray, w_qkv: np.ndarray,
                    pos: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Rotated Q [M,H,d], rotated K [M,H_kv,d], V [M,H_kv,d] of rows x at positions pos."""

    def shift_keys(self, shape: LayerShape, k_rows: np.ndarray, delta: int) -> np.ndarray:
        """Keys [n,H_kv,d] re-rotated by delta positions."""


# --------------------------------------------------------------------------
# chunk length recipes
# --------------------------------------------------------------------------

def ragged_lengths(rng: np.random.Generator, n: int, lo: int, hi: int, total: int) -> List[int]:
    """n integers drawn uniformly from [lo, hi], then nudged by +-1 round-robin
    (skipping any at a bound) until they sum to `total`."""
    if not (n * lo <= total <= n * hi):
        raise ValueError("total not reachable")
    lens = rng.integers(lo, hi + 1, size=n).astype(np.int64)
    i = 0
    while lens.sum() != total:
        step = 1 if lens.sum() < total else -1
        if lo <= lens[i] + step <= hi:
            lens[i] += step
        i = (i + 1) % n
    return [int(x) for x in lens]


# --------------------------------------------------------------------------
# raw draws
# --------------------------------------------------------------------------

def _normal(rng: np.random.Generator, shape, dtype: str, std: float = 1.0) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return round_to_dtype(a, dtype)


def _draw_request(rng, shape: LayerShape, lens: Sequence[int], n_q: int, n_a: int,
                  pool: Optional[List[Chunk]] = None, share_prob: float = 0.0,
                  uid_base: int = 0) -> Request:
    chunks: List[Chunk] = []
    used = set()
    for ci, n in enumerate(lens):
        if pool is not None and rng.random() < share_prob:
            cand = [p for p in range(len(pool)) if p not in used and pool[p].length == n]
            if cand:
                p = int(cand[int(rng.integers(0, len(cand)))])
                used.add(p)
                chunks.append(pool[p])
                continue
        chunks.append(Chunk(k=_normal(rng, (n, shape.n_kv_heads, shape.head_dim), shape.dtype),
                            v=_normal(rng, (n, shape.n_kv_heads, shape.head_dim), shape.dtype),
                            uid=uid_base + ci))
    T = int(sum(lens))
    return Request(chunks=chunks,
                   x_ctx=_normal(rng, (T, shape.d_model), shape.dtype),
                   x_probe=_normal(rng, (n_q + n_a, shape.d_model), shape.dtype),
                   n_q=n_q, n_a=n_a)


def _draw_weights(rng, shape: LayerShape) -> np.ndarray:
    return _normal(rng, (shape.qkv_rows, shape.d_model), shape.dtype,
                   std=1.0 / math.sqrt(shape.d_model))


# --------------------------------------------------------------------------
# planting (needs a backend)
# --------------------------------------------------------------------------

def probe_positions(req: Request) -> np.ndarray:
    """Probe rows sit right after the context: anchors first, then the query."""
    return np.arange(req.T, req.T + req.R, dtype=np.int64)


def assemble(wl: Workload, backend: PlantBackend, *, plant_per_chunk: Optional[int] = None,
             plant_frac: float = 0.0, coherent_probe: Optional[float] = None,
             plant_gain: float = 3.0, plant_noise: float = 0.5) -> Workload:
    """Fill q_probe for every request and plant query-relevant keys.

    For KV head g the planted key, seen at its global position, is
    plant_gain * mean(probe query vectors of the group) + N(0, plant_noise);
    it is stored in the chunk cache moved back to the chunk's local frame.
    Chunks that are planted are copied first, so a shared pool is never
    modified.  With coherent_probe = s every probe hidden row becomes
    u + s * eps for one shared u (a crisp-recovery variant for tests).
    """
    rng = np.random.default_rng([wl.seed, 0x9E3779B9])
    sh = wl.shape
    for req in wl.requests:
        if coherent_probe is not None:
            u = rng.standard_normal(size=(1, sh.d_model), dtype=np.float32)
            eps = rng.standard_normal(size=req.x_probe.shape, dtype=np.float32)
            req.x_probe = round_to_dtype(u + np.float32(coherent_probe) * eps, sh.dtype)
        q, _, _ = backend.project_qkv(sh, req.x_probe, wl.w_qkv, probe_positions(req))
        req.q_probe = round_to_dtype(np.asarray(q, dtype=np.float64), sh.dtype)
        planted_rows: List[int] = []
        if plant_per_chunk is None and plant_frac <= 0.0:
            req.planted = np.zeros((0,), dtype=np.int64)
            continue
        qbar = req.q_probe.astype(np.float64).reshape(req.R, sh.n_kv_heads, sh.group, sh.head_dim)
        qbar = qbar.mean(axis=(0, 2))                          # [H_kv, d]
        for ci, (ch, pos0) in enumerate(zip(list(req.chunks), req.dst_pos0)):
            n_pl = plant_per_chunk if plant_per_chunk is not None else int(round(plant_frac * ch.length))
            n_pl = min(n_pl, ch.length)
            if n_pl == 0:
                continue
            loc = np.sort(rng.choice(ch.length, size=n_pl, replace=False))
            noise = rng.standard_normal(size=(n_pl, sh.n_kv_heads, sh.head_dim))
            target = plant_gain * qbar[None, :, :] + plant_noise * noise
            local = backend.shift_keys(sh, target, -(pos0 - ch.src_pos0))
            new = Chunk(k=ch.k.copy(), v=ch.v, src_pos0=ch.src_pos0, uid=ch.uid)
            new.k[loc] = round_to_dtype(np.asarray(local, dtype=np.float64), sh.dtype)
            req.chunks[ci] = new
            planted_rows.extend(int(pos0 + t) for t in loc)
        req.planted = np.asarray(sorted(planted_rows), dtype=np.int64)
    return wl


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

LLAMA3_ROPE_BASE = 500000.0


def layer_shape(cfg: int) -> LayerShape:
    if cfg == 0:
        return LayerShape(256, 4, 2, 64, 10000.0, "f32")
    if cfg in (1, 2, 4):
        return LayerShape(4096, 32, 8, 128, LLAMA3_ROPE_BASE, "bf16")
    if cfg == 3:
        return LayerShape(8192, 64, 8, 128, LLAMA3_ROPE_BASE, "bf16")
    raise ValueError(cfg)


def make_raw(cfg: int, *, ratio: Optional[float] = None, seed: Optional[int] = None,
             scale: float = 1.0, shape: Optional[LayerShape] = None,
             batch: Optional[int] = None) -> Workload:
    """Unplanted workload for configuration `cfg` (0..4).

    `scale` < 1 shrinks token counts (chunk lengths or chunk counts) for tests
    that want the same structure at a size the CPU oracle finishes quickly.
    """
    sh = shape or layer_shape(cfg)
    seed = cfg if seed is None else seed
    rng = np.random.default_rng([seed, cfg])
    w = _draw_weights(rng, sh)
    if cfg == 0:
        lens, n_q, n_a, r = [max(1, int(128 * scale))] * 4, 16, 4, 0.15
        reqs = [_draw_request(rng, sh, lens, n_q, n_a)]
    elif cfg == 1:
        lens, n_q, n_a, r = [max(1, int(512 * scale))] * 8, 32, 8, 0.15
        reqs = [_draw_request(rng, sh, lens, n_q, n_a)]
    elif cfg == 2:
        lo, hi, tot = max(1, int(256 * scale)), max(1, int(768 * scale)), max(16, int(8192 * scale))
        lens = ragged_lengths(rng, 16, lo, hi, tot)
        n_q, n_a, r = 64, 16, 0.15
        reqs = [_draw_request(rng, sh, lens, n_q, n_a)]
    elif cfg == 3:
        lens, n_q, n_a, r = [max(1, int(1024 * scale))] * 32, 64, 16, 0.15
        reqs = [_draw_request(rng, sh, lens, n_q, n_a)]
    elif cfg == 4:
        B = 16 if batch is None else batch
        clen = max(1, int(512 * scale))
        pool = [Chunk(k=_normal(rng, (clen, sh.n_kv_heads, sh.head_dim), sh.dtype),
                      v=_normal(rng, (clen, sh.n_kv_heads, sh.head_dim), sh.dtype),
                      uid=p) for p in range(64)]
        r = 0.15
        reqs = []
        for b in range(B):
            n_chunks = int(rng.integers(4, 33))
            n_q = int(rng.integers(16, 65))
            reqs.append(_draw_request(rng, sh, [clen] * n_chunks, n_q, 8, pool=pool,
                                      share_prob=0.7, uid_base=1000 * (b + 1)))
    else:
        raise ValueError(cfg)
    return Workload(name=f"cfg{cfg}", shape=sh, w_qkv=w, requests=reqs,
                    ratio=r if ratio is None else ratio, seed=seed)


def make_config(cfg: int, backend: PlantBackend, **kw) -> Workload:
    """Configuration `cfg` with probe queries filled in and relevant tokens planted
    (8 per chunk for cfg 0, 2 % of each chunk for cfg 1-3, none for the ragged batch)."""
    wl = make_raw(cfg, **kw)
    if cfg == 0:
        return assemble(wl, backend, plant_per_chunk=8)
    if cfg in (1, 2, 3):
        return assemble(wl, backend, plant_frac=0.02)
    return assemble(wl, backend)


def assert_bf16_headroom(wl: Workload, bound: float = 8.0) -> None:
    """bf16 keeps a half-ulp below the 2e-2 tolerance only for |x| < 8; the
    Gaussian recipes stay inside with overwhelming probability - check it."""
    for req in wl.requests:
        for ch in req.chunks:
            if np.abs(ch.k).max() >= bound or np.abs(ch.v).max() >= bound:
                raise AssertionError("chunk cache value outside the bf16 headroom")
        if req.q_probe is not None and np.abs(req.q_probe).max() >= bound:
            raise AssertionError("probe query outside the bf16 headroom")
