"""CPU oracle for the per-layer query-centric KV-cache fusion step.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
library is checked against.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does, and
this file imports nothing from the product.

Everything is float64 NumPy.  A matrix product (`@`) and a stable sort are the
only library primitives used as steps; there is no tiling, fusion or
reordering beyond what each definition states.

What the path computes, per request (Section 3.1, Phases 3-4, and Section 3.2
of the paper; the re-rotation is the mechanism behind the paper's
"location-independent" chunk reuse with "absolute locations"):

  1. rerope   chunk keys, prefilled at local positions, are rotated to their
              global positions in the concatenated prompt; values are copied.
  2. score    attention of the probe rows (user query + summary anchors) over
              the context keys of the critical layer, softmax over the context,
              averaged over heads and probe rows (Section 3.2, token selector).
  3. select   Top-N tokens by that score, N from the recompute ratio.
  4. qkv      Q/K/V of the selected tokens are recomputed from their hidden
              states and rotated at their absolute positions (Phase 4).
  5. scatter  the recomputed K/V rows replace the cached rows.
  6. attn     the selected rows attend causally, by absolute position, over the
              patched cache (Section 3.2, location-aware sparse attention).

Pins: every function below is pinned by tests/test_oracle_*.py against facts it
does not compute itself (hand-worked values in tests/golden/, closed forms,
group laws, SciPy's softmax, torch's float64 scaled_dot_product_attention,
brute-force loops).  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# rotary embedding
# --------------------------------------------------------------------------

def rope_frequencies(head_dim: int, base: float) -> np.ndarray:
    """theta_i = base^(-2i/d) for i in [0, d/2)."""
    i = np.arange(head_dim // 2, dtype=F64)
    return np.power(F64(base), -2.0 * i / F64(head_dim))


def rotate(x: np.ndarray, phi: np.ndarray, style: int = 0) -> np.ndarray:
    """Rotate the pairs of the last axis of x by the angles phi.

    x   [..., d]
    phi broadcastable to [..., d/2]
    style 0: pair i is (x[i], x[i + d/2]);  style 1: pair i is (x[2i], x[2i+1]).
    A pair (a, b) becomes (a cos - b sin, b cos + a sin): a counter-clockwise
    rotation by phi, so a token at position p carries angle +p*theta_i.
    """
    x = np.asarray(x, dtype=F64)
    d = x.shape[-1]
    c, s = np.cos(phi), np.sin(phi)
    out = np.empty_like(x)
    if style == 0:
        a, b = x[..., : d // 2], x[..., d // 2:]
        out[..., : d // 2] = a * c - b * s
        out[..., d // 2:] = b * c + a * s
    elif style == 1:
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = b * c + a * s
    else:
        raise ValueError("rope style must be 0 or 1")
    return out


def rope_at(x: np.ndarray, pos: np.ndarray, base: float, style: int = 0) -> np.ndarray:
    """Rotary embedding of rows x [M, heads, d] at integer positions pos [M]."""
    theta = rope_frequencies(x.shape[-1], base)
    phi = np.asarray(pos, dtype=F64)[:, None, None] * theta[None, None, :]
    return rotate(x, phi, style)


# --------------------------------------------------------------------------
# step 1: rerope
# --------------------------------------------------------------------------

def rerope(k_chunks: Sequence[np.ndarray], v_chunks: Optional[Sequence[np.ndarray]],
           deltas: Sequence[int], base: float, style: int = 0
           ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Concatenate chunk caches into the fused cache.

    Chunk c's keys [L_c, H_kv, d] already carry the rotation of their local
    positions; moving the chunk by deltas[c] = (new global start - old local
    start) positions adds the angle deltas[c] * theta_i to every pair.  Values
    carry no position and are copied.
    """
    ks, vs = [], []
    for c, k in enumerate(k_chunks):
        k = np.asarray(k, dtype=F64)
        theta = rope_frequencies(k.shape[-1], base)
        ks.append(rotate(k, F64(deltas[c]) * theta, style))
        if v_chunks is not None:
            vs.append(np.asarray(v_chunks[c], dtype=F64))
    k_fused = np.concatenate(ks, axis=0) if ks else np.zeros((0, 0, 0))
    v_fused = (np.concatenate(vs, axis=0) if vs else np.zeros((0, 0, 0))) if v_chunks is not None else None
    return k_fused, v_fused


# --------------------------------------------------------------------------
# step 2: score
# --------------------------------------------------------------------------

def score(q_probe: np.ndarray, k_fused: np.ndarray,
          probe_limit: Optional[np.ndarray] = None) -> np.ndarray:
    """Head- and row-averaged attention each context token receives.

    q_probe [R, H, d] rotated probe queries; k_fused [T, H_kv, d].
    logit(i,h,j) = q[i,h] . k[j, h // G] / sqrt(d); softmax over the T context
    tokens j; the result is the mean over all (i,h).  With probe_limit, row i
    only sees tokens j < probe_limit[i] (rows that see nothing contribute 0).
    """
    q = np.asarray(q_probe, dtype=F64)
    k = np.asarray(k_fused, dtype=F64)
    R, H, d = q.shape
    T, Hkv, _ = k.shape
    G = H // Hkv
    out = np.zeros(T, dtype=F64)
    if T == 0 or R == 0:
        return out
    for h in range(H):
        logits = (q[:, h, :] @ k[:, h // G, :].T) / math.sqrt(d)        # [R, T]
        if probe_limit is not None:
            j = np.arange(T)[None, :]
            logits = np.where(j < np.asarray(probe_limit)[:, None], logits, -np.inf)
        m = logits.max(axis=1, keepdims=True)
        m = np.where(np.isfinite(m), m, 0.0)
        e = np.exp(logits - m)
        z = e.sum(axis=1, keepdims=True)
        p = np.divide(e, z, out=np.zeros_like(e), where=z > 0)
        out += p.sum(axis=0)
    return out / (R * H)


def score_layers(q_probes: Sequence[np.ndarray], k_layers: Sequence[np.ndarray],
                 weights: Optional[Sequence[float]] = None) -> np.ndarray:
    """Token scores from the attention of several layers: sum_l weights[l] * score(q_probes[l], k_layers[l]).

    Section 2 of the paper describes selectors that rank tokens by the attention of all layers, or of the last
    layer with probes that never saw the context (Section 3.3 compares the critical-layer analysis with both).
    They use the same per-layer quantity as `score`; all layers = equal weights over every layer, last layer =
    one term.  weights default to 1 / L (the mean); a common positive factor does not change the ranking.
    """
    L = len(k_layers)
    assert len(q_probes) == L and L > 0
    w = [1.0 / L] * L if weights is None else [float(x) for x in weights]
    out = np.zeros(np.asarray(k_layers[0]).shape[0], dtype=F64)
    for l in range(L):
        out += w[l] * score(q_probes[l], k_layers[l])
    return out


# --------------------------------------------------------------------------
# step 3: select
# --------------------------------------------------------------------------

def select_count(T: int, ratio: float) -> int:
    """N = ceil(ratio * T), guarded against ratio*T landing a hair above an
    integer, clamped to [0, T]."""
    n = int(math.ceil(ratio * T - 1e-9))
    return max(0, min(int(T), n))


def select(scores: np.ndarray, n: int) -> np.ndarray:
    """Indices of the n largest scores, ties to the lower index, ascending."""
    s = np.asarray(scores)
    order = np.argsort(-s, kind="stable")          # descending score, index order among equals
    return np.sort(order[:n]).astype(np.int64)


# --------------------------------------------------------------------------
# step 4: qkv
# --------------------------------------------------------------------------

def recompute_qkv(x: np.ndarray, w_qkv: np.ndarray, pos: np.ndarray, n_q_heads: int,
                  n_kv_heads: int, head_dim: int, base: float, style: int = 0
                  ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """[Q | K | V] = x W^T, split into heads, rotary embedding on Q and K.

    x [M, d_model]; w_qkv [(H + 2 H_kv) d, d_model], rows ordered Q heads,
    K heads, V heads; pos [M] absolute positions.
    """
    x = np.asarray(x, dtype=F64)
    w = np.asarray(w_qkv, dtype=F64)
    M = x.shape[0]
    y = x @ w.T
    nq, nk = n_q_heads * head_dim, n_kv_heads * head_dim
    q = y[:, :nq].reshape(M, n_q_heads, head_dim)
    k = y[:, nq:nq + nk].reshape(M, n_kv_heads, head_dim)
    v = y[:, nq + nk:].reshape(M, n_kv_heads, head_dim)
    return rope_at(q, pos, base, style), rope_at(k, pos, base, style), v.copy()


# --------------------------------------------------------------------------
# step 5: scatter
# --------------------------------------------------------------------------

def scatter(k_fused: np.ndarray, v_fused: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
            rows: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Copies of the fused caches with rows `rows` replaced by the new K/V rows."""
    k2, v2 = np.array(k_fused, copy=True), np.array(v_fused, copy=True)
    rows = np.asarray(rows, dtype=np.int64)
    if rows.size:
        k2[rows] = k_new
        v2[rows] = v_new
    return k2, v2


# --------------------------------------------------------------------------
# step 6: attn
# --------------------------------------------------------------------------

def recompute_attn(q_sel: np.ndarray, sel_pos: np.ndarray, k_fused: np.ndarray,
                   v_fused: np.ndarray, ctx_pos0: int = 0
                   ) -> Tuple[np.ndarray, np.ndarray]:
    """Causal attention of the selected rows over the (patched) fused cache.

    q_sel [N, H, d] at absolute positions sel_pos [N]; fused row j sits at
    position ctx_pos0 + j and is visible to row i iff ctx_pos0 + j <= sel_pos[i].
    Returns O [N, H, d] and the log-sum-exp of each row's logits [N, H]
    (-inf and a zero output row where nothing is visible).
    """
    q = np.asarray(q_sel, dtype=F64)
    k = np.asarray(k_fused, dtype=F64)
    v = np.asarray(v_fused, dtype=F64)
    N, H, d = q.shape
    T, Hkv, _ = k.shape
    G = H // Hkv
    o = np.zeros((N, H, d), dtype=F64)
    lse = np.full((N, H), -np.inf, dtype=F64)
    if N == 0 or T == 0:
        return o, lse
    visible = (ctx_pos0 + np.arange(T))[None, :] <= np.asarray(sel_pos)[:, None]   # [N, T]
    for h in range(H):
        g = h // G
        logits = (q[:, h, :] @ k[:, g, :].T) / math.sqrt(d)
        logits = np.where(visible, logits, -np.inf)
        m = logits.max(axis=1, keepdims=True)
        m = np.where(np.isfinite(m), m, 0.0)
        e = np.exp(logits - m)
        z = e.sum(axis=1, keepdims=True)
        p = np.divide(e, z, out=np.zeros_like(e), where=z > 0)
        o[:, h, :] = p @ v[:, g, :]
        with np.errstate(divide="ignore"):
            lse[:, h] = (m + np.log(z))[:, 0]
        lse[z[:, 0] == 0, h] = -np.inf
    return o, lse


# --------------------------------------------------------------------------
# the chained layer, and the backend the workload assembler borrows
# --------------------------------------------------------------------------

def fuse_layer(k_chunks, v_chunks, deltas, q_probe, x_ctx, w_qkv, ratio, n_q_heads, n_kv_heads,
               head_dim, base, style=0, sel_idx=None, quantize=None):
    """Steps 1-6 in the order rerope, score, select, qkv, scatter, attn.

    `quantize` (optional) is applied to every tensor the GPU path stores in its
    storage dtype (fused K/V, new Q/K/V rows, O) so the chained comparison sees
    the same stored values; pass sel_idx to force the selected set.
    """
    qz = quantize or (lambda a: a)
    k_f, v_f = rerope(k_chunks, v_chunks, deltas, base, style)
    k_f, v_f = qz(k_f), qz(v_f)
    s = score(q_probe, k_f)
    T = k_f.shape[0]
    n = select_count(T, ratio)
    idx = select(s, n) if sel_idx is None else np.asarray(sel_idx, dtype=np.int64)
    pos = idx.copy()
    q_s, k_s, v_s = recompute_qkv(np.asarray(x_ctx)[idx], w_qkv, pos, n_q_heads, n_kv_heads,
                                  head_dim, base, style)
    q_s, k_s, v_s = qz(q_s), qz(k_s), qz(v_s)
    k_p, v_p = scatter(k_f, v_f, k_s, v_s, idx)
    o, lse = recompute_attn(q_s, pos, k_p, v_p)
    return dict(k_fused=k_f, v_fused=v_f, score=s, sel_idx=idx, q_sel=q_s, k_sel=k_s, v_sel=v_s,
                k_patched=k_p, v_patched=v_p, o_sel=qz(o), lse=lse)


# --------------------------------------------------------------------------
# rest of the layer for the recomputed rows (next row after the six-call path)
# --------------------------------------------------------------------------
# Section 3.1, Phase 4 of the paper recomputes the selected tokens "layer by layer": after the sparse
# attention their hidden states must pass through the remainder of the transformer block before the next
# layer's projection.  The paper does not spell the block out; the model families it evaluates
# (Llama-3.1, Qwen3, Mistral) all use the pre-norm block with a gated SiLU feed-forward written below.

def rmsnorm(x: np.ndarray, weight: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2 over the last axis) + eps) * weight."""
    x = np.asarray(x, dtype=F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + F64(eps)) * np.asarray(weight, dtype=F64)


def linear(x: np.ndarray, w: np.ndarray, residual: Optional[np.ndarray] = None) -> np.ndarray:
    """y = x w^T (+ residual);  x [M, K], w [N, K] (one row per output feature)."""
    y = np.asarray(x, dtype=F64) @ np.asarray(w, dtype=F64).T
    if residual is not None:
        y = y + np.asarray(residual, dtype=F64)
    return y


def swiglu(gate_up: np.ndarray) -> np.ndarray:
    """silu(gate) * up for gate_up = [gate | up] along the last axis;  silu(g) = g / (1 + exp(-g))."""
    gu = np.asarray(gate_up, dtype=F64)
    f = gu.shape[-1] // 2
    g, u = gu[..., :f], gu[..., f:]
    return g / (1.0 + np.exp(-g)) * u


def layer_tail(h_in: np.ndarray, o_rows: np.ndarray, w_o: np.ndarray, norm_weight: np.ndarray,
               w_gate_up: np.ndarray, w_down: np.ndarray, eps: float, quantize=None) -> np.ndarray:
    """Hidden states of the rows after the block, given their attention outputs.

    h_in [M, d_model] block input (residual stream);  o_rows [M, H, d] attention output;
    w_o [d_model, H d];  norm_weight [d_model];  w_gate_up [2 F, d_model] (gate rows, then up rows);
    w_down [d_model, F].
        h1 = h_in + o w_o^T;  h_out = h1 + (silu(n w_gate^T) * (n w_up^T)) w_down^T,  n = rmsnorm(h1).
    `quantize` (optional) is applied to every stored intermediate, as the GPU path stores them in its
    element type between calls.
    """
    q = quantize if quantize is not None else (lambda a: a)
    m = o_rows.shape[0]
    h1 = q(linear(o_rows.reshape(m, -1), w_o, h_in))
    n = q(rmsnorm(h1, norm_weight, eps))
    gu = q(linear(n, w_gate_up))
    act = q(swiglu(gu))
    return q(linear(act, w_down, h1))


# --------------------------------------------------------------------------
# anchor extraction (offline, per chunk)
# --------------------------------------------------------------------------
# Section 3.1, Phase 1 of the paper keeps, for every precomputed chunk, a small fraction of its tokens - the ones
# with the largest key norm - as a compressed summary ("anchors").  The paper does not say which heads enter the
# norm; reading taken here: the Euclidean norm of the token's key over all KV heads of the layer at hand.

def key_norm(k: np.ndarray) -> np.ndarray:
    """norm[t] = sqrt(sum over heads and elements of k[t]^2);  k [T, H_kv, d]."""
    k = np.asarray(k, dtype=F64)
    return np.sqrt(np.sum(k * k, axis=(1, 2)))


def extract_anchors(k_chunk: np.ndarray, v_chunk: np.ndarray, n: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Indices (ascending; ties to the lower index) of the n tokens of the chunk with the largest key norm,
    and their K and V rows."""
    idx = select(key_norm(k_chunk), n)
    return idx, np.asarray(k_chunk)[idx], np.asarray(v_chunk)[idx]


class PlantOps:
    """Backend handed to the workload assembler by tests: the oracle's own
    projection and key shift."""

    def project_qkv(self, shape, x, w_qkv, pos):
        return recompute_qkv(x, w_qkv, pos, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                             shape.rope_base, shape.rope_style)

    def shift_keys(self, shape, k_rows, delta):
        k, _ = rerope([k_rows], None, [delta], shape.rope_base, shape.rope_style)
        return k
