/*
 * qcf.h - C ABI of the MI355X (gfx950) per-layer query-centric KV-cache fusion library.
 *
 * One decoder layer of the cache-fusion step of QCFuse (Section 3.1, Phases 3-4, and
 * Section 3.2 of the paper): chunk KV caches that were prefilled independently are
 * concatenated, the critical layer's keys are scored against the probe rows (user
 * query + summary anchors), the Top-N context tokens are selected, their Q/K/V are
 * recomputed, written back, and they attend causally over the patched cache.
 *
 *   call order for one layer:
 *     qcf_rerope -> [critical layer only: qcf_score -> qcf_select] ->
 *     qcf_recompute_qkv -> qcf_scatter -> qcf_recompute_attn
 *   (qcf_recompute_qkv_scatter does the fourth and the fifth in one call)
 *   (attention runs after the scatter: a recomputed row must see the recomputed K/V
 *   of the other selected rows, otherwise recomputing every token would not reproduce
 *   full causal prefill - the paper's "Full Computation" end point.)
 *
 * Conventions, for every entry point
 *   - All tensor pointers are DEVICE pointers (HIP), 16-byte aligned, dense row-major,
 *     owned by the caller.  Descriptor structs passed by pointer without the `_dev`
 *     suffix live in HOST memory.  The library never allocates or frees memory; scratch
 *     comes from a caller-supplied device `workspace` of at least
 *     qcf_<call>_workspace_bytes(...) bytes (its contents are undefined afterwards).
 *   - Calls validate their scalar arguments on the host, enqueue kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and return without
 *     synchronising.  Tables that live on the device (chunk table, offsets, indices)
 *     cannot be validated on the host: kernels clamp every index they read against the
 *     totals passed by value, so inconsistent tables give wrong results, never
 *     out-of-bounds accesses.
 *   - Empty work (zero rows, zero requests) returns QCF_OK and launches nothing.
 *   - Supported: dtype f32 or bf16; head_dim 64 or 128; n_q_heads a multiple of
 *     n_kv_heads; rope_style 0 (pairs (i, i+d/2)) or 1 (pairs (2i, 2i+1)).  Anything
 *     else returns QCF_ERR_UNSUPPORTED.  On error nothing is enqueued and
 *     qcf_last_error() describes the problem (thread-local text).
 *   - Element type of q/k/v/x/w/o buffers is desc->dtype; scores and log-sum-exp are
 *     float32; offsets are int64; indices and positions are int32.
 *   - Batches are ragged: request b owns context rows [ctx_off[b], ctx_off[b+1]) of the
 *     fused cache, probe rows [probe_off[b], probe_off[b+1]) and selected rows
 *     [sel_off[b], sel_off[b+1]).  Offset arrays have B+1 entries, start at 0, are
 *     non-decreasing and end at the matching total.
 */
#ifndef QCF_H_
#define QCF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum qcf_status {
  QCF_OK = 0,
  QCF_ERR_INVALID_ARG = 1,
  QCF_ERR_UNSUPPORTED = 2,
  QCF_ERR_WORKSPACE_TOO_SMALL = 3,
  QCF_ERR_HIP = 4
} qcf_status;

enum { QCF_DTYPE_F32 = 0, QCF_DTYPE_BF16 = 1 };
enum { QCF_ROPE_HALF_SPLIT = 0, QCF_ROPE_INTERLEAVED = 1 };

/* Geometry of one attention layer (host struct). */
typedef struct qcf_layer_desc {
  int32_t d_model;     /* hidden size */
  int32_t n_q_heads;   /* H */
  int32_t n_kv_heads;  /* H_kv; query head h reads KV head h / (H / H_kv) */
  int32_t head_dim;    /* d: 64 or 128 */
  double  rope_base;   /* theta_i = rope_base^(-2i/d) */
  int32_t rope_style;  /* QCF_ROPE_* */
  int32_t dtype;       /* QCF_DTYPE_* */
} qcf_layer_desc;

/* One independently prefilled context chunk (element of a DEVICE array).  The chunk
 * cache is read-only: it may be shared by many requests at different offsets. */
typedef struct qcf_chunk {
  const void* k_src;   /* [len, H_kv, d] keys carrying the rotation of their local positions */
  const void* v_src;   /* [len, H_kv, d] values (ignored when v_fused is NULL) */
  int32_t len;         /* tokens in the chunk (> 0) */
  int32_t src_pos0;    /* local position its first token was prefilled at */
  int64_t dst_row;     /* first row of the chunk in the fused cache */
  int32_t dst_pos0;    /* global position of its first token in the fused prompt */
  int32_t reserved;    /* set to 0 */
} qcf_chunk;

const char* qcf_status_string(qcf_status s);
/* Text of the last error raised on the calling thread ("" if none). */
const char* qcf_last_error(void);
/* Library version, major*10000 + minor*100 + patch. */
int32_t qcf_version(void);

/* ---- step 1: re-rotation + concatenation ("location-independent" chunk reuse,
 * Section 3.2 indexing module / Section 4 scenario 2).
 * For every chunk c and token t < len: fused K row dst_row + t = key row t with every
 * rotary pair turned by (dst_pos0 - src_pos0) * theta_i; fused V row = value row t.
 * chunks_dev: DEVICE array of n_chunks entries sorted by dst_row, ranges disjoint and
 * inside [0, total_rows); rows covered by no chunk are left untouched.  v_fused may be
 * NULL (keys only, e.g. loading just the critical layer's K for scoring). */
size_t qcf_rerope_workspace_bytes(const qcf_layer_desc* desc, int32_t n_chunks, int64_t total_rows);
qcf_status qcf_rerope(const qcf_layer_desc* desc, const qcf_chunk* chunks_dev, int32_t n_chunks,
                      int64_t total_rows, void* k_fused, void* v_fused,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- step 2: critical-layer attention analysis (Section 3.1 Phase 3; Section 3.2,
 * query-related token selector: multi-head attention weights, averaged).
 * score[j] = mean over the request's probe rows i and all heads h of
 *            softmax_j( q_probe[i,h] . k_fused[j, h/G] / sqrt(d) ), softmax over the
 * request's own context rows.  q_probe [total_probe, H, d] holds rotated queries
 * (anchor rows and user-query rows alike).  probe_limit (NULL = none): per probe row,
 * the number of leading context rows of its request it may see; a row that sees nothing
 * contributes 0 (it still counts in the mean).  score [total_ctx] float32; each request's
 * scores sum to 1 when every probe row sees at least one token (always, without
 * probe_limit); a request without probe rows gets zeros.  Deterministic: no
 * floating-point atomics. */
size_t qcf_score_workspace_bytes(const qcf_layer_desc* desc, int32_t B, int64_t total_probe,
                                 int64_t total_ctx);
qcf_status qcf_score(const qcf_layer_desc* desc, int32_t B,
                     const void* q_probe, const int64_t* probe_off_dev, int64_t total_probe,
                     const void* k_fused, const int64_t* ctx_off_dev, int64_t total_ctx,
                     const int32_t* probe_limit_dev, float* score,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Scoring over several layers (Section 2 and Section 3.3 of the paper: the selectors it compares its critical-layer
 * analysis with rank tokens by the attention of all layers, or of the last layer with probes that have not seen
 * the context).  Same computation as qcf_score for one layer, blended into what `score` already holds:
 *   score[j] = beta * score[j] + alpha * (this call's mean attention on token j)
 * beta = 0 ignores (never reads) the old contents.  A sum over L layers is L calls, the first with beta = 0 and the
 * others with beta = 1; alpha = 1 / L gives the mean (the ranking does not depend on a positive common factor).
 * The last-layer variant is one call on the last layer's keys with probe rows projected from the bare query.
 * Workspace as for qcf_score.  Deterministic. */
qcf_status qcf_score_accumulate(const qcf_layer_desc* desc, int32_t B,
                                const void* q_probe, const int64_t* probe_off_dev, int64_t total_probe,
                                const void* k_fused, const int64_t* ctx_off_dev, int64_t total_ctx,
                                const int32_t* probe_limit_dev, float alpha, float beta, float* score,
                                void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): qcf_score with its scratch in a buffer built
 * into the library (QCF_SCORE_STATIC_SCRATCH_BYTES of device memory per GPU, held until the process
 * ends).  Same arguments, results and kernels as qcf_score, without the workspace.  It allocates and frees
 * nothing.  A problem whose qcf_score_workspace_bytes(...) exceeds the built-in buffer returns
 * QCF_ERR_WORKSPACE_TOO_SMALL (nothing is enqueued; qcf_last_error() gives both sizes).  All calls on one
 * GPU share that GPU's buffer: calls that may overlap in time on one GPU (different streams, or several
 * threads) race on it; calls ordered on one stream are safe. */
#define QCF_SCORE_STATIC_SCRATCH_BYTES (16u << 20)
qcf_status qcf_score_static(const qcf_layer_desc* desc, int32_t B,
                            const void* q_probe, const int64_t* probe_off_dev, int64_t total_probe,
                            const void* k_fused, const int64_t* ctx_off_dev, int64_t total_ctx,
                            const int32_t* probe_limit_dev, float* score, void* stream);

/* ---- step 3: Top-N selection (Section 3.1 Phase 3, "Top-N"; the recompute ratio of
 * Section 3.2).  Host helper: N = ceil(ratio * T) (guarded by 1e-9), clamped to [0, T]. */
int64_t qcf_select_count(int64_t T, double ratio);
/* For request b, the N_b = sel_off[b+1]-sel_off[b] highest-scoring of its context rows,
 * ties to the lower index, written in ascending order.  Outputs (each may be NULL
 * except sel_idx): sel_idx = request-local index; sel_row = ctx_off[b] + index (row in
 * the fused cache / hidden-state matrix); sel_pos = ctx_pos0[b] + index (absolute
 * position; ctx_pos0_dev NULL = 0).  N_b is clamped to T_b.  Exact and deterministic. */
size_t qcf_select_workspace_bytes(int32_t B, int64_t total_ctx);
qcf_status qcf_select(int32_t B, const float* score, const int64_t* ctx_off_dev, int64_t total_ctx,
                      const int64_t* sel_off_dev, int64_t total_sel, const int32_t* ctx_pos0_dev,
                      int32_t* sel_idx, int32_t* sel_row, int32_t* sel_pos,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- step 4: Q/K/V of the selected tokens (Section 3.1 Phase 4, discrete token
 * recomputation).  For m < M: y = x[row(m)] . w_qkv^T, row(m) = x_gather[m] (or m when
 * x_gather is NULL; indices outside [0, x_rows) produce zero rows; x_rows must be > 0 and,
 * without x_gather, >= M), split into H query
 * heads, H_kv key heads, H_kv value heads; rotary embedding at pos[m] on Q and K.
 * x [x_rows, d_model]; w_qkv [(H + 2 H_kv) d, d_model]; outputs q_out [M, H, d],
 * k_out / v_out [M, H_kv, d]; any output pointer may be NULL to skip that part
 * (e.g. only Q for probe rows).  fp32 accumulation, outputs stored in desc->dtype. */
size_t qcf_recompute_qkv_workspace_bytes(const qcf_layer_desc* desc, int64_t M);
qcf_status qcf_recompute_qkv(const qcf_layer_desc* desc, const void* x, int64_t x_rows,
                             const int32_t* x_gather_dev, int64_t M, const void* w_qkv,
                             const int32_t* pos_dev, void* q_out, void* k_out, void* v_out,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ---- steps 4 and 5 in one call (Section 3.1 Phase 4: the recomputed K/V replace the stale rows of the
 * fused cache).  Same results as qcf_recompute_qkv followed by qcf_scatter(k_out, v_out, dst_rows_dev, M,
 * k_fused, v_fused, total_rows): q_out / k_out / v_out as above (k_out and v_out are required here), and row
 * dst_rows[m] of k_fused / v_fused <- row m of k_out / v_out (rows outside [0, total_rows) are skipped;
 * dst_rows must not repeat).  On the bf16 MFMA path the cache rows are written from the projection's epilogue,
 * without a second pass over them.  Workspace: qcf_recompute_qkv_workspace_bytes. */
qcf_status qcf_recompute_qkv_scatter(const qcf_layer_desc* desc, const void* x, int64_t x_rows,
                                     const int32_t* x_gather_dev, int64_t M, const void* w_qkv,
                                     const int32_t* pos_dev, void* q_out, void* k_out, void* v_out,
                                     const int32_t* dst_rows_dev, void* k_fused, void* v_fused,
                                     int64_t total_rows, void* workspace, size_t workspace_bytes, void* stream);

/* ---- step 5: write the recomputed K/V rows into the fused cache (Section 3.1 Phase 4,
 * "updated" KV).  Row dst_rows[m] of k_fused / v_fused <- row m of k_new / v_new; rows
 * outside [0, total_rows) are skipped; other rows are untouched.  dst_rows must not
 * repeat.  v_new/v_fused may both be NULL. */
qcf_status qcf_scatter(const qcf_layer_desc* desc, const void* k_new, const void* v_new,
                       const int32_t* dst_rows_dev, int64_t M, void* k_fused, void* v_fused,
                       int64_t total_rows, void* stream);

/* ---- step 6: location-aware sparse causal attention (Section 3.2, the kernel that
 * takes the table of discrete token indices with their absolute locations).
 * o[i,h] = sum_j softmax_j( q_sel[i,h] . k_fused[j, h/G] / sqrt(d) ) v_fused[j, h/G]
 * over the context rows j of row i's request with ctx_pos0[b] + j <= sel_pos[i]
 * (ctx_pos0_dev NULL = 0).  The rows of a request may come in any order and positions may
 * repeat; ascending order (what qcf_select produces) balances the work best, because rows
 * are processed in blocks of consecutive rows and a block runs as far as its highest
 * position.  o_out [total_sel, H, d]; lse_out (may be NULL) [total_sel, H]
 * float32 natural-log sum-exp of the scaled logits.  A row that sees nothing gets a zero
 * output row and lse = -inf. */
size_t qcf_recompute_attn_workspace_bytes(const qcf_layer_desc* desc, int32_t B,
                                          int64_t total_sel, int64_t total_ctx);
qcf_status qcf_recompute_attn(const qcf_layer_desc* desc, int32_t B,
                              const void* q_sel, const int32_t* sel_pos_dev,
                              const int64_t* sel_off_dev, int64_t total_sel,
                              const void* k_fused, const void* v_fused,
                              const int64_t* ctx_off_dev, int64_t total_ctx,
                              const int32_t* ctx_pos0_dev, void* o_out, float* lse_out,
                              void* workspace, size_t workspace_bytes, void* stream);

/* ---- rest of the layer for the recomputed rows (Section 3.1 Phase 4: the selected tokens are
 * recomputed "layer by layer", so after the sparse attention their hidden states pass through the
 * remainder of the transformer block before the next layer's projection.  The paper does not spell
 * the block out; these are the pieces of the pre-norm block with a gated SiLU feed-forward that the
 * model families it evaluates share).  Element type desc->dtype (only the dtype field of the
 * descriptor is used), fp32 accumulation, results rounded once when stored.
 *
 * qcf_linear:  out[m, :] = x[m, :] . w^T (+ residual[m, :]);  x [M, K], w [N, K] (one row per
 *   output feature), residual / out [M, N].  residual may be NULL, and may be the same buffer as out.
 *   K and N must be multiples of 8.  Uses the MFMA path when dtype is bf16, K % 64 == 0, N % 128 == 0.
 * qcf_rmsnorm: out[m, :] = x[m, :] / sqrt(mean_c x[m, c]^2 + eps) * weight[:];  x / out [M, cols],
 *   weight [cols]; cols a multiple of 8; out may be the same buffer as x.
 * qcf_swiglu:  out[m, f] = silu(gate_up[m, f]) * gate_up[m, F + f], silu(g) = g / (1 + exp(-g));
 *   gate_up [M, 2F], out [M, F]; F a multiple of 8.
 * One block for M rows:  h1 = linear(o, w_o, residual = h_in);  n = rmsnorm(h1);
 *   h_out = linear(swiglu(linear(n, w_gate_up)), w_down, residual = h1). */
size_t qcf_linear_workspace_bytes(const qcf_layer_desc* desc, int64_t M, int32_t K, int32_t N);
qcf_status qcf_linear(const qcf_layer_desc* desc, const void* x, int64_t M, int32_t K,
                      const void* w, int32_t N, const void* residual, void* out,
                      void* workspace, size_t workspace_bytes, void* stream);
qcf_status qcf_rmsnorm(const qcf_layer_desc* desc, const void* x, const void* weight, double eps,
                       int64_t M, int32_t cols, void* out, void* stream);
qcf_status qcf_swiglu(const qcf_layer_desc* desc, const void* gate_up, int64_t M, int32_t F,
                      void* out, void* stream);

/* ---- anchor extraction (Section 3.1 Phase 1, offline: for every precomputed chunk "a minor fraction
 * of tokens with the highest key-norm values" is kept as a compressed summary).  The paper does not say
 * which heads enter the norm; here norm[t] = sqrt(sum over the KV heads and elements of k[t]^2) of the
 * layer at hand.  k [rows, H_kv, d]; norm [rows] float32.  The anchors of a set of chunks are then
 * qcf_select(B = number of chunks, score = norm, ctx_off = chunk boundaries, sel_off = anchors per
 * chunk) followed by qcf_gather of the K/V rows. */
qcf_status qcf_key_norm(const qcf_layer_desc* desc, const void* k, int64_t rows, float* norm, void* stream);
/* Row m of k_out / v_out <- row src_rows[m] of k_src / v_src (rows of H_kv * d elements); an index
 * outside [0, total_rows) gives a zero row.  v_src and v_out may both be NULL.  The inverse of qcf_scatter. */
qcf_status qcf_gather(const qcf_layer_desc* desc, const void* k_src, const void* v_src,
                      const int32_t* src_rows_dev, int64_t M, int64_t total_rows, void* k_out, void* v_out,
                      void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QCF_H_ */
