// C-ABI entry points: host-side validation, then one launcher per call.
#include <cstdarg>
#include <cstdio>
#include <cmath>

#include "qcf_internal.h"

namespace qcf {

static thread_local char g_err[512] = "";

qcf_status fail(qcf_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

qcf_status check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return QCF_OK;
  return fail(QCF_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

qcf_status check_launch(const char* what) { return check_hip(hipGetLastError(), what); }

qcf_status allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  QCF_TRY(check_hip(hipGetDevice(&dev), "hipGetDevice"));
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return QCF_OK;
  QCF_TRY(check_hip(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes),
                    "hipFuncSetAttribute(MaxDynamicSharedMemorySize)"));
  done.fetch_or(bit, std::memory_order_release);
  return QCF_OK;
}

int compute_unit_count() {
  // read once (thread-safe initialisation); the launch shapes derived from it must not change between a
  // workspace-size query and the call that uses the workspace
  static const int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    return n;
  }();
  return cus;
}

static qcf_status check_desc(const qcf_layer_desc* d) {
  if (!d) return fail(QCF_ERR_INVALID_ARG, "layer descriptor is NULL");
  if (d->dtype != QCF_DTYPE_F32 && d->dtype != QCF_DTYPE_BF16)
    return fail(QCF_ERR_UNSUPPORTED, "dtype %d (supported: 0 = f32, 1 = bf16)", d->dtype);
  if (d->head_dim != 64 && d->head_dim != 128)
    return fail(QCF_ERR_UNSUPPORTED, "head_dim %d (supported: 64, 128)", d->head_dim);
  if (d->rope_style != QCF_ROPE_HALF_SPLIT && d->rope_style != QCF_ROPE_INTERLEAVED)
    return fail(QCF_ERR_UNSUPPORTED, "rope_style %d", d->rope_style);
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads != 0)
    return fail(QCF_ERR_INVALID_ARG, "heads: H=%d must be a positive multiple of H_kv=%d",
                d->n_q_heads, d->n_kv_heads);
  if (d->n_q_heads > 1024)
    return fail(QCF_ERR_UNSUPPORTED, "n_q_heads %d > 1024", d->n_q_heads);
  if (d->d_model <= 0 || d->d_model % 8 != 0)
    return fail(QCF_ERR_INVALID_ARG, "d_model %d must be a positive multiple of 8", d->d_model);
  if (!(d->rope_base > 1.0) || !std::isfinite(d->rope_base))
    return fail(QCF_ERR_INVALID_ARG, "rope_base must be finite and > 1");
  return QCF_OK;
}

static qcf_status need_ptr(const void* p, const char* name) {
  if (!p) return fail(QCF_ERR_INVALID_ARG, "%s is NULL", name);
  if (!aligned16(p)) return fail(QCF_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
  return QCF_OK;
}
static qcf_status opt_ptr(const void* p, const char* name) {
  if (p && !aligned16(p)) return fail(QCF_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
  return QCF_OK;
}
static qcf_status need_idx_ptr(const void* p, const char* name) {
  if (!p) return fail(QCF_ERR_INVALID_ARG, "%s is NULL", name);
  if (reinterpret_cast<uintptr_t>(p) & 3u) return fail(QCF_ERR_INVALID_ARG, "%s is misaligned", name);
  return QCF_OK;
}
static qcf_status need_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return QCF_OK;
  if (!ws) return fail(QCF_ERR_WORKSPACE_TOO_SMALL, "workspace is NULL, %zu bytes needed", need);
  if (!aligned16(ws)) return fail(QCF_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
  if (have < need)
    return fail(QCF_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", have, need);
  return QCF_OK;
}

constexpr int64_t kMaxRows = (int64_t)1 << 30;   // indices are int32

qcf_status check_score_args(const qcf_layer_desc* desc, int32_t B, const void* q_probe,
                            const int64_t* probe_off_dev, int64_t total_probe, const void* k_fused,
                            const int64_t* ctx_off_dev, int64_t total_ctx, const int32_t* probe_limit_dev,
                            float* score, bool* empty) {
  *empty = false;
  QCF_TRY(check_desc(desc));
  if (B < 0 || total_probe < 0 || total_ctx < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (total_ctx > kMaxRows || total_probe > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (B > 65535) return fail(QCF_ERR_UNSUPPORTED, "B %d > 65535", B);
  if (B == 0 || total_ctx == 0) { *empty = true; return QCF_OK; }
  QCF_TRY(need_ptr(score, "score"));
  QCF_TRY(need_idx_ptr(probe_off_dev, "probe_off_dev"));
  QCF_TRY(need_idx_ptr(ctx_off_dev, "ctx_off_dev"));
  if (total_probe > 0) QCF_TRY(need_ptr(q_probe, "q_probe"));
  QCF_TRY(need_ptr(k_fused, "k_fused"));
  if (probe_limit_dev) QCF_TRY(need_idx_ptr(probe_limit_dev, "probe_limit_dev"));
  return QCF_OK;
}

}  // namespace qcf

using namespace qcf;

extern "C" {

const char* qcf_status_string(qcf_status s) {
  switch (s) {
    case QCF_OK: return "QCF_OK";
    case QCF_ERR_INVALID_ARG: return "QCF_ERR_INVALID_ARG";
    case QCF_ERR_UNSUPPORTED: return "QCF_ERR_UNSUPPORTED";
    case QCF_ERR_WORKSPACE_TOO_SMALL: return "QCF_ERR_WORKSPACE_TOO_SMALL";
    case QCF_ERR_HIP: return "QCF_ERR_HIP";
  }
  return "QCF_ERR_UNKNOWN";
}

const char* qcf_last_error(void) { return g_err; }

int32_t qcf_version(void) { return 100; }

int64_t qcf_select_count(int64_t T, double ratio) {
  if (T <= 0 || !(ratio > 0.0)) return 0;
  double n = std::ceil(ratio * (double)T - 1e-9);
  if (n < 0) n = 0;
  if (n > (double)T) n = (double)T;
  return (int64_t)n;
}

// ---- rerope ---------------------------------------------------------------------
size_t qcf_rerope_workspace_bytes(const qcf_layer_desc* desc, int32_t n_chunks, int64_t total_rows) {
  if (check_desc(desc) != QCF_OK || n_chunks <= 0 || total_rows <= 0) return 0;
  return rerope_workspace(*desc, n_chunks, total_rows);
}

qcf_status qcf_rerope(const qcf_layer_desc* desc, const qcf_chunk* chunks_dev, int32_t n_chunks,
                      int64_t total_rows, void* k_fused, void* v_fused, void* workspace,
                      size_t workspace_bytes, void* stream) {
  QCF_TRY(check_desc(desc));
  if (n_chunks < 0 || total_rows < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (total_rows > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "total_rows %lld too large", (long long)total_rows);
  if (n_chunks == 0 || total_rows == 0) return QCF_OK;
  if (!chunks_dev || (reinterpret_cast<uintptr_t>(chunks_dev) & 7u))
    return fail(QCF_ERR_INVALID_ARG, "chunks_dev is NULL or misaligned");
  QCF_TRY(need_ptr(k_fused, "k_fused"));
  QCF_TRY(opt_ptr(v_fused, "v_fused"));
  QCF_TRY(need_ws(workspace, workspace_bytes, rerope_workspace(*desc, n_chunks, total_rows)));
  return launch_rerope(*desc, chunks_dev, n_chunks, total_rows, k_fused, v_fused, workspace,
                       (hipStream_t)stream);
}

// ---- score ----------------------------------------------------------------------
size_t qcf_score_workspace_bytes(const qcf_layer_desc* desc, int32_t B, int64_t total_probe,
                                 int64_t total_ctx) {
  if (check_desc(desc) != QCF_OK || B <= 0 || total_probe <= 0 || total_ctx <= 0) return 0;
  return score_workspace(*desc, B, total_probe, total_ctx);
}

qcf_status qcf_score(const qcf_layer_desc* desc, int32_t B, const void* q_probe,
                     const int64_t* probe_off_dev, int64_t total_probe, const void* k_fused,
                     const int64_t* ctx_off_dev, int64_t total_ctx, const int32_t* probe_limit_dev,
                     float* score, void* workspace, size_t workspace_bytes, void* stream) {
  bool empty = false;
  QCF_TRY(check_score_args(desc, B, q_probe, probe_off_dev, total_probe, k_fused, ctx_off_dev, total_ctx,
                           probe_limit_dev, score, &empty));
  if (empty) return QCF_OK;
  QCF_TRY(need_ws(workspace, workspace_bytes, score_workspace(*desc, B, total_probe, total_ctx)));
  return launch_score(*desc, B, q_probe, probe_off_dev, total_probe, k_fused, ctx_off_dev, total_ctx,
                      probe_limit_dev, score, 1.f, 0.f, workspace, (hipStream_t)stream);
}

qcf_status qcf_score_accumulate(const qcf_layer_desc* desc, int32_t B, const void* q_probe,
                                const int64_t* probe_off_dev, int64_t total_probe, const void* k_fused,
                                const int64_t* ctx_off_dev, int64_t total_ctx, const int32_t* probe_limit_dev,
                                float alpha, float beta, float* score, void* workspace, size_t workspace_bytes,
                                void* stream) {
  bool empty = false;
  QCF_TRY(check_score_args(desc, B, q_probe, probe_off_dev, total_probe, k_fused, ctx_off_dev, total_ctx,
                           probe_limit_dev, score, &empty));
  if (!std::isfinite(alpha) || !std::isfinite(beta)) return fail(QCF_ERR_INVALID_ARG, "alpha and beta must be finite");
  if (empty) return QCF_OK;
  QCF_TRY(need_ws(workspace, workspace_bytes, score_workspace(*desc, B, total_probe, total_ctx)));
  return launch_score(*desc, B, q_probe, probe_off_dev, total_probe, k_fused, ctx_off_dev, total_ctx,
                      probe_limit_dev, score, alpha, beta, workspace, (hipStream_t)stream);
}

// ---- select ---------------------------------------------------------------------
size_t qcf_select_workspace_bytes(int32_t B, int64_t total_ctx) {
  if (B <= 0 || total_ctx <= 0) return 0;
  return select_workspace(B, total_ctx);
}

qcf_status qcf_select(int32_t B, const float* score, const int64_t* ctx_off_dev, int64_t total_ctx,
                      const int64_t* sel_off_dev, int64_t total_sel, const int32_t* ctx_pos0_dev,
                      int32_t* sel_idx, int32_t* sel_row, int32_t* sel_pos, void* workspace,
                      size_t workspace_bytes, void* stream) {
  if (B < 0 || total_ctx < 0 || total_sel < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (total_ctx > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (total_sel > total_ctx) return fail(QCF_ERR_INVALID_ARG, "total_sel %lld > total_ctx %lld",
                                         (long long)total_sel, (long long)total_ctx);
  if (B > 65535) return fail(QCF_ERR_UNSUPPORTED, "B %d > 65535", B);
  if (B == 0 || total_sel == 0) return QCF_OK;
  QCF_TRY(need_idx_ptr(score, "score"));
  QCF_TRY(need_idx_ptr(ctx_off_dev, "ctx_off_dev"));
  QCF_TRY(need_idx_ptr(sel_off_dev, "sel_off_dev"));
  QCF_TRY(need_idx_ptr(sel_idx, "sel_idx"));
  if (ctx_pos0_dev) QCF_TRY(need_idx_ptr(ctx_pos0_dev, "ctx_pos0_dev"));
  if (sel_row) QCF_TRY(need_idx_ptr(sel_row, "sel_row"));
  if (sel_pos) QCF_TRY(need_idx_ptr(sel_pos, "sel_pos"));
  QCF_TRY(need_ws(workspace, workspace_bytes, select_workspace(B, total_ctx)));
  return launch_select(B, score, ctx_off_dev, total_ctx, sel_off_dev, total_sel, ctx_pos0_dev, sel_idx,
                       sel_row, sel_pos, workspace, (hipStream_t)stream);
}

// ---- qkv ------------------------------------------------------------------------
size_t qcf_recompute_qkv_workspace_bytes(const qcf_layer_desc* desc, int64_t M) {
  if (check_desc(desc) != QCF_OK || M <= 0) return 0;
  return qkv_workspace(*desc, M);
}

qcf_status qcf_recompute_qkv(const qcf_layer_desc* desc, const void* x, int64_t x_rows,
                             const int32_t* x_gather_dev, int64_t M, const void* w_qkv,
                             const int32_t* pos_dev, void* q_out, void* k_out, void* v_out,
                             void* workspace, size_t workspace_bytes, void* stream) {
  QCF_TRY(check_desc(desc));
  if (M < 0 || x_rows < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (M > kMaxRows || x_rows > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (M == 0) return QCF_OK;
  if (!x_gather_dev && x_rows < M)
    return fail(QCF_ERR_INVALID_ARG, "x has %lld rows, M = %lld", (long long)x_rows, (long long)M);
  // (the kernels replace an index outside x by row 0 and zero the result: x needs at least that row)
  if (x_rows == 0) return fail(QCF_ERR_INVALID_ARG, "x has no rows, M = %lld", (long long)M);
  if (!q_out && !k_out && !v_out) return QCF_OK;
  QCF_TRY(need_ptr(x, "x"));
  QCF_TRY(need_ptr(w_qkv, "w_qkv"));
  QCF_TRY(need_idx_ptr(pos_dev, "pos_dev"));
  if (x_gather_dev) QCF_TRY(need_idx_ptr(x_gather_dev, "x_gather_dev"));
  QCF_TRY(opt_ptr(q_out, "q_out"));
  QCF_TRY(opt_ptr(k_out, "k_out"));
  QCF_TRY(opt_ptr(v_out, "v_out"));
  QCF_TRY(need_ws(workspace, workspace_bytes, qkv_workspace(*desc, M)));
  return launch_qkv(*desc, x, x_rows, x_gather_dev, M, w_qkv, pos_dev, q_out, k_out, v_out, nullptr, nullptr,
                    nullptr, 0, workspace, (hipStream_t)stream);
}

qcf_status qcf_recompute_qkv_scatter(const qcf_layer_desc* desc, const void* x, int64_t x_rows,
                                     const int32_t* x_gather_dev, int64_t M, const void* w_qkv,
                                     const int32_t* pos_dev, void* q_out, void* k_out, void* v_out,
                                     const int32_t* dst_rows_dev, void* k_fused, void* v_fused,
                                     int64_t total_rows, void* workspace, size_t workspace_bytes, void* stream) {
  QCF_TRY(check_desc(desc));
  if (M < 0 || x_rows < 0 || total_rows < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (M > kMaxRows || x_rows > kMaxRows || total_rows > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (M == 0) return QCF_OK;
  if (!x_gather_dev && x_rows < M)
    return fail(QCF_ERR_INVALID_ARG, "x has %lld rows, M = %lld", (long long)x_rows, (long long)M);
  if (x_rows == 0) return fail(QCF_ERR_INVALID_ARG, "x has no rows, M = %lld", (long long)M);
  QCF_TRY(need_ptr(x, "x"));
  QCF_TRY(need_ptr(w_qkv, "w_qkv"));
  QCF_TRY(need_idx_ptr(pos_dev, "pos_dev"));
  if (x_gather_dev) QCF_TRY(need_idx_ptr(x_gather_dev, "x_gather_dev"));
  QCF_TRY(opt_ptr(q_out, "q_out"));
  QCF_TRY(need_ptr(k_out, "k_out"));
  QCF_TRY(need_ptr(v_out, "v_out"));
  QCF_TRY(need_idx_ptr(dst_rows_dev, "dst_rows_dev"));
  QCF_TRY(need_ptr(k_fused, "k_fused"));
  QCF_TRY(need_ptr(v_fused, "v_fused"));
  QCF_TRY(need_ws(workspace, workspace_bytes, qkv_workspace(*desc, M)));
  return launch_qkv(*desc, x, x_rows, x_gather_dev, M, w_qkv, pos_dev, q_out, k_out, v_out, dst_rows_dev, k_fused,
                    v_fused, total_rows, workspace, (hipStream_t)stream);
}

// ---- scatter --------------------------------------------------------------------
qcf_status qcf_scatter(const qcf_layer_desc* desc, const void* k_new, const void* v_new,
                       const int32_t* dst_rows_dev, int64_t M, void* k_fused, void* v_fused,
                       int64_t total_rows, void* stream) {
  QCF_TRY(check_desc(desc));
  if (M < 0 || total_rows < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (M > kMaxRows || total_rows > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (M == 0 || total_rows == 0) return QCF_OK;
  QCF_TRY(need_ptr(k_new, "k_new"));
  QCF_TRY(need_ptr(k_fused, "k_fused"));
  if ((v_new == nullptr) != (v_fused == nullptr))
    return fail(QCF_ERR_INVALID_ARG, "v_new and v_fused must both be given or both be NULL");
  QCF_TRY(opt_ptr(v_new, "v_new"));
  QCF_TRY(opt_ptr(v_fused, "v_fused"));
  QCF_TRY(need_idx_ptr(dst_rows_dev, "dst_rows_dev"));
  return launch_scatter(*desc, k_new, v_new, dst_rows_dev, M, k_fused, v_fused, total_rows,
                        (hipStream_t)stream);
}

// ---- attn -----------------------------------------------------------------------
size_t qcf_recompute_attn_workspace_bytes(const qcf_layer_desc* desc, int32_t B, int64_t total_sel,
                                          int64_t total_ctx) {
  if (check_desc(desc) != QCF_OK || B <= 0 || total_sel <= 0 || total_ctx <= 0) return 0;
  return attn_workspace(*desc, B, total_sel, total_ctx);
}

qcf_status qcf_recompute_attn(const qcf_layer_desc* desc, int32_t B, const void* q_sel,
                              const int32_t* sel_pos_dev, const int64_t* sel_off_dev, int64_t total_sel,
                              const void* k_fused, const void* v_fused, const int64_t* ctx_off_dev,
                              int64_t total_ctx, const int32_t* ctx_pos0_dev, void* o_out, float* lse_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
  QCF_TRY(check_desc(desc));
  if (B < 0 || total_sel < 0 || total_ctx < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (total_sel > kMaxRows || total_ctx > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (B > 65535) return fail(QCF_ERR_UNSUPPORTED, "B %d > 65535", B);
  if (B == 0 || total_sel == 0) return QCF_OK;
  QCF_TRY(need_ptr(q_sel, "q_sel"));
  QCF_TRY(need_ptr(o_out, "o_out"));
  QCF_TRY(need_idx_ptr(sel_pos_dev, "sel_pos_dev"));
  QCF_TRY(need_idx_ptr(sel_off_dev, "sel_off_dev"));
  QCF_TRY(need_idx_ptr(ctx_off_dev, "ctx_off_dev"));
  if (total_ctx > 0) {
    QCF_TRY(need_ptr(k_fused, "k_fused"));
    QCF_TRY(need_ptr(v_fused, "v_fused"));
  }
  if (ctx_pos0_dev) QCF_TRY(need_idx_ptr(ctx_pos0_dev, "ctx_pos0_dev"));
  if (lse_out) QCF_TRY(need_idx_ptr(lse_out, "lse_out"));
  QCF_TRY(need_ws(workspace, workspace_bytes, attn_workspace(*desc, B, total_sel, total_ctx)));
  return launch_attn(*desc, B, q_sel, sel_pos_dev, sel_off_dev, total_sel, k_fused, v_fused, ctx_off_dev,
                     total_ctx, ctx_pos0_dev, o_out, lse_out, workspace, (hipStream_t)stream);
}

// ---- rest of the layer ------------------------------------------------------------
static qcf_status check_dtype(const qcf_layer_desc* d) {
  if (!d) return fail(QCF_ERR_INVALID_ARG, "layer descriptor is NULL");
  if (d->dtype != QCF_DTYPE_F32 && d->dtype != QCF_DTYPE_BF16)
    return fail(QCF_ERR_UNSUPPORTED, "dtype %d (supported: 0 = f32, 1 = bf16)", d->dtype);
  return QCF_OK;
}

size_t qcf_linear_workspace_bytes(const qcf_layer_desc* desc, int64_t M, int32_t K, int32_t N) {
  if (check_dtype(desc) != QCF_OK || M <= 0 || K <= 0 || N <= 0) return 0;
  return linear_workspace(*desc, M, K, N);
}

qcf_status qcf_linear(const qcf_layer_desc* desc, const void* x, int64_t M, int32_t K, const void* w,
                      int32_t N, const void* residual, void* out, void* workspace, size_t workspace_bytes,
                      void* stream) {
  QCF_TRY(check_dtype(desc));
  if (M < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (M > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (K <= 0 || N <= 0 || K % 8 != 0 || N % 8 != 0)
    return fail(QCF_ERR_INVALID_ARG, "K = %d and N = %d must be positive multiples of 8", K, N);
  if (M == 0) return QCF_OK;
  QCF_TRY(need_ptr(x, "x"));
  QCF_TRY(need_ptr(w, "w"));
  QCF_TRY(opt_ptr(residual, "residual"));
  QCF_TRY(need_ptr(out, "out"));
  QCF_TRY(need_ws(workspace, workspace_bytes, linear_workspace(*desc, M, K, N)));
  return launch_linear(*desc, x, M, K, w, N, residual, out, workspace, (hipStream_t)stream);
}

qcf_status qcf_rmsnorm(const qcf_layer_desc* desc, const void* x, const void* weight, double eps, int64_t M,
                       int32_t cols, void* out, void* stream) {
  QCF_TRY(check_dtype(desc));
  if (M < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (M > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (cols <= 0 || cols % 8 != 0) return fail(QCF_ERR_INVALID_ARG, "cols = %d must be a positive multiple of 8", cols);
  if (!(eps >= 0.0) || !std::isfinite(eps)) return fail(QCF_ERR_INVALID_ARG, "eps must be finite and >= 0");
  if (M == 0) return QCF_OK;
  QCF_TRY(need_ptr(x, "x"));
  QCF_TRY(need_ptr(weight, "weight"));
  QCF_TRY(need_ptr(out, "out"));
  return launch_rmsnorm(*desc, x, weight, eps, M, cols, out, (hipStream_t)stream);
}

qcf_status qcf_swiglu(const qcf_layer_desc* desc, const void* gate_up, int64_t M, int32_t F, void* out,
                      void* stream) {
  QCF_TRY(check_dtype(desc));
  if (M < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (M > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (F <= 0 || F % 8 != 0) return fail(QCF_ERR_INVALID_ARG, "F = %d must be a positive multiple of 8", F);
  if (M == 0) return QCF_OK;
  QCF_TRY(need_ptr(gate_up, "gate_up"));
  QCF_TRY(need_ptr(out, "out"));
  return launch_swiglu(*desc, gate_up, M, F, out, (hipStream_t)stream);
}

// ---- anchor extraction ------------------------------------------------------------
qcf_status qcf_key_norm(const qcf_layer_desc* desc, const void* k, int64_t rows, float* norm, void* stream) {
  QCF_TRY(check_desc(desc));
  if (rows < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (rows > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (rows == 0) return QCF_OK;
  QCF_TRY(need_ptr(k, "k"));
  QCF_TRY(need_idx_ptr(norm, "norm"));
  return launch_key_norm(*desc, k, rows, norm, (hipStream_t)stream);
}

qcf_status qcf_gather(const qcf_layer_desc* desc, const void* k_src, const void* v_src,
                      const int32_t* src_rows_dev, int64_t M, int64_t total_rows, void* k_out, void* v_out,
                      void* stream) {
  QCF_TRY(check_desc(desc));
  if (M < 0 || total_rows < 0) return fail(QCF_ERR_INVALID_ARG, "negative size");
  if (M > kMaxRows || total_rows > kMaxRows) return fail(QCF_ERR_UNSUPPORTED, "too many rows");
  if (M == 0) return QCF_OK;
  QCF_TRY(need_ptr(k_src, "k_src"));
  QCF_TRY(need_ptr(k_out, "k_out"));
  QCF_TRY(need_idx_ptr(src_rows_dev, "src_rows_dev"));
  if ((v_src == nullptr) != (v_out == nullptr)) return fail(QCF_ERR_INVALID_ARG, "v_src and v_out must both be given or both be NULL");
  QCF_TRY(opt_ptr(v_src, "v_src"));
  QCF_TRY(opt_ptr(v_out, "v_out"));
  return launch_gather(*desc, k_src, v_src, src_rows_dev, M, total_rows, k_out, v_out, (hipStream_t)stream);
}

}  // extern "C"
