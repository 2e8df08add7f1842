// Step 5: write recomputed K/V rows back into the fused cache (Section 3.1, Phase 4).
// Pure data movement: one 16-byte vector per thread, rows addressed through dst_rows.
#include "qcf_internal.h"

namespace qcf {
namespace {

__global__ __launch_bounds__(256) void scatter_kernel(const u32x4* __restrict__ k_new,
                                                      const u32x4* __restrict__ v_new,
                                                      const int32_t* __restrict__ rows, int64_t M,
                                                      int vec_per_row, u32x4* __restrict__ kf,
                                                      u32x4* __restrict__ vf, int64_t total_rows) {
  const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (item >= M * vec_per_row) return;
  const int64_t m = item / vec_per_row;
  const int c = (int)(item - m * vec_per_row);
  const int64_t dst = rows[m];
  if (dst < 0 || dst >= total_rows) return;
  kf[dst * vec_per_row + c] = k_new[item];
  if (vf) vf[dst * vec_per_row + c] = v_new[item];
}

}  // namespace

qcf_status launch_scatter(const qcf_layer_desc& L, const void* k_new, const void* v_new,
                          const int32_t* rows, int64_t M, void* kf, void* vf, int64_t total_rows,
                          hipStream_t st) {
  const int vec_per_row = L.n_kv_heads * L.head_dim * elem_size(L.dtype) / 16;
  const int64_t items = M * vec_per_row;
  const int64_t blocks = (items + 255) / 256;
  if (blocks > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "scatter: too many rows");
  scatter_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(
      static_cast<const u32x4*>(k_new), static_cast<const u32x4*>(v_new), rows, M, vec_per_row,
      static_cast<u32x4*>(kf), static_cast<u32x4*>(vf), total_rows);
  return check_launch("scatter");
}

}  // namespace qcf
