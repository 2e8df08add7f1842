// Step 5: write recomputed K/V rows back into the fused cache (Section 3.1, Phase 4).
// Pure data movement: one 16-byte vector per thread, rows addressed through dst_rows.
// Also here, for the offline anchor extraction of Section 3.1 Phase 1: the per-token key norm (one wave
// per token row, fixed-order reduction) and the inverse copy (gather of K/V rows by index).
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

__global__ __launch_bounds__(256) void gather_kernel(const u32x4* __restrict__ k_src, const u32x4* __restrict__ v_src,
                                                     const int32_t* __restrict__ rows, int64_t M, int vec_per_row,
                                                     int64_t src_rows, u32x4* __restrict__ k_out,
                                                     u32x4* __restrict__ v_out) {
  const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (item >= M * vec_per_row) return;
  const int64_t m = item / vec_per_row;
  const int c = (int)(item - m * vec_per_row);
  const int64_t src = rows[m];
  const bool ok = src >= 0 && src < src_rows;                 // rows outside the source come out as zeros
  const u32x4 zero = {0u, 0u, 0u, 0u};
  k_out[item] = ok ? k_src[src * vec_per_row + c] : zero;
  if (v_out) v_out[item] = ok ? v_src[src * vec_per_row + c] : zero;
}

// norm[t] = sqrt(sum of squares of row t); one wave per row, four rows per workgroup
template <typename T>
__global__ __launch_bounds__(256) void key_norm_kernel(const T* __restrict__ k, int64_t rows, int row_elems,
                                                       float* __restrict__ norm) {
  constexpr int VEC = Elem<T>::kVec;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* src = k + row * row_elems;
  float ss = 0.f;
  for (int v = lane; v < row_elems / VEC; v += 64) {
    float f[VEC];
    Vec16<T>::unpack(*reinterpret_cast<const u32x4*>(src + v * VEC), f);
#pragma unroll
    for (int e = 0; e < VEC; ++e) ss += f[e] * f[e];
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) ss += __shfl_xor(ss, d, 64);
  if (lane == 0) norm[row] = sqrtf(ss);
}

}  // namespace

qcf_status launch_gather(const qcf_layer_desc& L, const void* k_src, const void* v_src, const int32_t* rows,
                         int64_t M, int64_t src_rows, void* k_out, void* v_out, hipStream_t st) {
  const int vec_per_row = L.n_kv_heads * L.head_dim * elem_size(L.dtype) / 16;
  const int64_t blocks = (M * vec_per_row + 255) / 256;
  if (blocks > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "gather: too many rows");
  gather_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(
      static_cast<const u32x4*>(k_src), static_cast<const u32x4*>(v_src), rows, M, vec_per_row, src_rows,
      static_cast<u32x4*>(k_out), static_cast<u32x4*>(v_out));
  return check_launch("gather");
}

qcf_status launch_key_norm(const qcf_layer_desc& L, const void* k, int64_t rows, float* norm, hipStream_t st) {
  const int row_elems = L.n_kv_heads * L.head_dim;
  const int64_t blocks = (rows + 3) / 4;
  if (blocks > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "key norm: too many rows");
  if (L.dtype == QCF_DTYPE_BF16)
    key_norm_kernel<bf16_t><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<const bf16_t*>(k), rows,
                                                                          row_elems, norm);
  else
    key_norm_kernel<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<const float*>(k), rows,
                                                                         row_elems, norm);
  return check_launch("key norm");
}

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
