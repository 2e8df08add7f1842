// Step 1: re-rotate chunk keys to their global positions and concatenate chunk K/V into
// the fused cache (location-independent chunk reuse, Section 3.2 of the paper).
//
// The shift of a chunk is constant, so only d/2 distinct (cos, sin) pairs exist per chunk.  Up to
// kMaxLdsChunks chunks: a single streaming kernel; every workgroup finds the chunks its rows belong to
// in an LDS copy of the chunk table and computes their (cos, sin) pairs itself (angles in float64), then
// every thread moves two 16-byte vectors of one key row (the two halves of its rotary pairs) and the
// matching two vectors of the value row.  Longer chunk tables: a small plan kernel writes the pairs and
// a block->chunk map to the workspace first.
#include "qcf_internal.h"

namespace qcf {
namespace {

constexpr int kThreads = 256;

struct RopeGeom {
  int D;            // head_dim
  int slots;        // work items per row = H_kv * (D/2) / vec
  int row_elems;    // H_kv * D
};

__global__ void rerope_plan_kernel(const qcf_chunk* __restrict__ chunks, int n_chunks, int D,
                                   double neg2_over_d_log2base, float2* __restrict__ cs,
                                   int* __restrict__ block_chunk, int n_blocks, int slots) {
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;
  const int half = D / 2;
  if (gid < n_chunks * half) {
    const int c = gid / half, i = gid - c * half;
    const double theta = exp2(neg2_over_d_log2base * (double)i);
    const double phi = (double)(chunks[c].dst_pos0 - chunks[c].src_pos0) * theta;
    double sn, cn;
    sincos(phi, &sn, &cn);
    cs[gid] = make_float2((float)cn, (float)sn);
  }
  if (gid < n_blocks) {
    // last chunk whose first row is <= the block's first row (0 if none)
    const int64_t row = ((int64_t)gid * kThreads) / slots;
    int lo = 0, hi = n_chunks - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (chunks[mid].dst_row <= row) lo = mid; else hi = mid - 1;
    }
    block_chunk[gid] = lo;
  }
}

// ---- single-kernel path ------------------------------------------------------------------------
constexpr int kMaxLdsChunks = 256;      // chunk table entries kept in LDS
constexpr int kMaxWgPairs = 1024;       // (cos, sin) pairs a workgroup keeps: chunks its rows touch x d/2

template <typename T, int STYLE>
__global__ __launch_bounds__(kThreads) void rerope_fused_kernel(
    const qcf_chunk* __restrict__ chunks, int n_chunks, double neg2_over_d_log2base, int64_t total_items,
    int64_t total_rows, RopeGeom g, T* __restrict__ kf, T* __restrict__ vf) {
  constexpr int VEC = Elem<T>::kVec;
  __shared__ int64_t s_row[kMaxLdsChunks];
  __shared__ int s_len[kMaxLdsChunks];
  __shared__ float2 s_cs[kMaxWgPairs];
  __shared__ int s_first;
  const int tid = threadIdx.x;
  const int half = g.D / 2;
  for (int c = tid; c < n_chunks; c += kThreads) { s_row[c] = chunks[c].dst_row; s_len[c] = chunks[c].len; }
  __syncthreads();
  // rows of this workgroup; last chunk whose first row is <= the workgroup's first row (0 if none)
  const int64_t item0 = (int64_t)blockIdx.x * kThreads;
  const int64_t r_first = item0 / g.slots;
  const int64_t r_last = min(total_rows - 1, (item0 + kThreads - 1) / g.slots);
  if (tid == 0) {
    int lo = 0, hi = n_chunks - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (s_row[mid] <= r_first) lo = mid; else hi = mid - 1;
    }
    s_first = lo;
  }
  __syncthreads();
  const int c_first = s_first;
  int c_last = c_first;                                  // last chunk that starts at or before the last row
  while (c_last + 1 < n_chunks && s_row[c_last + 1] <= r_last) ++c_last;
  const int n_mine = min(c_last - c_first + 1, kMaxWgPairs / half);   // (the launcher keeps this from truncating)
  for (int e = tid; e < n_mine * half; e += kThreads) {
    const int c = c_first + e / half, i = e % half;
    const double theta = exp2(neg2_over_d_log2base * (double)i);
    double sn, cn;
    sincos((double)(chunks[c].dst_pos0 - chunks[c].src_pos0) * theta, &sn, &cn);
    s_cs[e] = make_float2((float)cn, (float)sn);
  }
  __syncthreads();

  const int64_t item = item0 + tid;
  if (item >= total_items) return;
  const int64_t r = item / g.slots;
  const int s = (int)(item - r * g.slots);
  int ci = c_first;
  while (ci < c_last && r >= s_row[ci] + s_len[ci]) ++ci;
  const int64_t c_row = s_row[ci];
  if (r < c_row || r >= c_row + s_len[ci] || r >= total_rows || ci - c_first >= n_mine) return;   // not covered by a chunk
  const int64_t t = r - c_row;
  const int slots_per_head = half / VEC;
  const int head = s / slots_per_head;
  const int i0 = (s - head * slots_per_head) * VEC;                  // first rotary pair of this item
  int e0, e1;
  if (STYLE == 0) { e0 = head * g.D + i0;     e1 = e0 + half; }
  else            { e0 = head * g.D + 2 * i0; e1 = e0 + VEC; }

  const T* ksrc = static_cast<const T*>(chunks[ci].k_src) + t * g.row_elems;
  const u32x4 ra = *reinterpret_cast<const u32x4*>(ksrc + e0);
  const u32x4 rb = *reinterpret_cast<const u32x4*>(ksrc + e1);
  u32x4 va, vb;
  if (vf) {
    const T* vsrc = static_cast<const T*>(chunks[ci].v_src) + t * g.row_elems;
    va = *reinterpret_cast<const u32x4*>(vsrc + e0);
    vb = *reinterpret_cast<const u32x4*>(vsrc + e1);
  }
  float f[2 * VEC], o[2 * VEC];
  Vec16<T>::unpack(ra, f);
  Vec16<T>::unpack(rb, f + VEC);
  const float2* my = s_cs + (ci - c_first) * half + i0;
#pragma unroll
  for (int p = 0; p < VEC; ++p) {
    const float2 w = my[p];
    const int ia = (STYLE == 0) ? p : 2 * p;
    const int ib = (STYLE == 0) ? p + VEC : 2 * p + 1;
    o[ia] = f[ia] * w.x - f[ib] * w.y;
    o[ib] = f[ib] * w.x + f[ia] * w.y;
  }
  T* kdst = kf + r * g.row_elems;
  *reinterpret_cast<u32x4*>(kdst + e0) = Vec16<T>::pack(o);
  *reinterpret_cast<u32x4*>(kdst + e1) = Vec16<T>::pack(o + VEC);
  if (vf) {
    T* vdst = vf + r * g.row_elems;
    *reinterpret_cast<u32x4*>(vdst + e0) = va;
    *reinterpret_cast<u32x4*>(vdst + e1) = vb;
  }
}

// ---- two-kernel path (long chunk tables) ---------------------------------------------------------
template <typename T, int STYLE>
__global__ __launch_bounds__(kThreads) void rerope_main_kernel(
    const qcf_chunk* __restrict__ chunks, int n_chunks, const float2* __restrict__ cs,
    const int* __restrict__ block_chunk, int64_t total_items, int64_t total_rows, RopeGeom g,
    T* __restrict__ kf, T* __restrict__ vf) {
  constexpr int VEC = Elem<T>::kVec;
  const int64_t item = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (item >= total_items) return;
  const int64_t r = item / g.slots;
  const int s = (int)(item - r * g.slots);
  int ci = block_chunk[blockIdx.x];
  int64_t c_row = chunks[ci].dst_row;
  int c_len = chunks[ci].len;
  while (r >= c_row + c_len && ci + 1 < n_chunks) {
    ++ci;
    c_row = chunks[ci].dst_row;
    c_len = chunks[ci].len;
  }
  if (r < c_row || r >= c_row + c_len || r >= total_rows) return;   // row not covered by a chunk
  const int64_t t = r - c_row;
  const int slots_per_head = (g.D / 2) / VEC;
  const int head = s / slots_per_head;
  const int i0 = (s - head * slots_per_head) * VEC;                  // first rotary pair of this item
  int e0, e1;
  if (STYLE == 0) { e0 = head * g.D + i0;     e1 = e0 + g.D / 2; }
  else            { e0 = head * g.D + 2 * i0; e1 = e0 + VEC; }

  const T* ksrc = static_cast<const T*>(chunks[ci].k_src) + t * g.row_elems;
  const u32x4 ra = *reinterpret_cast<const u32x4*>(ksrc + e0);
  const u32x4 rb = *reinterpret_cast<const u32x4*>(ksrc + e1);
  u32x4 va, vb;
  const T* vsrc = nullptr;
  if (vf) {
    vsrc = static_cast<const T*>(chunks[ci].v_src) + t * g.row_elems;
    va = *reinterpret_cast<const u32x4*>(vsrc + e0);
    vb = *reinterpret_cast<const u32x4*>(vsrc + e1);
  }
  float f[2 * VEC], o[2 * VEC];
  Vec16<T>::unpack(ra, f);
  Vec16<T>::unpack(rb, f + VEC);
  const float2* my = cs + (int64_t)ci * (g.D / 2) + i0;
#pragma unroll
  for (int p = 0; p < VEC; ++p) {
    const float2 w = my[p];
    const int ia = (STYLE == 0) ? p : 2 * p;
    const int ib = (STYLE == 0) ? p + VEC : 2 * p + 1;
    o[ia] = f[ia] * w.x - f[ib] * w.y;
    o[ib] = f[ib] * w.x + f[ia] * w.y;
  }
  T* kdst = kf + r * g.row_elems;
  *reinterpret_cast<u32x4*>(kdst + e0) = Vec16<T>::pack(o);
  *reinterpret_cast<u32x4*>(kdst + e1) = Vec16<T>::pack(o + VEC);
  if (vf) {
    T* vdst = vf + r * g.row_elems;
    *reinterpret_cast<u32x4*>(vdst + e0) = va;
    *reinterpret_cast<u32x4*>(vdst + e1) = vb;
  }
}

RopeGeom geom(const qcf_layer_desc& L) {
  RopeGeom g;
  const int vec = 16 / elem_size(L.dtype);
  g.D = L.head_dim;
  g.slots = L.n_kv_heads * (L.head_dim / 2) / vec;
  g.row_elems = L.n_kv_heads * L.head_dim;
  return g;
}

int64_t n_blocks_for(const RopeGeom& g, int64_t total_rows) {
  return (total_rows * g.slots + kThreads - 1) / kThreads;
}

}  // namespace

size_t rerope_workspace(const qcf_layer_desc& L, int32_t n_chunks, int64_t total_rows) {
  const RopeGeom g = geom(L);
  size_t cs_bytes = align_up((size_t)n_chunks * (L.head_dim / 2) * sizeof(float2), 256);
  size_t map_bytes = align_up((size_t)n_blocks_for(g, total_rows) * sizeof(int), 256);
  return cs_bytes + map_bytes;
}

qcf_status launch_rerope(const qcf_layer_desc& L, const qcf_chunk* chunks, int32_t n_chunks,
                         int64_t total_rows, void* kf, void* vf, void* ws, hipStream_t st) {
  const RopeGeom g = geom(L);
  const int64_t n_blocks = n_blocks_for(g, total_rows);
  if (n_blocks > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "rerope: too many rows");
  const double c = -2.0 / (double)L.head_dim * std::log2(L.rope_base);
  const int64_t items = total_rows * g.slots;
  const dim3 grid((unsigned)n_blocks), block(kThreads);
  // a workgroup covers at most ceil(256 / slots) + 1 rows, hence at most that many chunks
  const int64_t wg_chunks = (kThreads + g.slots - 1) / g.slots + 1;
  if (n_chunks <= kMaxLdsChunks && wg_chunks * (L.head_dim / 2) <= kMaxWgPairs) {
#define QCF_RF(T, S)                                                                                  \
  rerope_fused_kernel<T, S><<<grid, block, 0, st>>>(chunks, n_chunks, c, items, total_rows, g,        \
                                                    static_cast<T*>(kf), static_cast<T*>(vf))
    if (L.dtype == QCF_DTYPE_BF16) {
      if (L.rope_style == 0) QCF_RF(bf16_t, 0); else QCF_RF(bf16_t, 1);
    } else {
      if (L.rope_style == 0) QCF_RF(float, 0); else QCF_RF(float, 1);
    }
#undef QCF_RF
    return check_launch("rerope");
  }
  float2* cs = static_cast<float2*>(ws);
  int* block_chunk = reinterpret_cast<int*>(static_cast<char*>(ws) +
                                            align_up((size_t)n_chunks * (L.head_dim / 2) * sizeof(float2), 256));
  const int64_t plan_threads = std::max<int64_t>((int64_t)n_chunks * (L.head_dim / 2), n_blocks);
  rerope_plan_kernel<<<dim3((unsigned)((plan_threads + 255) / 256)), dim3(256), 0, st>>>(
      chunks, n_chunks, L.head_dim, c, cs, block_chunk, (int)n_blocks, g.slots);
  QCF_TRY_LAUNCH("rerope plan");
#define QCF_RR(T, S)                                                                          \
  rerope_main_kernel<T, S><<<grid, block, 0, st>>>(chunks, n_chunks, cs, block_chunk, items,  \
                                                   total_rows, g, static_cast<T*>(kf), static_cast<T*>(vf))
  if (L.dtype == QCF_DTYPE_BF16) {
    if (L.rope_style == 0) QCF_RR(bf16_t, 0); else QCF_RR(bf16_t, 1);
  } else {
    if (L.rope_style == 0) QCF_RR(float, 0); else QCF_RR(float, 1);
  }
#undef QCF_RR
  return check_launch("rerope main");
}

}  // namespace qcf
