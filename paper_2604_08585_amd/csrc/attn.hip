// Step 6: location-aware sparse causal attention (Section 3.2 of the paper): the selected
// rows, given with their absolute positions, attend over the patched fused cache.
//
// bf16 / head_dim 128 path: flash-style online softmax on 32x32x16 MFMA.  A workgroup owns a
// block of consecutive selected rows times the G query heads of one KV head (128 "rows"), so
// every K/V tile is loaded once per KV head.  Logits are produced transposed (S^T = K Q^T):
// a lane then owns one row and the softmax statistics need no cross-lane traffic beyond one
// exchange between the two lane halves; the probabilities, still in registers, are already
// the B operand of O^T += V^T P^T.  V tiles are transposed on their way into LDS.  Key tiles
// wholly above a wave's highest position are skipped, tiles wholly below its lowest run
// unmasked, only the straddling tiles compare positions.  When the launch has too few row blocks
// to balance the causal triangle over the compute units, a row block's keys are cut into segments
// that run as separate workgroups; each writes a normalised partial output and its log-sum-exp,
// and a second kernel merges them (the usual softmax merge, exact up to rounding).
//
// Generic path (f32, or other shapes): one workgroup per (row, head), online softmax over
// 256-token tiles.
#include <type_traits>

#include "qcf_internal.h"

namespace qcf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int find_request(const int64_t* __restrict__ off, int B, int64_t row) {
  int b = 0;
  while (b < B && row >= off[b + 1]) ++b;
  return b;
}

struct AttnArgs {
  const void* q;
  const void* k;
  const void* v;
  const int32_t* sel_pos;
  const int64_t* sel_off;
  const int64_t* ctx_off;
  const int32_t* ctx_pos0;
  int64_t total_sel, total_ctx;
  int B, H, Hkv, G, D;
  void* o;
  float* lse;
  int n_row_blocks;      // upper bound on row blocks over all requests (MFMA path)
  int seg_tiles;         // key tiles per work unit; a row block with more tiles is split over units
  int n_seg_max;         // units per row block the grid provides
  bf16_t* part_o;        // [unit][128 rows][128] normalised partial outputs of split row blocks
  float* part_lse;       // [unit][128 rows] log2-domain log-sum-exp of each partial (-inf: no visible key)
  int32_t* units;        // units[0] = number of work units, then (row block << 8 | segment), longest first
  int32_t* blk_tiles;    // [row block] key tiles of the block, written by the plan kernel for the merge kernel
};

// ------------------------------------------------------------------ generic path

template <typename T>
__global__ __launch_bounds__(256) void attn_generic(AttnArgs a) {
  __shared__ float sq[128];
  __shared__ float sp[256];
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x / a.H;
  const int h = blockIdx.x - (int)row * a.H;
  const int b = find_request(a.sel_off, a.B, row);
  if (b >= a.B) return;
  const int64_t c0 = min(max(a.ctx_off[b], (int64_t)0), a.total_ctx);
  const int64_t c1 = min(max(a.ctx_off[b + 1], c0), a.total_ctx);
  const int Tn = (int)(c1 - c0);
  const int64_t p0 = a.ctx_pos0 ? a.ctx_pos0[b] : 0;
  const int n_vis = (int)min((int64_t)Tn, max((int64_t)0, (int64_t)a.sel_pos[row] - p0 + 1));
  const int g = h / a.G, D = a.D;
  const T* q = static_cast<const T*>(a.q) + (row * a.H + h) * D;
  const T* kb = static_cast<const T*>(a.k) + (c0 * a.Hkv + g) * D;
  const T* vb = static_cast<const T*>(a.v) + (c0 * a.Hkv + g) * D;
  const int64_t kv_stride = (int64_t)a.Hkv * D;
  if (tid < D) sq[tid] = Elem<T>::load(q + tid) * rsqrtf((float)D);
  __syncthreads();
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int j0 = 0; j0 < n_vis; j0 += 256) {
    const int j = j0 + tid;
    float s = -INFINITY;
    if (j < n_vis) {
      const T* kr = kb + j * kv_stride;
      float d = 0.f;
      for (int c = 0; c < D; ++c) d += sq[c] * Elem<T>::load(kr + c);
      s = d;
    }
    float mx = s;
    for (int d = 32; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float m_new = fmaxf(m_run, mx);          // finite: the tile has at least one visible token
    const float p = (j < n_vis) ? expf(s - m_new) : 0.f;
    sp[tid] = p;
    float sum = p;
    for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
    __syncthreads();
    if (lane == 0) red[wave] = sum;
    __syncthreads();
    sum = (red[0] + red[1]) + (red[2] + red[3]);
    const float alpha = expf(m_run - m_new);       // 0 on the first tile
    l_run = l_run * alpha + sum;
    if (tid < D) {
      acc *= alpha;
      const int n = min(256, n_vis - j0);
      for (int jj = 0; jj < n; ++jj) acc += sp[jj] * Elem<T>::load(vb + (j0 + jj) * kv_stride + tid);
    }
    m_run = m_new;
    __syncthreads();
  }
  if (tid < D) Elem<T>::store(static_cast<T*>(a.o) + (row * a.H + h) * D + tid, n_vis > 0 ? acc / l_run : 0.f);
  if (tid == 0 && a.lse) a.lse[row * a.H + h] = n_vis > 0 ? m_run + logf(l_run) : -INFINITY;
}

// ------------------------------------------------------------------ MFMA path (bf16, d = 128)

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

constexpr int kBKV = 64;                    // tokens per K/V tile
constexpr int kKTile = kBKV * 128;          // bf16 elements; rows are 256 B, no padding (swizzled instead)
constexpr int kVTile = kBKV * 128;
constexpr int kStage = kKTile + kVTile;
constexpr size_t kAttnLds = (size_t)2 * kStage * 2;
constexpr int kRowsPerWg = 128;             // (selected row, head-in-group) pairs per workgroup
constexpr float kLazyRescale = 8.f;         // log2 units the running maximum may lag behind the true one

// LDS transposing read: within each group of 16 lanes, lane i receives element i%4 of the four
// 8-byte rows addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4 of the group.
__device__ __forceinline__ shortx4 lds_read_tr(uint32_t lds_addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(uintptr_t)lds_addr);
}
// 16-byte LDS read at a byte address (a register plus a compile-time constant becomes the offset field)
__device__ __forceinline__ u32x4 lds_read16(uint32_t lds_addr) {
  return *(const u32x4 __attribute__((address_space(3)))*)(uintptr_t)lds_addr;
}

// Tile layouts in LDS (rows of 256 bytes = 16 chunks of 16 bytes, no padding):
//   keys:   chunk c of token row r sits in slot c ^ (r % 16), so the 16-byte reads of 16 consecutive
//           rows at one chunk index touch 16 different bank groups;
//   values: chunk c of row r sits in slot c ^ (4 * (r % 4)), so the 8-byte transposing reads of
//           8 consecutive rows x 64 bytes touch every bank exactly twice.
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(AttnArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_vis_max[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wave-uniform: keeps tile addresses in scalar registers
  const int hf = lane >> 5, l32 = lane & 31;
  const int BR = kRowsPerWg / a.G;           // selected rows per workgroup
  const uint32_t lds0 = lds_offset_of(smem);

  // consecutive workgroup ids land on different XCDs: give each XCD its own KV heads so that a
  // head's keys and values stay in one L2; later row blocks (longer key ranges) are scheduled first
  // Unsplit launches take the row blocks from the last (longest key range) to the first.  Split launches
  // read the unit list attn_plan_kernel sorted by length; segments are counted from the top of a block's
  // key range, so a block's remainder segment is the one at the start of the context.
  const int g = (int)(blockIdx.x % a.Hkv);
  const int unit = (int)(blockIdx.x / a.Hkv);
  int seg = 0, blk = a.n_row_blocks - 1 - unit;
  if (a.units) {
    if (unit >= a.units[0]) return;
    const int code = a.units[1 + unit];
    blk = code >> 8;
    seg = code & 255;
  }
  int wg = blk;
  int b = 0;
  int64_t s0 = 0, s1 = 0;
  for (; b < a.B; ++b) {
    s0 = min(max(a.sel_off[b], (int64_t)0), a.total_sel);
    s1 = min(max(a.sel_off[b + 1], s0), a.total_sel);
    const int nb = (int)((s1 - s0 + BR - 1) / BR);
    if (wg < nb) break;
    wg -= nb;
  }
  if (b >= a.B) return;
  const int64_t c0 = min(max(a.ctx_off[b], (int64_t)0), a.total_ctx);
  const int64_t c1 = min(max(a.ctx_off[b + 1], c0), a.total_ctx);
  const int T = (int)(c1 - c0);
  const int64_t p0 = a.ctx_pos0 ? a.ctx_pos0[b] : 0;

  // this lane's row
  const int r = wave * 32 + l32;
  const int64_t srow = s0 + (int64_t)wg * BR + r / a.G;
  const int head = g * a.G + r % a.G;
  const bool row_ok = srow < s1;
  int vis = 0;                                  // number of visible tokens of this row
  if (row_ok) vis = (int)min((int64_t)T, max((int64_t)0, (int64_t)a.sel_pos[srow] - p0 + 1));
  int wave_vis_max = vis, wave_vis_min = row_ok ? vis : 0x7fffffff;
#pragma unroll
  for (int d = 16; d >= 1; d >>= 1) {
    wave_vis_max = max(wave_vis_max, __shfl_xor(wave_vis_max, d, 64));
    wave_vis_min = min(wave_vis_min, __shfl_xor(wave_vis_min, d, 64));
  }
  if (lane == 0) s_vis_max[wave] = wave_vis_max;
  __syncthreads();
  const int wg_vis_max = max(max(s_vis_max[0], s_vis_max[1]), max(s_vis_max[2], s_vis_max[3]));
  const int n_tiles = (wg_vis_max + kBKV - 1) / kBKV;
  const bool split = n_tiles > a.seg_tiles;
  if (seg > 0 && seg * a.seg_tiles >= n_tiles) return;      // this block has fewer segments
  const int t_end = n_tiles - seg * a.seg_tiles;
  const int t_begin = max(0, t_end - a.seg_tiles);
  if (n_tiles == 0) {                 // nothing visible to any row of the block
    if (row_ok) {
      bf16_t* op = static_cast<bf16_t*>(a.o) + (srow * a.H + head) * 128 + 64 * hf;
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(op + 8 * i) = u32x4{0u, 0u, 0u, 0u};
      if (a.lse && hf == 0) a.lse[srow * a.H + head] = -INFINITY;
    }
    return;
  }

  // asynchronous tile loads: instruction i of wave w fills rows 16*i + 4*w .. +3 (1 KB); lane L
  // fills slot L%16 of row 16*i + 4*w + L/16 with the chunk the swizzle assigns to that slot.
  // Tokens past the end of the context are clamped (their probabilities are zero).
  const bf16_t* kg = static_cast<const bf16_t*>(a.k) + (c0 * a.Hkv + g) * 128;
  const bf16_t* vg = static_cast<const bf16_t*>(a.v) + (c0 * a.Hkv + g) * 128;
  const int ld_row = 4 * wave + (lane >> 4);                      // + 16*i
  const uint32_t row_bytes = (uint32_t)a.Hkv * 256u;              // one token row of the cache
  const uint32_t ld_kchunk = (uint32_t)(((lane & 15) ^ ld_row) * 16);           // row % 16 == ld_row
  const uint32_t ld_vchunk = (uint32_t)(((lane & 15) ^ (4 * (ld_row & 3))) * 16);
  const uint32_t ld_koff = (uint32_t)ld_row * row_bytes + ld_kchunk;
  const uint32_t ld_voff = (uint32_t)ld_row * row_bytes + ld_vchunk;
  auto aload = [&](const bf16_t* src, uint32_t off0, uint32_t chunk, int t, uint32_t dst) {
    const char* base = reinterpret_cast<const char*>(src) + (int64_t)t * kBKV * row_bytes;
    if (t * kBKV + kBKV <= T) {
#pragma unroll
      for (int i = 0; i < 4; ++i) load_to_lds_at(base + (size_t)(16 * i) * row_bytes, off0, dst + (16 * i) * 256);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = min(16 * i + ld_row, T - 1 - t * kBKV);
        load_to_lds_at(base, (uint32_t)row * row_bytes + chunk, dst + (16 * i) * 256);
      }
    }
  };
  auto aload_k = [&](int t, int st) { aload(kg, ld_koff, ld_kchunk, t, lds0 + st * kStage * 2 + (4 * wave) * 256); };
  auto aload_v = [&](int t, int st) {
    aload(vg, ld_voff, ld_vchunk, t, lds0 + st * kStage * 2 + kKTile * 2 + (4 * wave) * 256);
  };
  auto aload2 = [&](int t, int st) { aload_k(t, st); aload_v(t, st); };
  aload2(t_begin, 0);

  // stationary query fragments: qf[ks] = row r, elements 16*ks + 8*hf .. +7
  bf16x8 qf[8];
  {
    const bf16_t* qp = static_cast<const bf16_t*>(a.q) + ((row_ok ? srow : s0) * a.H + head) * 128 + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 t = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
      if (!row_ok) t = u32x4{0u, 0u, 0u, 0u};
      qf[ks] = __builtin_bit_cast(bf16x8, t);
    }
  }

  // per-lane byte offsets of the fragment reads inside a stage
  uint32_t kofs[8];     // key fragment ks: token row l32 (+32), chunk 2*ks + hf
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) kofs[ks] = lds0 + l32 * 256 + (((2 * ks + hf) ^ (l32 & 15)) * 16);
  // values: the lane addresses the 8-byte piece (token 4*hf + (lane%16)/4, elements d0 .. d0+3) where
  // block q = 4*((lane/16)%2) + lane%4 of a 32-element slice starts at d0 = 16*(q%2) + 4*(q/2); after the
  // transposing read lane (row i = lane%32) holds four consecutive tokens of element
  // 16*(i/4 % 2) + 4*(i/8) + i%4, which makes MFMA output row 8b + 4h + c element 16h + 4b + c
  uint32_t vofs[4];     // value fragment of output tile dt
  {
    const int vq = 4 * ((lane >> 4) & 1) + (lane & 3);
    const int d0 = 16 * (vq & 1) + 4 * (vq >> 1);
    const int vrow = 4 * hf + ((lane & 15) >> 2);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
      vofs[dt] = lds0 + kKTile * 2 + vrow * 256 + (((4 * dt + d0 / 8) ^ (4 * (vrow & 3))) * 16) + (d0 & 4) * 2;
  }

  floatx16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) oacc[i] = floatx16{0};
  float m_run = -INFINITY;      // running max of the scaled logits (log2 domain), shared by both lane halves
  float l_run = 0.f;            // this lane's share of the running denominator
  const float k2 = kLog2e * 0.08838834764831845f;

  auto process = [&](const uint32_t stage, int kv0) {        // stage: byte offset of the stage (a constant at each call)
    floatx16 sa = {0}, sb = {0};
    {
      u32x4 fa[2], fb[2];
      fa[0] = lds_read16(kofs[0] + stage);
      fb[0] = lds_read16(kofs[0] + (stage + 32 * 256));
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        if (ks < 7) {
          fa[(ks + 1) & 1] = lds_read16(kofs[ks + 1] + stage);
          fb[(ks + 1) & 1] = lds_read16(kofs[ks + 1] + (stage + 32 * 256));
        }
        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[ks & 1]), qf[ks], sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[ks & 1]), qf[ks], sb, 0, 0, 0);
      }
    }
    // first value fragments can travel while the softmax runs
    shortx4 vlo[2], vhi[2];
    vlo[0] = lds_read_tr(vofs[0] + stage);
    vhi[0] = lds_read_tr(vofs[0] + (stage + 8 * 256));
    // register v of sa is token kv0 + 8*(v/4) + 4*hf + v%4 (sb: + 32) against this lane's row
    float p[32];
#pragma unroll
    for (int v = 0; v < 16; ++v) { p[v] = sa[v]; p[16 + v] = sb[v]; }
    if (kv0 + kBKV > wave_vis_min) {
#pragma unroll
      for (int v = 0; v < 32; ++v) {
        const int j = kv0 + 32 * (v >> 4) + 8 * ((v & 15) >> 2) + 4 * hf + (v & 3);
        p[v] = (j < vis) ? p[v] : -INFINITY;
      }
    }
    float mx = p[0];
#pragma unroll
    for (int v = 1; v < 32; ++v) mx = fmaxf(mx, p[v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The reference point of the exponentials only moves when the maximum grows by more than 2^8: until
    // then probabilities up to 256 are accumulated against the old one (the final division by the
    // denominator makes the result independent of the reference point), and the running output is
    // rescaled far less often.
    const float m_cand = fmaxf(m_run, mx * k2);
    const bool bump = m_cand > m_run + kLazyRescale;          // also the first visible tile (m_run = -inf)
    const float m_new = bump ? m_cand : m_run;
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = bump ? __builtin_amdgcn_exp2f(m_run - m_use) : 1.f;
    float sum = 0.f;
#pragma unroll
    for (int v = 0; v < 32; ++v) {
      p[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(p[v], k2, -m_use));
      sum += p[v];
    }
    l_run = l_run * alpha + sum;
    m_run = m_new;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[i][v] *= alpha;
    }
    // P^T fragments: step s = 2*mt + t' uses registers 8*s .. 8*s+7 (tokens 16*s + 8*(e/4) + 4*hf + e%4)
    bf16x8 pf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const u32x4 pk = mk4(cvt_pk_bf16(p[8 * s + 0], p[8 * s + 1]), cvt_pk_bf16(p[8 * s + 2], p[8 * s + 3]),
                           cvt_pk_bf16(p[8 * s + 4], p[8 * s + 5]), cvt_pk_bf16(p[8 * s + 6], p[8 * s + 7]));
      pf[s] = __builtin_bit_cast(bf16x8, pk);
    }
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) {
      const int s = idx >> 2, dt = idx & 3;
      if (idx < 15) {
        const int s2 = (idx + 1) >> 2, dt2 = (idx + 1) & 3;
        vlo[(idx + 1) & 1] = lds_read_tr(vofs[dt2] + (stage + (16 * s2) * 256));
        vhi[(idx + 1) & 1] = lds_read_tr(vofs[dt2] + (stage + (16 * s2 + 8) * 256));
      }
      const shortx8 both = __builtin_shufflevector(vlo[idx & 1], vhi[idx & 1], 0, 1, 2, 3, 4, 5, 6, 7);
      oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[s], oacc[dt], 0, 0, 0);
    }
  };

  for (int t = t_begin; t < t_end; t += 2) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                                  // tile t has landed; stage 1 is free again
    if (t + 1 < t_end) aload2(t + 1, 1);
    if (t * kBKV < wave_vis_max) process(0u, t * kBKV);
    if (t + 1 >= t_end) break;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (t + 2 < t_end) aload2(t + 2, 0);
    if ((t + 1) * kBKV < wave_vis_max) process((uint32_t)kStage * 2u, (t + 1) * kBKV);
  }

  // epilogue: output register v of tile dt is element 32*dt + 16*hf + v of this lane's row
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (split) {                        // partial result of one key segment; merged by attn_merge_kernel
    const int64_t slot = ((int64_t)blk * a.Hkv + g) * a.n_seg_max + seg;
    bf16_t* op = a.part_o + (slot * kRowsPerWg + r) * 128 + 16 * hf;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
      for (int h8 = 0; h8 < 2; ++h8) {
        const u32x4 pk = mk4(cvt_pk_bf16(oacc[dt][8 * h8 + 0] * inv, oacc[dt][8 * h8 + 1] * inv),
                             cvt_pk_bf16(oacc[dt][8 * h8 + 2] * inv, oacc[dt][8 * h8 + 3] * inv),
                             cvt_pk_bf16(oacc[dt][8 * h8 + 4] * inv, oacc[dt][8 * h8 + 5] * inv),
                             cvt_pk_bf16(oacc[dt][8 * h8 + 6] * inv, oacc[dt][8 * h8 + 7] * inv));
        *reinterpret_cast<u32x4*>(op + 32 * dt + 8 * h8) = pk;
      }
    }
    if (hf == 0) a.part_lse[slot * kRowsPerWg + r] = l_tot > 0.f ? m_run + log2f(l_tot) : -INFINITY;
    return;
  }
  if (row_ok) {
    bf16_t* op = static_cast<bf16_t*>(a.o) + (srow * a.H + head) * 128 + 16 * hf;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
      for (int h8 = 0; h8 < 2; ++h8) {
        const u32x4 pk = mk4(cvt_pk_bf16(oacc[dt][8 * h8 + 0] * inv, oacc[dt][8 * h8 + 1] * inv),
                             cvt_pk_bf16(oacc[dt][8 * h8 + 2] * inv, oacc[dt][8 * h8 + 3] * inv),
                             cvt_pk_bf16(oacc[dt][8 * h8 + 4] * inv, oacc[dt][8 * h8 + 5] * inv),
                             cvt_pk_bf16(oacc[dt][8 * h8 + 6] * inv, oacc[dt][8 * h8 + 7] * inv));
        *reinterpret_cast<u32x4*>(op + 32 * dt + 8 * h8) = pk;
      }
    }
    if (a.lse && hf == 0)
      a.lse[srow * a.H + head] = l_tot > 0.f ? (m_run + log2f(l_tot)) * kLn2 : -INFINITY;
  }
}

// Work list of a split launch: one entry per (row block, key segment) that has tiles, bucket-sorted by
// length (longest first) so that the short remainders fill the tail of the schedule.  The order inside a
// bucket depends on the race for the slots; results do not, because every unit's output location is given
// by its (row block, segment).
constexpr int kPlanBins = 64;
constexpr int kPlanMaxBlocks = 4096;        // row blocks a split launch may have (LDS table of the plan kernel)
__global__ __launch_bounds__(1024) void attn_plan_kernel(AttnArgs a) {
  __shared__ int s_vis[kPlanMaxBlocks];     // largest visible length of each row block
  __shared__ int s_cnt[kPlanBins + 1];
  __shared__ int s_off[kPlanBins + 1];
  const int tid = threadIdx.x;
  const int BR = kRowsPerWg / a.G;
  for (int i = tid; i < a.n_row_blocks; i += 1024) s_vis[i] = 0;
  for (int i = tid; i <= kPlanBins; i += 1024) s_cnt[i] = 0;
  __syncthreads();
  // every selected row raises the visible length of its block
  for (int64_t sr = tid; sr < a.total_sel; sr += 1024) {
    int blk0 = 0, b = 0;
    int64_t s0 = 0, s1 = 0;
    for (; b < a.B; ++b) {
      s0 = min(max(a.sel_off[b], (int64_t)0), a.total_sel);
      s1 = min(max(a.sel_off[b + 1], s0), a.total_sel);
      if (sr >= s0 && sr < s1) break;
      blk0 += (int)((s1 - s0 + BR - 1) / BR);
    }
    if (b >= a.B) continue;
    const int64_t c0 = min(max(a.ctx_off[b], (int64_t)0), a.total_ctx);
    const int64_t c1 = min(max(a.ctx_off[b + 1], c0), a.total_ctx);
    const int64_t p0 = a.ctx_pos0 ? a.ctx_pos0[b] : 0;
    const int vis = (int)min(c1 - c0, max((int64_t)0, (int64_t)a.sel_pos[sr] - p0 + 1));
    atomicMax(&s_vis[blk0 + (int)((sr - s0) / BR)], vis);
  }
  __syncthreads();
  // pass 0 counts the units of every length bucket, pass 1 places them
  for (int pass = 0; pass < 2; ++pass) {
    for (int blk = tid; blk < a.n_row_blocks; blk += 1024) {
      const int n_tiles = (s_vis[blk] + kBKV - 1) / kBKV;
      if (pass == 0) a.blk_tiles[blk] = n_tiles;
      const int n_seg = max(1, (n_tiles + a.seg_tiles - 1) / a.seg_tiles);   // a block without tiles still writes zeros
      for (int sg = 0; sg < n_seg; ++sg) {
        const int len = min(a.seg_tiles, n_tiles - sg * a.seg_tiles);
        const int bin = kPlanBins - (int)((int64_t)max(len, 0) * kPlanBins / a.seg_tiles);   // 0: whole segments
        if (pass == 0) atomicAdd(&s_cnt[bin], 1);
        else a.units[1 + atomicAdd(&s_off[bin], 1)] = (blk << 8) | sg;
      }
    }
    __syncthreads();
    if (pass == 0) {
      if (tid == 0) {
        int run = 0;
        for (int i = 0; i <= kPlanBins; ++i) { s_off[i] = run; run += s_cnt[i]; }
        a.units[0] = run;
      }
      __syncthreads();
    }
  }
}

// Merge of the partial results of split row blocks: kMergeWgs workgroups per (row block, KV head), one
// thread per 8 output elements.  out = sum_s w_s O_s with w_s = 2^(lse_s - lse), lse = log2 sum_s 2^lse_s.
constexpr int kMergeWgs = kRowsPerWg * 16 / 256;
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
  const int tid = threadIdx.x;
  const int BR = kRowsPerWg / a.G;
  const int part = (int)(blockIdx.x % kMergeWgs);
  const int bh = (int)(blockIdx.x / kMergeWgs);
  const int g = bh % a.Hkv;
  const int blk = bh / a.Hkv;
  const int n_tiles = a.blk_tiles[blk];
  if (n_tiles <= a.seg_tiles) return;               // not split: the main kernel wrote the result
  int wg = blk, b = 0;
  int64_t s0 = 0, s1 = 0;
  for (; b < a.B; ++b) {
    s0 = min(max(a.sel_off[b], (int64_t)0), a.total_sel);
    s1 = min(max(a.sel_off[b + 1], s0), a.total_sel);
    const int nb = (int)((s1 - s0 + BR - 1) / BR);
    if (wg < nb) break;
    wg -= nb;
  }
  if (b >= a.B) return;
  const int n_seg = (n_tiles + a.seg_tiles - 1) / a.seg_tiles;
  const int r = part * 16 + (tid >> 4), ch = tid & 15;          // row of the block, 8-element chunk
  const int64_t srow = s0 + (int64_t)wg * BR + r / a.G;
  if (srow >= s1) return;
  const int head = g * a.G + r % a.G;
  // unit (blk, g, seg) wrote slot ((blk * Hkv + g) * n_seg_max + seg)
  const int64_t slot0 = ((int64_t)blk * a.Hkv + g) * a.n_seg_max;
  const float* pl = a.part_lse + slot0 * kRowsPerWg + r;
  const bf16_t* po = a.part_o + (slot0 * kRowsPerWg + r) * 128 + 8 * ch;
  // four segments at a time: every load first, then the running maximum, the weights and the weighted sum
  float mx = -INFINITY, wsum = 0.f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int sg0 = 0; sg0 < n_seg; sg0 += 4) {
    float l[4];
    u32x4 raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool ok = sg0 + u < n_seg;
      l[u] = ok ? pl[(int64_t)(sg0 + u) * kRowsPerWg] : -INFINITY;
      raw[u] = ok ? *reinterpret_cast<const u32x4*>(po + (int64_t)(sg0 + u) * kRowsPerWg * 128) : u32x4{0u, 0u, 0u, 0u};
    }
    float mn = mx;
#pragma unroll
    for (int u = 0; u < 4; ++u) mn = fmaxf(mn, l[u]);
    if (mn > -INFINITY) {
      const float resc = __builtin_amdgcn_exp2f(mx - mn);        // 0 while nothing was visible so far
      wsum *= resc;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] *= resc;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float w = __builtin_amdgcn_exp2f(l[u] - mn);        // 0 for a segment that saw nothing
        float f[8];
        Vec16<bf16_t>::unpack(raw[u], f);
        wsum += w;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += w * f[e];
      }
      mx = mn;
    }
  }
  const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] *= inv;
  *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(a.o) + (srow * a.H + head) * 128 + 8 * ch) = Vec16<bf16_t>::pack(acc);
  if (a.lse && ch == 0) a.lse[srow * a.H + head] = wsum > 0.f ? (mx + log2f(wsum)) * kLn2 : -INFINITY;
}

// Key tiles per work unit.  With enough row blocks the causal triangle balances by itself and blocks
// stay whole; otherwise a segment is about the average causal work of a resident workgroup.
struct Split { int seg_tiles, n_seg_max; };
Split choose_split(int64_t n_blocks, int64_t total_ctx) {
  const int slots = 2 * compute_unit_count();         // two workgroups are resident per compute unit
  const int64_t n_t = std::max<int64_t>(1, (total_ctx + kBKV - 1) / kBKV);
  const int64_t per_slot = n_blocks * ((n_t + 1) / 2) / slots;     // average causal work per resident workgroup
  // a little above that average (a multiple of 4 tiles): most resident workgroups then take one whole
  // segment and the remainders fill the rest (measured best at recompute ratios 0.05, 0.15 and 0.30)
  int64_t seg = std::max<int64_t>(8, (per_slot * 27 / 25 + 3) / 4 * 4);
  while ((n_t + seg - 1) / seg > 256) seg *= 2;       // a unit's segment number is kept in 8 bits
  if (n_blocks > kPlanMaxBlocks) seg = n_t;            // (never the case when splitting pays: see per_slot)
  if (seg >= n_t) return Split{(int)std::min<int64_t>(n_t, 0x3fffffff), 1};
  return Split{(int)seg, (int)((n_t + seg - 1) / seg)};
}

size_t part_o_bytes(int64_t n_blocks, int n_seg_max) {
  return align_up((size_t)n_blocks * n_seg_max * kRowsPerWg * 128 * sizeof(bf16_t), 256);
}
size_t part_lse_bytes(int64_t n_blocks, int n_seg_max) {
  return align_up((size_t)n_blocks * n_seg_max * kRowsPerWg * sizeof(float), 256);
}
size_t units_bytes(int64_t n_row_blocks, int n_seg_max) {
  return align_up((size_t)(n_row_blocks * n_seg_max + 1) * sizeof(int32_t), 256);
}
size_t blk_tiles_bytes(int64_t n_row_blocks) { return align_up((size_t)n_row_blocks * sizeof(int32_t), 256); }

bool use_mfma(const qcf_layer_desc& L) {
  const int G = L.n_q_heads / L.n_kv_heads;
  return L.dtype == QCF_DTYPE_BF16 && L.head_dim == 128 && G <= kRowsPerWg && kRowsPerWg % G == 0;
}

}  // namespace

size_t attn_workspace(const qcf_layer_desc& L, int32_t B, int64_t total_sel, int64_t total_ctx) {
  if (!use_mfma(L) || total_sel <= 0 || total_ctx <= 0) return 0;
  const int BR = kRowsPerWg / (L.n_q_heads / L.n_kv_heads);
  const int64_t n_blocks = ((total_sel + BR - 1) / BR + B) * L.n_kv_heads;
  const Split sp = choose_split(n_blocks, total_ctx);
  if (sp.n_seg_max <= 1) return 0;
  return part_o_bytes(n_blocks, sp.n_seg_max) + part_lse_bytes(n_blocks, sp.n_seg_max) +
         units_bytes(n_blocks / L.n_kv_heads, sp.n_seg_max) + blk_tiles_bytes(n_blocks / L.n_kv_heads);
}

qcf_status launch_attn(const qcf_layer_desc& L, int32_t B, const void* q, const int32_t* sel_pos,
                       const int64_t* sel_off, int64_t total_sel, const void* k, const void* v,
                       const int64_t* ctx_off, int64_t total_ctx, const int32_t* ctx_pos0, void* o,
                       float* lse, void* ws, hipStream_t st) {
  AttnArgs a;
  a.q = q; a.k = k; a.v = v;
  a.sel_pos = sel_pos; a.sel_off = sel_off; a.ctx_off = ctx_off; a.ctx_pos0 = ctx_pos0;
  a.total_sel = total_sel; a.total_ctx = total_ctx;
  a.B = B; a.H = L.n_q_heads; a.Hkv = L.n_kv_heads; a.G = L.n_q_heads / L.n_kv_heads; a.D = L.head_dim;
  a.o = o; a.lse = lse;
  a.n_row_blocks = 0;
  a.seg_tiles = 0x3fffffff; a.n_seg_max = 1; a.part_o = nullptr; a.part_lse = nullptr; a.units = nullptr; a.blk_tiles = nullptr;
  if (use_mfma(L)) {
    const int BR = kRowsPerWg / a.G;
    const int64_t nb = (total_sel + BR - 1) / BR + B;
    const Split sp = choose_split(nb * a.Hkv, total_ctx);
    if (nb * a.Hkv * std::max(sp.n_seg_max, kMergeWgs) > 0x7fffffff)
      return fail(QCF_ERR_UNSUPPORTED, "attn: grid too large");
    a.n_row_blocks = (int)nb;
    a.seg_tiles = sp.seg_tiles;
    a.n_seg_max = sp.n_seg_max;
    if (sp.n_seg_max > 1) {
      a.part_o = static_cast<bf16_t*>(ws);
      char* w = static_cast<char*>(ws);
      a.part_lse = reinterpret_cast<float*>(w + part_o_bytes(nb * a.Hkv, sp.n_seg_max));
      a.units = reinterpret_cast<int32_t*>(w + part_o_bytes(nb * a.Hkv, sp.n_seg_max) +
                                           part_lse_bytes(nb * a.Hkv, sp.n_seg_max));
      a.blk_tiles = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(a.units) + units_bytes(nb, sp.n_seg_max));
    }
    static std::atomic<uint64_t> lds_ok{0};
    QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&attn_mfma_kernel), kAttnLds, lds_ok));
    if (sp.n_seg_max > 1) {
      attn_plan_kernel<<<dim3(1), dim3(1024), 0, st>>>(a);
      QCF_TRY_LAUNCH("attn plan");
    }
    attn_mfma_kernel<<<dim3((unsigned)(nb * a.Hkv * sp.n_seg_max)), dim3(256), kAttnLds, st>>>(a);
    QCF_TRY_LAUNCH("attn");
    if (sp.n_seg_max > 1) {
      attn_merge_kernel<<<dim3((unsigned)(nb * a.Hkv * kMergeWgs)), dim3(256), 0, st>>>(a);
      return check_launch("attn merge");
    }
    return QCF_OK;
  }
  if (total_sel * a.H > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "attn: grid too large");
  const dim3 grid((unsigned)(total_sel * a.H)), block(256);
  if (L.dtype == QCF_DTYPE_BF16) attn_generic<bf16_t><<<grid, block, 0, st>>>(a);
  else attn_generic<float><<<grid, block, 0, st>>>(a);
  return check_launch("attn");
}

}  // namespace qcf
