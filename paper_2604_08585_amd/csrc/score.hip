// Step 2: critical-layer attention analysis (Section 3.1 Phase 3; Section 3.2 token
// selector of the paper): score[j] = mean over probe rows and heads of the softmax
// attention the context token j receives.
//
// bf16 / head_dim 128 path (the dense contraction runs on MFMA):
//   pass 1  per (256-token tile, KV head, block of 128 group rows): logits of the block's probe rows
//           against the tile (a wave keeps 64 tokens) -> per-row (max, sum-exp) partials of the tile,
//           in the log2 domain;
//   pass 2  every workgroup first folds the partials of its group's rows over the request's tiles into
//           a log2-sum-exp per row (in a fixed order, so all workgroups get the same value); logits
//           again, p = exp2(logit - lse), summed over the rows of the group -> per-KV-head column sums;
//   reduce  fixed-order sum over KV heads, times 1/(R*H).
// No floating-point atomics anywhere, so scores (and the indices selected from them) are
// bit-stable from run to run.
//
// Generic path (f32, or head_dim 64): one workgroup per (probe row, head) materialises its
// softmax row in the workspace, then a column mean.
#include "qcf_internal.h"

namespace qcf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;

// request owning global row `row` given offsets[0..B]; returns B if none
__device__ __forceinline__ int find_request(const int64_t* __restrict__ off, int B, int64_t row) {
  int b = 0;
  while (b < B && row >= off[b + 1]) ++b;
  return b;
}

// ------------------------------------------------------------------ generic path

template <typename T>
__global__ __launch_bounds__(256) void score_rows_generic(
    const T* __restrict__ q, const int64_t* __restrict__ probe_off, int64_t total_probe,
    const T* __restrict__ k, const int64_t* __restrict__ ctx_off, int64_t total_ctx, int B,
    const int32_t* __restrict__ probe_limit, int H, int Hkv, int D, float* __restrict__ P) {
  __shared__ float sq[128];
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x / H;
  const int h = blockIdx.x - (int)row * H;
  const int b = find_request(probe_off, B, row);
  if (b >= B) return;
  int64_t c0 = min(max(ctx_off[b], (int64_t)0), total_ctx);
  int64_t c1 = min(max(ctx_off[b + 1], c0), total_ctx);
  const int Tn = (int)(c1 - c0);
  int limit = Tn;
  if (probe_limit) limit = min(Tn, max(0, probe_limit[row]));
  float* prow = P + ((int64_t)row * H + h) * total_ctx + c0;
  const int g = h / (H / Hkv);
  if (tid < D) sq[tid] = Elem<T>::load(q + ((int64_t)row * H + h) * D + tid);
  __syncthreads();
  const float scale = rsqrtf((float)D);
  float mx = -INFINITY;
  for (int j = tid; j < limit; j += 256) {
    const T* kr = k + ((c0 + j) * Hkv + g) * (int64_t)D;
    float acc = 0.f;
    for (int c = 0; c < D; ++c) acc += sq[c] * Elem<T>::load(kr + c);
    acc *= scale;
    prow[j] = acc;
    mx = fmaxf(mx, acc);
  }
  for (int d = 32; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int j = tid; j < limit; j += 256) {
    const float e = expf(prow[j] - mx);
    prow[j] = e;
    sum += e;
  }
  for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  sum = (red[0] + red[1]) + (red[2] + red[3]);
  for (int j = tid; j < Tn; j += 256) prow[j] = (j < limit) ? prow[j] / sum : 0.f;
}

__global__ __launch_bounds__(256) void score_colmean_generic(
    const float* __restrict__ P, const int64_t* __restrict__ probe_off, int64_t total_probe,
    const int64_t* __restrict__ ctx_off, int64_t total_ctx, int B, int H, float* __restrict__ score) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= total_ctx) return;
  const int b = find_request(ctx_off, B, j);
  if (b >= B) return;
  const int64_t r0 = min(max(probe_off[b], (int64_t)0), total_probe);
  const int64_t r1 = min(max(probe_off[b + 1], r0), total_probe);
  float acc = 0.f;
  for (int64_t r = r0 * H; r < r1 * H; ++r) acc += P[r * total_ctx + j];
  score[j] = (r1 > r0) ? acc / (float)((r1 - r0) * H) : 0.f;
}

// ------------------------------------------------------------------ MFMA path (bf16, d = 128)

constexpr int kTokPerWave = 64;                 // tokens a wave keeps stationary in registers
constexpr int kWavesPerWg = 4;
constexpr int kTokPerWg = kTokPerWave * kWavesPerWg;
constexpr int kRowBlock = 320;                  // probe rows (of one group) staged in LDS at a time
constexpr int kRowSplit1 = 128;                 // pass 1 only: group rows per workgroup (grid.z); its partials are
                                                // per row, so splitting the rows costs nothing downstream and puts
                                                // several workgroups on a compute unit
constexpr int kQStride = 128;                   // bf16 elements per staged row (swizzled, no padding)

struct ScoreArgs {
  const bf16_t* q;            // [total_probe, H, 128]
  const bf16_t* k;            // [total_ctx, Hkv, 128]
  const int64_t* probe_off;
  const int64_t* ctx_off;
  const int32_t* probe_limit;
  int64_t total_probe, total_ctx;
  int B, H, Hkv, G;
  float2* part;               // [n_tiles][total_probe * H] (max2, sumexp2) per 256-token tile
  float* colsum;              // [Hkv][total_ctx]
  float* score;
};

// Maps a workgroup index (= tile number over all requests) to (request, first token of its 256-token
// tile, number of the request's first tile).  Tiles are aligned to the start of each request.  Returns
// false when the index is past the last tile.
__device__ __forceinline__ bool locate_tile(const ScoreArgs& a, int wg, int& b, int64_t& c0, int& T,
                                            int& tile_tok0, int& tile_first) {
  tile_first = 0;
  for (b = 0; b < a.B; ++b) {
    c0 = min(max(a.ctx_off[b], (int64_t)0), a.total_ctx);
    const int64_t c1 = min(max(a.ctx_off[b + 1], c0), a.total_ctx);
    T = (int)(c1 - c0);
    const int nt = (T + kTokPerWg - 1) / kTokPerWg;
    if (wg < nt) {
      tile_tok0 = wg * kTokPerWg;
      return true;
    }
    wg -= nt;
    tile_first += nt;
  }
  return false;
}

// Loads the wave's 64 key rows (tokens tok0 .. tok0+63 of KV head g) as MFMA operand
// fragments: kf[mt][ks] holds, for lane l, token mt*32 + l%32, elements 16*ks + 8*(l/32) .. +7.
__device__ __forceinline__ void load_k_frags(const ScoreArgs& a, int64_t c0, int T, int tok0, int g,
                                             int lane, bf16x8 kf[2][8]) {
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    const int tok = tok0 + mt * 32 + (lane & 31);
    const bool ok = tok < T;
    const bf16_t* src = a.k + ((c0 + (ok ? tok : 0)) * a.Hkv + g) * 128 + 8 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 r = u32x4{0u, 0u, 0u, 0u};
      if (ok) r = *reinterpret_cast<const u32x4*>(src + 16 * ks);
      kf[mt][ks] = __builtin_bit_cast(bf16x8, r);
    }
  }
}

// Stages probe rows [r_begin, r_begin + n_rows) of group g (row r = i*G + hh <-> probe row i,
// head g*G + hh) into LDS with asynchronous direct-to-LDS loads; the caller waits and synchronises.
// Staged rows are 256 bytes (16 chunks of 16 bytes) without padding; chunk c of row r sits in slot
// c ^ (r % 16), so the 16-byte fragment reads of 16 consecutive rows touch 16 different bank groups.
// Rows up to the next multiple of 32 are filled with a copy of the last row (never used in a result).
__device__ __forceinline__ void stage_q_async(const ScoreArgs& a, int64_t p0, int g, int r_begin, int n_rows,
                                              int n_rows_pad, unsigned char* sQ, int wave, int lane) {
  for (int j = wave; j < n_rows_pad / 4; j += kWavesPerWg) {       // one 1 KB instruction = 4 rows
    const int r = 4 * j + (lane >> 4);
    const int rr = r_begin + min(r, n_rows - 1);
    const int i = rr / a.G, hh = rr - i * a.G;
    const int chunk = (lane & 15) ^ (r & 15);
    load_to_lds_addr(a.q + ((p0 + i) * a.H + g * a.G + hh) * 128 + chunk * 8, sQ + j * 1024);
  }
}

template <bool LIMIT>
__global__ __launch_bounds__(256) void score_pass1(ScoreArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float2* sPart = reinterpret_cast<float2*>(smem + (size_t)kRowSplit1 * kQStride * 2);   // [4 waves][kRowSplit1]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = blockIdx.y;
  int b, T, tile_tok0, tile_first;
  int64_t c0;
  if (!locate_tile(a, blockIdx.x, b, c0, T, tile_tok0, tile_first)) return;
  const int64_t p0 = min(max(a.probe_off[b], (int64_t)0), a.total_probe);
  const int64_t p1 = min(max(a.probe_off[b + 1], p0), a.total_probe);
  const int rows = (int)(p1 - p0) * a.G;         // probe rows x heads of the group
  const int r_begin = (int)blockIdx.z * kRowSplit1;
  if (r_begin >= rows) return;
  const int n_rows = min(rows - r_begin, kRowSplit1);
  const int n_pad = (n_rows + 31) & ~31;
  const int tok0 = tile_tok0 + wave * kTokPerWave;
  const bool wave_active = tok0 < T;
  const float k2 = kLog2e * 0.08838834764831845f;   // log2(e) / sqrt(128)
  // byte offset of this lane's fragment (row lane%32, chunk 2*ks + lane/32) is qb0 ^ (32 * ks)
  const int qb0 = (lane & 31) * 256 + (((lane >> 5) ^ (lane & 15)) * 16);

  bf16x8 kf[2][8];
  load_k_frags(a, c0, T, tok0, g, lane, kf);
  stage_q_async(a, p0, g, r_begin, n_rows, n_pad, smem, wave, lane);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  for (int rt = 0; rt < n_pad; rt += 32) {
    float mx = -INFINITY, sum = 0.f;
    if (wave_active) {
      floatx16 acc0 = {0}, acc1 = {0};
      const unsigned char* qrow = smem + rt * 256;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 qf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + (qb0 ^ (32 * ks))));
        // S^T tile: rows = tokens (A = keys), columns = probe rows (B = queries)
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][ks], qf, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][ks], qf, acc1, 0, 0, 0);
      }
      // lane owns probe row rt + lane%32; its registers hold tokens 8*(v/4) + 4*(lane/32) + v%4
      const int r = r_begin + rt + (lane & 31);
      int lim = T;
      if (LIMIT && r < rows) lim = min(T, max(0, a.probe_limit[p0 + r / a.G]));
      float s[32];
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[v] = acc0[v]; s[16 + v] = acc1[v]; }
      if (LIMIT || tok0 + kTokPerWave > T) {        // wave-uniform: only ragged or limited tiles compare
#pragma unroll
        for (int v = 0; v < 32; ++v) {
          const int t0 = tok0 + 32 * (v >> 4) + 8 * ((v & 15) >> 2) + 4 * (lane >> 5) + (v & 3);
          s[v] = (t0 < lim) ? s[v] : -INFINITY;
        }
      }
      mx = s[0];
#pragma unroll
      for (int v = 1; v < 32; ++v) mx = fmaxf(mx, s[v]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * k2;          // k2 > 0: scaling commutes with the maximum
      const float m_use = (mx == -INFINITY) ? 0.f : mx;
#pragma unroll
      for (int v = 0; v < 32; ++v) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[v], k2, -m_use));
      sum += __shfl_xor(sum, 32, 64);
    }
    if (lane < 32) sPart[wave * kRowSplit1 + rt + lane] = make_float2(mx, sum);
  }
  __syncthreads();
  // the four waves' 64-token partials of a row fold, in wave order, into the tile's partial
  float2* part = a.part + (int64_t)blockIdx.x * (a.total_probe * a.H);
  for (int r = tid; r < n_rows; r += 256) {
    float2 p[kWavesPerWg];
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWavesPerWg; ++w) { p[w] = sPart[w * kRowSplit1 + r]; m = fmaxf(m, p[w].x); }
    float z = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerWg; ++w)
      if (p[w].x > -INFINITY) z += p[w].y * exp2f(p[w].x - m);
    const int rr = r_begin + r;
    const int i = rr / a.G, hh = rr - i * a.G;
    part[(p0 + i) * a.H + g * a.G + hh] = make_float2(m, z);
  }
}

// Folds a batch of (max2, sumexp2) partials, in order, into the running pair (m, z).  A partial that saw
// nothing is (-inf, 0) and contributes 0 * exp2(-inf) = 0.
constexpr int kFoldBatch = 32;
__device__ __forceinline__ void fold_partials(const float2 (&p)[kFoldBatch], float& m, float& z) {
  float mn = m;
#pragma unroll
  for (int u = 0; u < kFoldBatch; ++u) mn = fmaxf(mn, p[u].x);
  if (mn > -INFINITY) {
    z *= __builtin_amdgcn_exp2f(m - mn);
#pragma unroll
    for (int u = 0; u < kFoldBatch; ++u) z = __builtin_fmaf(p[u].y, __builtin_amdgcn_exp2f(p[u].x - mn), z);
    m = mn;
  }
}

template <bool LIMIT>
__global__ __launch_bounds__(256) void score_pass2(ScoreArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* sL = reinterpret_cast<float*>(smem + (size_t)kRowBlock * kQStride * 2);   // [kRowBlock] lse2
  int* sLim = reinterpret_cast<int*>(sL + kRowBlock);                                // [kRowBlock]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = blockIdx.y;
  int b, T, tile_tok0, tile_first;
  int64_t c0;
  if (!locate_tile(a, blockIdx.x, b, c0, T, tile_tok0, tile_first)) return;
  const int64_t p0 = min(max(a.probe_off[b], (int64_t)0), a.total_probe);
  const int64_t p1 = min(max(a.probe_off[b + 1], p0), a.total_probe);
  const int rows = (int)(p1 - p0) * a.G;
  const int n_tiles = (T + kTokPerWg - 1) / kTokPerWg;
  const int64_t part_stride = a.total_probe * a.H;
  const int tok0 = tile_tok0 + wave * kTokPerWave;
  const bool wave_active = tok0 < T;
  const float k2 = kLog2e * 0.08838834764831845f;
  const int qb0 = (lane & 31) * 256 + (((lane >> 5) ^ (lane & 15)) * 16);

  bf16x8 kf[2][8];
  load_k_frags(a, c0, T, tok0, g, lane, kf);
  float col0 = 0.f, col1 = 0.f;        // column sums of tokens tok0 + lane%32 and + 32

  for (int r_begin = 0; r_begin < rows; r_begin += kRowBlock) {
    const int n_rows = min(kRowBlock, rows - r_begin);
    const int n_pad = (n_rows + 31) & ~31;
    __syncthreads();
    stage_q_async(a, p0, g, r_begin, n_rows, n_pad, smem, wave, lane);
    // log2-sum-exp of every staged row over the request: the tiles' partials folded in tile order,
    // kFoldBatch at a time (all loads of a thread's two rows first, then per row one maximum and one
    // rescaled sum); every workgroup of the request computes the same values
    {
      static_assert(kRowBlock <= 512, "a thread folds at most two staged rows");
      const int ra = tid, rb = tid + 256;
      const bool has_a = ra < n_rows, has_b = rb < n_rows;
      const float2* ppa = nullptr;
      const float2* ppb = nullptr;
      int lim_a = 0, lim_b = 0;
      if (has_a) {
        const int rr = r_begin + ra, i = rr / a.G, hh = rr - i * a.G;
        ppa = a.part + (int64_t)tile_first * part_stride + (p0 + i) * a.H + g * a.G + hh;
        lim_a = LIMIT ? min(T, max(0, a.probe_limit[p0 + i])) : T;
      }
      if (has_b) {
        const int rr = r_begin + rb, i = rr / a.G, hh = rr - i * a.G;
        ppb = a.part + (int64_t)tile_first * part_stride + (p0 + i) * a.H + g * a.G + hh;
        lim_b = LIMIT ? min(T, max(0, a.probe_limit[p0 + i])) : T;
      }
      float ma = -INFINITY, za = 0.f, mb = -INFINITY, zb = 0.f;
      for (int t0 = 0; t0 < n_tiles; t0 += kFoldBatch) {
        float2 pa[kFoldBatch], pb[kFoldBatch];
        if (has_a) {
#pragma unroll
          for (int u = 0; u < kFoldBatch; ++u) {
            pa[u] = (t0 + u < n_tiles) ? *ppa : make_float2(-INFINITY, 0.f);
            ppa += part_stride;               // (stays inside the workspace: n_tiles <= the tiles allocated)
          }
        }
        if (has_b) {
#pragma unroll
          for (int u = 0; u < kFoldBatch; ++u) {
            pb[u] = (t0 + u < n_tiles) ? *ppb : make_float2(-INFINITY, 0.f);
            ppb += part_stride;
          }
          fold_partials(pb, mb, zb);
        }
        if (has_a) fold_partials(pa, ma, za);
      }
      // rows that see nothing get +inf so that exp2(logit - lse) is 0
      if (ra < n_pad) {
        sL[ra] = (za > 0.f) ? ma + log2f(za) : INFINITY;
        sLim[ra] = lim_a;
      }
      if (rb < n_pad) {
        sL[rb] = (zb > 0.f) ? mb + log2f(zb) : INFINITY;
        sLim[rb] = lim_b;
      }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (!wave_active) continue;
    for (int rt = 0; rt < n_pad; rt += 32) {
      floatx16 acc0 = {0}, acc1 = {0};
      const unsigned char* qrow = smem + rt * 256;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 qf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + (qb0 ^ (32 * ks))));
        // S tile: rows = probe rows (A = queries), columns = tokens (B = keys)
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[0][ks], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[1][ks], acc1, 0, 0, 0);
      }
      // lane owns tokens tok0 + lane%32 (acc0) and + 32 (acc1); register v is probe row
      // rt + 8*(v/4) + 4*(lane/32) + v%4
      const int tA = tok0 + (lane & 31), tB = tA + 32;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int rbase = rt + 8 * q4 + 4 * (lane >> 5);
        const float4 l4 = *reinterpret_cast<const float4*>(sL + rbase);
        const float ls[4] = {l4.x, l4.y, l4.z, l4.w};
        int lims[4] = {T, T, T, T};
        if (LIMIT) {
          const int4 m4 = *reinterpret_cast<const int4*>(sLim + rbase);
          lims[0] = m4.x; lims[1] = m4.y; lims[2] = m4.z; lims[3] = m4.w;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int v = 4 * q4 + c;
          float pa = __builtin_amdgcn_exp2f(__builtin_fmaf(acc0[v], k2, -ls[c]));
          float pb = __builtin_amdgcn_exp2f(__builtin_fmaf(acc1[v], k2, -ls[c]));
          if (LIMIT) {
            if (tA >= lims[c]) pa = 0.f;
            if (tB >= lims[c]) pb = 0.f;
          }
          col0 += pa;
          col1 += pb;
        }
      }
    }
  }
  if (!wave_active) return;
  col0 += __shfl_xor(col0, 32, 64);
  col1 += __shfl_xor(col1, 32, 64);
  if (lane < 32) {
    float* dst = a.colsum + (int64_t)g * a.total_ctx + c0;
    const int tA = tok0 + lane;
    if (tA < T) dst[tA] = col0;
    if (tA + 32 < T) dst[tA + 32] = col1;
  }
}

__global__ __launch_bounds__(256) void score_reduce(ScoreArgs a) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= a.total_ctx) return;
  const int b = find_request(a.ctx_off, a.B, j);
  if (b >= a.B) return;
  const int64_t p0 = min(max(a.probe_off[b], (int64_t)0), a.total_probe);
  const int64_t p1 = min(max(a.probe_off[b + 1], p0), a.total_probe);
  float acc = 0.f;
  for (int g = 0; g < a.Hkv; ++g) acc += a.colsum[(int64_t)g * a.total_ctx + j];
  a.score[j] = (p1 > p0) ? acc / (float)((p1 - p0) * a.H) : 0.f;
}

__global__ __launch_bounds__(256) void score_zero(float* __restrict__ score, int64_t n) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j < n) score[j] = 0.f;
}

bool use_mfma(const qcf_layer_desc& L) { return L.dtype == QCF_DTYPE_BF16 && L.head_dim == 128; }

int64_t n_tiles_upper(int32_t B, int64_t total_ctx) { return (total_ctx + kTokPerWg - 1) / kTokPerWg + B; }

struct MfmaWs { size_t part, colsum, total; };
MfmaWs mfma_ws(const qcf_layer_desc& L, int32_t B, int64_t total_probe, int64_t total_ctx) {
  MfmaWs w;
  w.part = 0;
  size_t off = align_up((size_t)n_tiles_upper(B, total_ctx) * total_probe * L.n_q_heads * sizeof(float2), 256);
  w.colsum = off;
  off += align_up((size_t)L.n_kv_heads * total_ctx * sizeof(float), 256);
  w.total = off;
  return w;
}

constexpr size_t kPass1Lds = (size_t)kRowSplit1 * kQStride * 2 + (size_t)kWavesPerWg * kRowSplit1 * sizeof(float2);
constexpr size_t kPass2Lds = (size_t)kRowBlock * kQStride * 2 + (size_t)kRowBlock * 8;

}  // namespace

size_t score_workspace(const qcf_layer_desc& L, int32_t B, int64_t total_probe, int64_t total_ctx) {
  if (use_mfma(L)) return mfma_ws(L, B, total_probe, total_ctx).total;
  return align_up((size_t)total_probe * L.n_q_heads * total_ctx * sizeof(float), 256);
}

qcf_status launch_score(const qcf_layer_desc& L, int32_t B, const void* q, const int64_t* probe_off,
                        int64_t total_probe, const void* k, const int64_t* ctx_off, int64_t total_ctx,
                        const int32_t* probe_limit, float* score, void* ws, hipStream_t st) {
  const int H = L.n_q_heads, Hkv = L.n_kv_heads, D = L.head_dim;
  if (total_probe == 0) {      // no probe rows at all: every score is 0 (no workspace was asked for)
    const int64_t blocks = (total_ctx + 255) / 256;
    score_zero<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(score, total_ctx);
    return check_launch("score zero");
  }
  if (!use_mfma(L)) {
    float* P = static_cast<float*>(ws);
    const int64_t col_blocks = (total_ctx + 255) / 256;
    if (total_probe * H > 0x7fffffff || col_blocks > 0x7fffffff)
      return fail(QCF_ERR_UNSUPPORTED, "score: too many rows");
    if (total_probe > 0) {
      const dim3 grid((unsigned)(total_probe * H)), block(256);
      if (L.dtype == QCF_DTYPE_BF16)
        score_rows_generic<bf16_t><<<grid, block, 0, st>>>(
            static_cast<const bf16_t*>(q), probe_off, total_probe, static_cast<const bf16_t*>(k), ctx_off,
            total_ctx, B, probe_limit, H, Hkv, D, P);
      else
        score_rows_generic<float><<<grid, block, 0, st>>>(
            static_cast<const float*>(q), probe_off, total_probe, static_cast<const float*>(k), ctx_off,
            total_ctx, B, probe_limit, H, Hkv, D, P);
      QCF_TRY_LAUNCH("score rows");
    }
    score_colmean_generic<<<dim3((unsigned)col_blocks), dim3(256), 0, st>>>(P, probe_off, total_probe, ctx_off,
                                                                           total_ctx, B, H, score);
    return check_launch("score column mean");
  }

  const MfmaWs w = mfma_ws(L, B, total_probe, total_ctx);
  ScoreArgs a;
  a.q = static_cast<const bf16_t*>(q);
  a.k = static_cast<const bf16_t*>(k);
  a.probe_off = probe_off;
  a.ctx_off = ctx_off;
  a.probe_limit = probe_limit;
  a.total_probe = total_probe;
  a.total_ctx = total_ctx;
  a.B = B; a.H = H; a.Hkv = Hkv; a.G = H / Hkv;
  a.part = reinterpret_cast<float2*>(static_cast<char*>(ws) + w.part);
  a.colsum = reinterpret_cast<float*>(static_cast<char*>(ws) + w.colsum);
  a.score = score;
  const int64_t n_tiles = n_tiles_upper(B, total_ctx);
  if (n_tiles > 0x7fffffff || Hkv > 65535) return fail(QCF_ERR_UNSUPPORTED, "score: grid too large");
  const dim3 grid((unsigned)n_tiles, (unsigned)Hkv), block(256);
  const int64_t red_blocks = (total_ctx + 255) / 256;

  static std::atomic<uint64_t> lds_ok[4];
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass1<false>), kPass1Lds, lds_ok[0]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass1<true>), kPass1Lds, lds_ok[1]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass2<false>), kPass2Lds, lds_ok[2]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass2<true>), kPass2Lds, lds_ok[3]));
  if (total_probe > 0) {
    const int64_t row_splits = (total_probe * a.G + kRowSplit1 - 1) / kRowSplit1;      // upper bound over the requests
    if (row_splits > 65535) return fail(QCF_ERR_UNSUPPORTED, "score: too many probe rows");
    const dim3 grid1((unsigned)n_tiles, (unsigned)Hkv, (unsigned)row_splits);
    if (probe_limit) score_pass1<true><<<grid1, block, kPass1Lds, st>>>(a);
    else score_pass1<false><<<grid1, block, kPass1Lds, st>>>(a);
    QCF_TRY_LAUNCH("score pass 1");
    if (probe_limit) score_pass2<true><<<grid, block, kPass2Lds, st>>>(a);
    else score_pass2<false><<<grid, block, kPass2Lds, st>>>(a);
    QCF_TRY_LAUNCH("score pass 2");
  }
  score_reduce<<<dim3((unsigned)red_blocks), dim3(256), 0, st>>>(a);
  return check_launch("score reduce");
}

}  // namespace qcf
