// Step 2: critical-layer attention analysis (Section 3.1 Phase 3; Section 3.2 token
// selector of the paper): score[j] = mean over probe rows and heads of the softmax
// attention the context token j receives.
//
// bf16 / head_dim 128 path (the dense contraction runs on MFMA).  A workgroup of twelve waves owns a
// 256-token tile of one KV head: the tile's keys and the group's probe rows both arrive in LDS through
// asynchronous loads that request every 128-byte line once (loading keys straight into registers in MFMA
// operand layout touches 64 different lines per instruction, which is what bounded the earlier version);
// wave (tw, rg) keeps the 64 tokens of slice tw in registers and takes every third 32-row tile of the rows.
//   pass 1  logits of the probe rows against the tile -> per-row (max, sum-exp) of the tile, in the log2
//           domain (the four token slices folded in LDS);
//   pass 2  every workgroup first folds the partials of its group's rows over the request's tiles into
//           a log2-sum-exp per row (in a fixed order, so all workgroups get the same value); logits
//           again, p = exp2(logit - lse), summed over the rows of the group -> per-KV-head column sums;
//   reduce  fixed-order sum over KV heads, times 1/(R*H).
// Launches that are resident at once (one workgroup per compute unit at most, up to 320 probe rows per KV
// group) take a single kernel instead (score_fused, further down): the exponentials of pass 1 stay in registers
// across a grid-wide exchange of the per-row partials, so the keys are read once and no second pass or reduce
// kernel runs.
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
    const T* __restrict__ q, const int64_t* __restrict__ probe_off, int64_t /*total_probe*/,
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
    const int64_t* __restrict__ ctx_off, int64_t total_ctx, int B, int H, float* score, float alpha, float beta) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= total_ctx) return;
  const int b = find_request(ctx_off, B, j);
  if (b >= B) return;
  const int64_t r0 = min(max(probe_off[b], (int64_t)0), total_probe);
  const int64_t r1 = min(max(probe_off[b + 1], r0), total_probe);
  float acc = 0.f;
  for (int64_t r = r0 * H; r < r1 * H; ++r) acc += P[r * total_ctx + j];
  const float sj = (r1 > r0) ? acc / (float)((r1 - r0) * H) : 0.f;
  score[j] = (beta == 0.f) ? alpha * sj : __builtin_fmaf(beta, score[j], alpha * sj);
}

// ------------------------------------------------------------------ MFMA path (bf16, d = 128)

constexpr int kTokPerWave = 64;                 // tokens a wave keeps stationary in registers
constexpr int kTokWaves = 4;                    // token slices of a workgroup
constexpr int kRowGroups = 3;                   // waves per token slice; they share out the row tiles
constexpr int kWavesPerWg = kTokWaves * kRowGroups;
constexpr int kThreads = 64 * kWavesPerWg;
constexpr int kTokPerWg = kTokPerWave * kTokWaves;
constexpr int kRowBlock = 320;                  // probe rows (of one group) staged in LDS at a time
constexpr int kQStride = 128;                   // bf16 elements per staged row (swizzled, no padding)
constexpr size_t kQBytes = (size_t)kRowBlock * kQStride * 2;
constexpr size_t kKBytes = (size_t)kTokPerWg * 256;
constexpr int kFoldBatch = 16;

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
  float alpha, beta;          // score = beta * score + alpha * (this call's mean attention); beta == 0: plain store
};

// the one place a score is written: plain store, or blended into what is there (accumulation over layers)
__device__ __forceinline__ void write_score(const ScoreArgs& a, int64_t j, float s) {
  a.score[j] = (a.beta == 0.f) ? a.alpha * s : __builtin_fmaf(a.beta, a.score[j], a.alpha * s);
}

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

// Stages the workgroup's 256 key rows (tokens tile_tok0 .. +255 of KV head g) into LDS with asynchronous
// direct-to-LDS loads (a 1 KB instruction = 4 token rows, every 128-byte line requested once); same row
// layout as the probe rows below.  Tokens past the end are clamped (masked or never written later).
__device__ __forceinline__ void stage_k_async(const ScoreArgs& a, int64_t c0, int T, int tile_tok0, int g,
                                              unsigned char* sK, int wave, int lane) {
  for (int j = wave; j < kTokPerWg / 4; j += kWavesPerWg) {
    const int r = 4 * j + (lane >> 4);
    const int tok = min(tile_tok0 + r, T - 1);
    const int chunk = (lane & 15) ^ (r & 15);
    load_to_lds_addr(a.k + ((c0 + tok) * a.Hkv + g) * 128 + chunk * 8, sK + j * 1024);
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

// Pass 1.  A workgroup = (256-token tile, KV head); wave (tw, rg) keeps the 64 tokens of slice tw in
// registers and takes every third 32-row tile of the staged probe rows, starting with tile rg.
template <bool LIMIT>
__global__ __launch_bounds__(kThreads) void score_pass1(ScoreArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* sK = smem + kQBytes;
  float2* sPart = reinterpret_cast<float2*>(smem + kQBytes + kKBytes);     // [kTokWaves][kRowBlock]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tw = wave % kTokWaves, rg = wave / kTokWaves;
  const int g = blockIdx.y;
  int b, T, tile_tok0, tile_first;
  int64_t c0;
  if (!locate_tile(a, blockIdx.x, b, c0, T, tile_tok0, tile_first)) return;
  const int64_t p0 = min(max(a.probe_off[b], (int64_t)0), a.total_probe);
  const int64_t p1 = min(max(a.probe_off[b + 1], p0), a.total_probe);
  const int rows = (int)(p1 - p0) * a.G;         // probe rows x heads of the group
  if (rows == 0) return;
  const int tok0 = tile_tok0 + tw * kTokPerWave;
  const bool wave_active = tok0 < T;
  const float k2 = kLog2e * 0.08838834764831845f;   // log2(e) / sqrt(128)
  // byte offset of this lane's fragment (row lane%32, chunk 2*ks + lane/32) is qb0 ^ (32 * ks)
  const int qb0 = (lane & 31) * 256 + (((lane >> 5) ^ (lane & 15)) * 16);
  float2* part = a.part + (int64_t)blockIdx.x * (a.total_probe * a.H);

  stage_k_async(a, c0, T, tile_tok0, g, sK, wave, lane);
  bf16x8 kf[2][8];
  for (int r_begin = 0; r_begin < rows; r_begin += kRowBlock) {
    const int n_rows = min(kRowBlock, rows - r_begin);
    const int n_pad = (n_rows + 31) & ~31;
    __syncthreads();                        // the previous block's rows and partials are no longer read
    stage_q_async(a, p0, g, r_begin, n_rows, n_pad, smem, wave, lane);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (r_begin == 0) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          kf[mt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                                                      sK + (kTokPerWave * tw + 32 * mt) * 256 + (qb0 ^ (32 * ks))));
    }
    for (int rt = 32 * rg; rt < n_pad; rt += 32 * kRowGroups) {
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
      if (lane < 32) sPart[tw * kRowBlock + rt + lane] = make_float2(mx, sum);
    }
    __syncthreads();
    // the four token slices' partials of a row fold, in slice order, into the tile's partial
    for (int r = tid; r < n_rows; r += kThreads) {
      float2 p[kTokWaves];
      float m = -INFINITY;
#pragma unroll
      for (int w = 0; w < kTokWaves; ++w) { p[w] = sPart[w * kRowBlock + r]; m = fmaxf(m, p[w].x); }
      float z = 0.f;
#pragma unroll
      for (int w = 0; w < kTokWaves; ++w)
        if (p[w].x > -INFINITY) z += p[w].y * exp2f(p[w].x - m);
      const int rr = r_begin + r;
      const int i = rr / a.G, hh = rr - i * a.G;
      part[(p0 + i) * a.H + g * a.G + hh] = make_float2(m, z);
    }
  }
}

// Folds a batch of (max2, sumexp2) partials, in order, into the running pair (m, z).  A partial that saw
// nothing is (-inf, 0) and contributes 0 * exp2(-inf) = 0.
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

// Pass 2, same division of work; the three row groups' column sums are added in a fixed order at the end.
template <bool LIMIT>
__global__ __launch_bounds__(kThreads) void score_pass2(ScoreArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* sK = smem + kQBytes;
  float* sL = reinterpret_cast<float*>(smem + kQBytes + kKBytes);          // [kRowBlock] log2-sum-exp
  int* sLim = reinterpret_cast<int*>(sL + kRowBlock);                       // [kRowBlock]
  float* sCol = reinterpret_cast<float*>(sLim + kRowBlock);                 // [kRowGroups][kTokPerWg]
  static_assert(kRowBlock <= kThreads, "one thread folds one staged row");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tw = wave % kTokWaves, rg = wave / kTokWaves;
  const int g = blockIdx.y;
  int b, T, tile_tok0, tile_first;
  int64_t c0;
  if (!locate_tile(a, blockIdx.x, b, c0, T, tile_tok0, tile_first)) return;
  const int64_t p0 = min(max(a.probe_off[b], (int64_t)0), a.total_probe);
  const int64_t p1 = min(max(a.probe_off[b + 1], p0), a.total_probe);
  const int rows = (int)(p1 - p0) * a.G;
  if (rows == 0) return;                 // (the reduce kernel gives such a request zeros without reading the sums)
  const int n_tiles = (T + kTokPerWg - 1) / kTokPerWg;
  const int64_t part_stride = a.total_probe * a.H;
  const int tok0 = tile_tok0 + tw * kTokPerWave;
  const bool wave_active = tok0 < T;
  const float k2 = kLog2e * 0.08838834764831845f;
  const int qb0 = (lane & 31) * 256 + (((lane >> 5) ^ (lane & 15)) * 16);

  stage_k_async(a, c0, T, tile_tok0, g, sK, wave, lane);
  bf16x8 kf[2][8];
  float col0 = 0.f, col1 = 0.f;        // column sums of tokens tok0 + lane%32 and + 32 over this wave's row tiles

  for (int r_begin = 0; r_begin < rows; r_begin += kRowBlock) {
    const int n_rows = min(kRowBlock, rows - r_begin);
    const int n_pad = (n_rows + 31) & ~31;
    __syncthreads();
    stage_q_async(a, p0, g, r_begin, n_rows, n_pad, smem, wave, lane);
    // log2-sum-exp of staged row tid over the request: the tiles' partials folded in tile order, kFoldBatch
    // at a time (all loads first, then one maximum and one rescaled sum); every workgroup of the request
    // computes the same values
    if (tid < n_pad) {
      float l = INFINITY;               // rows that do not exist or see nothing: exp2(logit - lse) = 0
      int lim = 0;
      if (tid < n_rows) {
        const int rr = r_begin + tid, i = rr / a.G, hh = rr - i * a.G;
        const float2* pp = a.part + (int64_t)tile_first * part_stride + (p0 + i) * a.H + g * a.G + hh;
        float m = -INFINITY, z = 0.f;
        for (int t0 = 0; t0 < n_tiles; t0 += kFoldBatch) {
          float2 p[kFoldBatch];
#pragma unroll
          for (int u = 0; u < kFoldBatch; ++u) {
            p[u] = (t0 + u < n_tiles) ? *pp : make_float2(-INFINITY, 0.f);
            pp += part_stride;          // (stays inside the workspace: n_tiles <= the tiles allocated)
          }
          fold_partials(p, m, z);
        }
        if (z > 0.f) l = m + log2f(z);
        lim = LIMIT ? min(T, max(0, a.probe_limit[p0 + i])) : T;
      }
      sL[tid] = l;
      sLim[tid] = lim;
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (r_begin == 0) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          kf[mt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                                                      sK + (kTokPerWave * tw + 32 * mt) * 256 + (qb0 ^ (32 * ks))));
    }
    if (!wave_active) continue;
    for (int rt = 32 * rg; rt < n_pad; rt += 32 * kRowGroups) {
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
  col0 += __shfl_xor(col0, 32, 64);
  col1 += __shfl_xor(col1, 32, 64);
  if (lane < 32) {
    float* sc = sCol + rg * kTokPerWg + tw * kTokPerWave;
    sc[lane] = col0;                      // (zero for a slice past the end of the request)
    sc[32 + lane] = col1;
  }
  __syncthreads();
  if (tid < kTokPerWg && tile_tok0 + tid < T) {
    float sum = sCol[tid];
#pragma unroll
    for (int r3 = 1; r3 < kRowGroups; ++r3) sum += sCol[r3 * kTokPerWg + tid];
    a.colsum[(int64_t)g * a.total_ctx + c0 + tile_tok0 + tid] = sum;
  }
}

// ------------------------------------------------------------------ single-kernel path
//
// When the whole launch is resident at once (one workgroup per compute unit, at most as many workgroups as
// compute units) and a KV group has at most kRowBlock probe rows, one kernel does everything.  A workgroup of
// eight waves owns a 256-token tile of one KV head; wave w keeps tokens 32w .. 32w+31 stationary and walks all
// row tiles.  It keeps, in registers, e = 2^(logit - m) against the maximum m of its own 32 tokens for every
// (token, row) pair of the tile: the second exponential of a two-pass scheme becomes one multiply-add by
// 2^(m - lse) once the row's log-sum-exp over the whole request is known.
//
// Two hand-offs between workgroups, both through device-scope relaxed atomics on data that is itself written
// and read with device-scope atomic stores and loads (they bypass the non-coherent caches; a wave waits for
// its own stores to complete before it signals, so no cache-wide release or acquire fence is needed):
//   1. the tiles of one (request, KV head) exchange their per-row (max, sum-exp): every workgroup publishes
//      its partials, adds one to the group's arrival counter and waits until all tiles of the request have
//      arrived (bounded wait: all workgroups of the launch are resident, so every one of them is running);
//   2. the KV heads of one tile exchange their column sums: the last head to arrive (found with a counter; no
//      waiting) adds the heads in head order and writes the scores.
// All sums run in a fixed order, so the scores are bit-stable.  The counters live in a device array that the
// loader zero-fills; the last workgroup to finish resets the ones this launch used, so every launch starts from
// zero without a clearing kernel.  Launches take turns over kSyncSlots sets of counters.

constexpr int kFusedWaves = 8;
constexpr int kFusedThreads = 64 * kFusedWaves;
constexpr int kFusedRowTiles = kRowBlock / 32;
constexpr int kSyncSlots = 8;
constexpr int kSyncWords = 1024;           // counters per slot: [0] finished workgroups, then groups, then tiles
constexpr uint32_t kSpinLimit = 1u << 20;  // polls (a microsecond or two each) before a workgroup gives up waiting

__device__ uint32_t g_sync[kSyncSlots * kSyncWords];

struct FusedArgs {
  ScoreArgs s;
  float2* part;        // [tile][Hkv][kRowBlock] (max2, sumexp2) of the tile, published with atomic stores
  float* colpart;      // [tile][Hkv][kTokPerWg] column sums of one KV head
  uint32_t* sync;      // this launch's counter slot
  int n_wg_tiles;      // tiles the grid provides (upper bound on the tiles of all requests)
  uint32_t spin_limit;
};

__device__ __forceinline__ void publish(float2* p, float2 v) {
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), __builtin_bit_cast(uint64_t, v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 fetch(const float2* p) {
  return __builtin_bit_cast(float2, __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void publish(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float fetch(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// exchange between the two 32-lane halves of a wave (one vector instruction, no LDS round trip):
// returns the value the lane 32 away holds
__device__ __forceinline__ float other_half(float x) {
  typedef unsigned u2v __attribute__((ext_vector_type(2)));
  const u2v r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  // r.x = (lower half's value in both halves), r.y = (upper half's value in both halves)
  return (threadIdx.x & 32) ? __uint_as_float(r.x) : __uint_as_float(r.y);
}
// sum over the 32 lanes of each half of a wave, in a fixed order; every lane of the half gets the total
__device__ __forceinline__ float half_wave_sum(float x) {
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x128, 0xf, 0xf, false));   // row_ror:8
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x124, 0xf, 0xf, false));   // row_ror:4
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x122, 0xf, 0xf, false));   // row_ror:2
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x121, 0xf, 0xf, false));   // row_ror:1
  typedef unsigned u2v __attribute__((ext_vector_type(2)));
  const u2v r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r.x) + __uint_as_float(r.y);     // rows (0, 1) and (2, 3) of 16 lanes each
}

template <bool LIMIT>
__global__ __launch_bounds__(kFusedThreads) void score_fused(FusedArgs fa) {
  const ScoreArgs& a = fa.s;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* sK = smem + kQBytes;
  // (reused once the key fragments are in registers)
  float2* sPart = reinterpret_cast<float2*>(sK);                            // [kFusedWaves][kRowBlock]
  float* sL = reinterpret_cast<float*>(sK + kFusedWaves * kRowBlock * 8);   // [kRowBlock] log2-sum-exp
  float* sCol = sL + kRowBlock;                                             // [kTokPerWg]
  __shared__ int s_flag[2];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hf = lane >> 5, l32 = lane & 31;
  const int g = (int)(blockIdx.x % a.Hkv);
  const int wg_tile = (int)(blockIdx.x / a.Hkv);
  const int n_wg = fa.n_wg_tiles * a.Hkv;

  int b, T, tile_tok0, tile_first;
  int64_t c0;
  const bool have_tile = locate_tile(a, wg_tile, b, c0, T, tile_tok0, tile_first);
  int rows = 0;
  int64_t p0 = 0;
  if (have_tile) {
    p0 = min(max(a.probe_off[b], (int64_t)0), a.total_probe);
    const int64_t p1 = min(max(a.probe_off[b + 1], p0), a.total_probe);
    rows = min((int)(p1 - p0) * a.G, kRowBlock);       // (the launcher only takes this path when all rows fit)
  }
  const int n_tiles = have_tile ? (T + kTokPerWg - 1) / kTokPerWg : 0;
  const int n_rt = (rows + 31) >> 5;
  const float k2 = kLog2e * 0.08838834764831845f;   // log2(e) / sqrt(128)

  float e[kFusedRowTiles][16];      // 2^(logit - m_w) of (token, row) pairs; row = 32 rt + l32

  if (rows > 0) {
    for (int j = wave; j < kTokPerWg / 4; j += kFusedWaves) {          // keys: 1 KB per instruction = 4 token rows
      const int r = 4 * j + (lane >> 4);
      const int tok = min(tile_tok0 + r, T - 1);
      const int chunk = (lane & 15) ^ (r & 15);
      load_to_lds_addr(a.k + ((c0 + tok) * a.Hkv + g) * 128 + chunk * 8, sK + j * 1024);
    }
    for (int j = wave; j < n_rt * 8; j += kFusedWaves) {               // probe rows of the group
      const int r = 4 * j + (lane >> 4);
      const int rr = min(r, rows - 1);
      const int i = rr / a.G, hh = rr - i * a.G;
      const int chunk = (lane & 15) ^ (r & 15);
      load_to_lds_addr(a.q + ((p0 + i) * a.H + g * a.G + hh) * 128 + chunk * 8, smem + j * 1024);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    const int fb0 = l32 * 256 + ((hf ^ (lane & 15)) * 16);       // fragment ks of row l32 sits at fb0 ^ (32 ks)
    bf16x8 kf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      kf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(sK + (32 * wave) * 256 + (fb0 ^ (32 * ks))));
    // probe-row fragments travel through a ring of four registers: fragment ks + 4 (or the next tile's
    // fragment ks - 4) is requested right behind the MFMA that used the slot.  One address register per
    // fragment index; the row tile is a constant offset of the read.
    uint32_t qaddr[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qaddr[ks] = lds_offset_of(smem) + (uint32_t)(fb0 ^ (32 * ks));
    auto qfrag = [&](int rt, int ks) {
      return *(const u32x4 __attribute__((address_space(3)))*)(uintptr_t)(qaddr[ks] + (uint32_t)(rt * 32 * 256));
    };
    u32x4 ring[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ring[i] = qfrag(0, i);
    __syncthreads();                               // the key tile's LDS is reused from here on
    const int tok0 = tile_tok0 + 32 * wave;
#pragma unroll
    for (int rt = 0; rt < kFusedRowTiles; ++rt) {
      if (rt < n_rt) {
        floatx16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          // S^T tile: rows = tokens (A = keys), columns = probe rows (B = queries)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], __builtin_bit_cast(bf16x8, ring[ks & 3]), acc, 0, 0, 0);
          if (ks < 4) ring[ks & 3] = qfrag(rt, ks + 4);
          else if (rt + 1 < kFusedRowTiles) ring[ks & 3] = qfrag(rt + 1, ks - 4);   // (unused after the last tile)
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {          // issue order: every read sits behind the MFMA that frees its slot
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (ks < 4 || rt + 1 < kFusedRowTiles) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        // lane owns probe row 32 rt + l32; register v is token tok0 + 8 (v/4) + 4 hf + v%4
        float sv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) sv[v] = acc[v];
        if (LIMIT || tok0 + 32 > T) {            // wave-uniform: only ragged or limited tiles compare
          const int r = 32 * rt + l32;
          int lim = T;
          if (LIMIT && r < rows) lim = min(T, max(0, a.probe_limit[p0 + r / a.G]));
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int t0 = tok0 + 8 * (v >> 2) + 4 * hf + (v & 3);
            sv[v] = (t0 < lim) ? sv[v] : -INFINITY;
          }
        }
        float mx = sv[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sv[v]);
        mx = fmaxf(mx, other_half(mx)) * k2;          // k2 > 0: scaling commutes with the maximum
        const float m_use = (mx == -INFINITY) ? 0.f : mx;
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          e[rt][v] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[v], k2, -m_use));
          sum += e[rt][v];
        }
        sum += other_half(sum);
        if (lane < 32) sPart[wave * kRowBlock + 32 * rt + lane] = make_float2(mx, sum);
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) e[rt][v] = 0.f;
      }
    }
    __syncthreads();
    // the eight token slices' partials of a row fold, in slice order, into the tile's partial
    float2* part = fa.part + ((int64_t)wg_tile * a.Hkv + g) * kRowBlock;
    for (int r = tid; r < rows; r += kFusedThreads) {
      float2 p[kFusedWaves];
      float m = -INFINITY;
#pragma unroll
      for (int w = 0; w < kFusedWaves; ++w) { p[w] = sPart[w * kRowBlock + r]; m = fmaxf(m, p[w].x); }
      float z = 0.f;
#pragma unroll
      for (int w = 0; w < kFusedWaves; ++w)
        if (p[w].x > -INFINITY) z += p[w].y * exp2f(p[w].x - m);
      publish(part + r, make_float2(m, z));
    }
    __builtin_amdgcn_s_waitcnt(0);            // this thread's partials have reached memory
    __syncthreads();
    // hand-off 1: the tiles of (request b, KV head g)
    if (tid == 0) {
      uint32_t* cnt = fa.sync + 1 + b * a.Hkv + g;
      __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      uint32_t spins = 0;
      while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (uint32_t)n_tiles &&
             ++spins < fa.spin_limit)
        __builtin_amdgcn_s_sleep(1);
    }
    __syncthreads();
    // log2-sum-exp of row r over the request: the tiles' partials folded in tile order (up to 32 loads in
    // flight per thread)
    for (int r = tid; r < rows; r += kFusedThreads) {
      const float2* pp = fa.part + ((int64_t)tile_first * a.Hkv + g) * kRowBlock + r;
      const int64_t stride = (int64_t)a.Hkv * kRowBlock;
      float m = -INFINITY, z = 0.f;
      for (int t0 = 0; t0 < n_tiles; t0 += 2 * kFoldBatch) {
        float2 pa[kFoldBatch], pb[kFoldBatch];
#pragma unroll
        for (int u = 0; u < kFoldBatch; ++u) {
          pa[u] = (t0 + u < n_tiles) ? fetch(pp + u * stride) : make_float2(-INFINITY, 0.f);
          pb[u] = (t0 + kFoldBatch + u < n_tiles) ? fetch(pp + (kFoldBatch + u) * stride) : make_float2(-INFINITY, 0.f);
        }
        pp += 2 * kFoldBatch * stride;
        fold_partials(pa, m, z);
        fold_partials(pb, m, z);
      }
      sL[r] = (z > 0.f) ? m + log2f(z) : INFINITY;      // a row that sees nothing: every weight is 0
    }
    for (int r = rows + tid; r < 32 * n_rt; r += kFusedThreads) sL[r] = INFINITY;
    __syncthreads();
    // column sums over this wave's rows: e * 2^(m_w - lse), row tiles in order, then over the lanes
    float col[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) col[v] = 0.f;
#pragma unroll
    for (int rt = 0; rt < kFusedRowTiles; ++rt) {
      if (rt < n_rt) {
        const float l = sL[32 * rt + l32];
        const float mw = sPart[wave * kRowBlock + 32 * rt + l32].x;
        const float w = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - l);
#pragma unroll
        for (int v = 0; v < 16; ++v) col[v] = __builtin_fmaf(e[rt][v], w, col[v]);
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) col[v] = half_wave_sum(col[v]);
    if (l32 == 0) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sCol[32 * wave + 8 * (v >> 2) + 4 * hf + (v & 3)] = col[v];
    }
    __syncthreads();
    float* colpart = fa.colpart + ((int64_t)wg_tile * a.Hkv + g) * kTokPerWg;
    if (tid < kTokPerWg) publish(colpart + tid, sCol[tid]);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    // hand-off 2: the KV heads of this tile; the last one to arrive adds them up.  The count of finished
    // workgroups is sent right behind (its operand depends on the first counter's answer, so the two
    // additions cannot pass each other) and its answer is only looked at after the sums.
    uint32_t fin = 0;
    if (tid == 0) {
      uint32_t* cnt = fa.sync + 1 + a.B * a.Hkv + wg_tile;
      const uint32_t old = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_flag[0] = (old == (uint32_t)a.Hkv - 1u) ? 1 : 0;
      fin = __hip_atomic_fetch_add(fa.sync, 1u + (old >> 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (s_flag[0] && tid < kTokPerWg && tile_tok0 + tid < T) {
      const float* cp = fa.colpart + (int64_t)wg_tile * a.Hkv * kTokPerWg + tid;
      float acc = 0.f;
      for (int gg = 0; gg < a.Hkv; ++gg) acc += fetch(cp + gg * kTokPerWg);
      write_score(a, c0 + tile_tok0 + tid, acc / (float)((rows / a.G) * a.H));
    }
    if (tid == 0) s_flag[1] = (fin == (uint32_t)n_wg - 1u) ? 1 : 0;
    __syncthreads();
  } else {
    // a request without probe rows scores zero everywhere
    if (have_tile && g == 0 && tid < kTokPerWg && tile_tok0 + tid < T) write_score(a, c0 + tile_tok0 + tid, 0.f);
    if (tid == 0) {
      const uint32_t fin = __hip_atomic_fetch_add(fa.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_flag[1] = (fin == (uint32_t)n_wg - 1u) ? 1 : 0;
    }
    __syncthreads();
  }
  // the last workgroup of the launch to have counted itself finished puts the launch's counters back to zero
  // (every other workgroup has used its counters by then: a workgroup counts itself after its last use)
  if (s_flag[1]) {
    const int n_words = 1 + a.B * a.Hkv + fa.n_wg_tiles;
    for (int i = tid; i < n_words; i += kFusedThreads)
      __hip_atomic_store(fa.sync + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
  write_score(a, j, (p1 > p0) ? acc / (float)((p1 - p0) * a.H) : 0.f);
}

__global__ __launch_bounds__(256) void score_zero(float* score, int64_t n, float beta) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j < n) score[j] = (beta == 0.f) ? 0.f : beta * score[j];
}

bool use_mfma(const qcf_layer_desc& L) { return L.dtype == QCF_DTYPE_BF16 && L.head_dim == 128; }

// upper bound on the 256-token tiles of all requests (tiles start at request boundaries: every request adds at
// most one partly filled tile); exact for a single request
int64_t n_tiles_upper(int32_t B, int64_t total_ctx) { return (total_ctx + (int64_t)B * (kTokPerWg - 1)) / kTokPerWg; }

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

constexpr size_t kPass1Lds = kQBytes + kKBytes + (size_t)kTokWaves * kRowBlock * sizeof(float2);
constexpr size_t kPass2Lds = kQBytes + kKBytes + (size_t)kRowBlock * 8 + (size_t)kRowGroups * kTokPerWg * sizeof(float);
constexpr size_t kFusedLds = kQBytes + kKBytes;
static_assert((size_t)kFusedWaves * kRowBlock * 8 + (size_t)kRowBlock * 4 + (size_t)kTokPerWg * 4 <= kKBytes,
              "the single-kernel path's tables fit in the key tile's LDS");

// The single-kernel path needs every workgroup of the launch resident at once (one per compute unit) and all
// probe rows of a KV group in one staged block.  The host only knows totals, so the test is on those.
bool use_fused(const qcf_layer_desc& L, int32_t B, int64_t total_probe, int64_t total_ctx) {
  if (!use_mfma(L) || total_probe <= 0) return false;
  const int64_t G = L.n_q_heads / L.n_kv_heads;
  const int64_t tiles = n_tiles_upper(B, total_ctx);
  return total_probe * G <= kRowBlock && tiles * L.n_kv_heads <= compute_unit_count() &&
         1 + (int64_t)B * L.n_kv_heads + tiles <= kSyncWords;
}
struct FusedWs { size_t part, colpart, total; };
FusedWs fused_ws(const qcf_layer_desc& L, int32_t B, int64_t total_ctx) {
  const size_t slots = (size_t)n_tiles_upper(B, total_ctx) * L.n_kv_heads;
  FusedWs w;
  w.part = 0;
  w.colpart = align_up(slots * kRowBlock * sizeof(float2), 256);
  w.total = w.colpart + align_up(slots * kTokPerWg * sizeof(float), 256);
  return w;
}

// Device address of the zero-initialised counter array on the current device (asked for once per device).
qcf_status sync_counters(uint32_t** out) {
  constexpr int kMaxDev = 64;
  static std::atomic<uint32_t*> ptr[kMaxDev];
  int dev = 0;
  QCF_TRY(check_hip(hipGetDevice(&dev), "hipGetDevice"));
  if (dev < 0 || dev >= kMaxDev) return fail(QCF_ERR_UNSUPPORTED, "device id %d >= %d", dev, kMaxDev);
  uint32_t* p = ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void* q = nullptr;
    QCF_TRY(check_hip(hipGetSymbolAddress(&q, HIP_SYMBOL(g_sync)), "hipGetSymbolAddress(g_sync)"));
    if (!q) return fail(QCF_ERR_HIP, "hipGetSymbolAddress(g_sync) returned a null address");
    p = static_cast<uint32_t*>(q);
    ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return QCF_OK;
}

}  // namespace

size_t score_workspace(const qcf_layer_desc& L, int32_t B, int64_t total_probe, int64_t total_ctx) {
  if (use_fused(L, B, total_probe, total_ctx)) return fused_ws(L, B, total_ctx).total;
  if (use_mfma(L)) return mfma_ws(L, B, total_probe, total_ctx).total;
  return align_up((size_t)total_probe * L.n_q_heads * total_ctx * sizeof(float), 256);
}

qcf_status launch_score(const qcf_layer_desc& L, int32_t B, const void* q, const int64_t* probe_off,
                        int64_t total_probe, const void* k, const int64_t* ctx_off, int64_t total_ctx,
                        const int32_t* probe_limit, float* score, float alpha, float beta, void* ws, hipStream_t st) {
  const int H = L.n_q_heads, Hkv = L.n_kv_heads, D = L.head_dim;
  if (total_probe == 0) {      // no probe rows at all: every score is 0 (no workspace was asked for)
    const int64_t blocks = (total_ctx + 255) / 256;
    score_zero<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(score, total_ctx, beta);
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
                                                                           total_ctx, B, H, score, alpha, beta);
    return check_launch("score column mean");
  }

  ScoreArgs a;
  a.q = static_cast<const bf16_t*>(q);
  a.k = static_cast<const bf16_t*>(k);
  a.probe_off = probe_off;
  a.ctx_off = ctx_off;
  a.probe_limit = probe_limit;
  a.total_probe = total_probe;
  a.total_ctx = total_ctx;
  a.B = B; a.H = H; a.Hkv = Hkv; a.G = H / Hkv;
  a.part = nullptr;
  a.colsum = nullptr;
  a.score = score;
  a.alpha = alpha;
  a.beta = beta;
  if (use_fused(L, B, total_probe, total_ctx)) {
    const FusedWs fw = fused_ws(L, B, total_ctx);
    FusedArgs fa;
    fa.s = a;
    fa.part = reinterpret_cast<float2*>(static_cast<char*>(ws) + fw.part);
    fa.colpart = reinterpret_cast<float*>(static_cast<char*>(ws) + fw.colpart);
    fa.n_wg_tiles = (int)n_tiles_upper(B, total_ctx);
    fa.spin_limit = kSpinLimit;
    uint32_t* counters = nullptr;
    QCF_TRY(sync_counters(&counters));
    static std::atomic<uint32_t> next_slot{0};
    fa.sync = counters + (size_t)(next_slot.fetch_add(1, std::memory_order_relaxed) % kSyncSlots) * kSyncWords;
    static std::atomic<uint64_t> fused_lds_ok[2];
    QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_fused<false>), kFusedLds, fused_lds_ok[0]));
    QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_fused<true>), kFusedLds, fused_lds_ok[1]));
    const dim3 fgrid((unsigned)(fa.n_wg_tiles * Hkv)), fblock(kFusedThreads);
    if (probe_limit) score_fused<true><<<fgrid, fblock, kFusedLds, st>>>(fa);
    else score_fused<false><<<fgrid, fblock, kFusedLds, st>>>(fa);
    return check_launch("score (single kernel)");
  }
  const MfmaWs w = mfma_ws(L, B, total_probe, total_ctx);
  a.part = reinterpret_cast<float2*>(static_cast<char*>(ws) + w.part);
  a.colsum = reinterpret_cast<float*>(static_cast<char*>(ws) + w.colsum);
  a.score = score;
  const int64_t n_tiles = n_tiles_upper(B, total_ctx);
  if (n_tiles > 0x7fffffff || Hkv > 65535) return fail(QCF_ERR_UNSUPPORTED, "score: grid too large");
  const dim3 grid((unsigned)n_tiles, (unsigned)Hkv), block(kThreads);
  const int64_t red_blocks = (total_ctx + 255) / 256;

  static std::atomic<uint64_t> lds_ok[4];
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass1<false>), kPass1Lds, lds_ok[0]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass1<true>), kPass1Lds, lds_ok[1]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass2<false>), kPass2Lds, lds_ok[2]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&score_pass2<true>), kPass2Lds, lds_ok[3]));
  if (total_probe > 0) {
    if (probe_limit) score_pass1<true><<<grid, block, kPass1Lds, st>>>(a);
    else score_pass1<false><<<grid, block, kPass1Lds, st>>>(a);
    QCF_TRY_LAUNCH("score pass 1");
    if (probe_limit) score_pass2<true><<<grid, block, kPass2Lds, st>>>(a);
    else score_pass2<false><<<grid, block, kPass2Lds, st>>>(a);
    QCF_TRY_LAUNCH("score pass 2");
  }
  score_reduce<<<dim3((unsigned)red_blocks), dim3(256), 0, st>>>(a);
  return check_launch("score reduce");
}

}  // namespace qcf

// ---- scoring for callers that cannot allocate -----------------------------------------------------
// The scratch of the kernels above (tile partials and per-head column sums, or the probability rows of
// the generic path) lives in a device array that is part of the loaded code object: every GPU the library
// runs on holds its own copy, at its own address, until the process ends.  In host code the array's name is
// only a handle: the device address is asked for once per device (with that device current) and kept, and
// that pointer is what the launchers receive.
namespace {

__device__ __align__(256) unsigned char scratch[QCF_SCORE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

qcf_status scratch_of_current_device(void** out) {
  int dev = 0;
  QCF_TRY(qcf::check_hip(hipGetDevice(&dev), "hipGetDevice"));
  if (dev < 0 || dev >= kMaxDevices) return qcf::fail(QCF_ERR_UNSUPPORTED, "device id %d >= %d", dev, kMaxDevices);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    // (two threads may both ask; they get the same address)
    QCF_TRY(qcf::check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)"));
    if (!p) return qcf::fail(QCF_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return QCF_OK;
}

}  // namespace

extern "C" qcf_status qcf_score_static(const qcf_layer_desc* desc, int32_t B, const void* q_probe,
                                       const int64_t* probe_off_dev, int64_t total_probe, const void* k_fused,
                                       const int64_t* ctx_off_dev, int64_t total_ctx,
                                       const int32_t* probe_limit_dev, float* score, void* stream) {
  bool empty = false;
  QCF_TRY(qcf::check_score_args(desc, B, q_probe, probe_off_dev, total_probe, k_fused, ctx_off_dev, total_ctx,
                                probe_limit_dev, score, &empty));
  if (empty) return QCF_OK;
  const size_t need = qcf::score_workspace(*desc, B, total_probe, total_ctx);
  if (need > (size_t)QCF_SCORE_STATIC_SCRATCH_BYTES)
    return qcf::fail(QCF_ERR_WORKSPACE_TOO_SMALL,
                     "qcf_score_static: this problem needs %zu bytes of scratch, the built-in buffer has %zu; "
                     "use qcf_score with a caller-supplied workspace",
                     need, (size_t)QCF_SCORE_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  QCF_TRY(scratch_of_current_device(&ws));
  return qcf::launch_score(*desc, B, q_probe, probe_off_dev, total_probe, k_fused, ctx_off_dev, total_ctx,
                           probe_limit_dev, score, 1.f, 0.f, ws, (hipStream_t)stream);
}
