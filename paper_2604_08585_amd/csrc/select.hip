// Step 3: Top-N selection (Section 3.1 Phase 3 / Section 3.2 token selector of the paper).
//
// One 1024-thread workgroup per request.  Scores map to order-preserving 32-bit keys; an
// MSB-first radix select over the bits in which the keys actually differ finds the N-th
// largest key and how many of its ties to admit; a block-wide prefix scan then compacts the
// admitted indices in index order, so the output is ascending and ties go to the lower index.
// Integer work only: exact and deterministic.
#include "qcf_internal.h"

namespace qcf {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kDigitBits = 9;                 // bits resolved per pass (measured best of 8..11 at 8192 keys)
constexpr int kBins = 1 << kDigitBits;
constexpr int kBinsPerLane = kBins / 64;     // the first wave scans the histogram

__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t u = __float_as_uint(s);
  if (u == 0x80000000u) u = 0u;      // -0 and +0 are the same score
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t wave_incl_scan(uint64_t v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t lo = __shfl_up((uint32_t)v, d, 64);
    const uint32_t hi = __shfl_up((uint32_t)(v >> 32), d, 64);
    if (lane >= d) v += ((uint64_t)hi << 32) | lo;
  }
  return v;
}

// SEG > 0: each thread keeps up to SEG keys of its contiguous segment in registers.
// SEG == 0: keys are re-read from global memory in every pass (any length).
template <int SEG>
__global__ __launch_bounds__(kThreads) void select_kernel(
    const float* __restrict__ score, const int64_t* __restrict__ ctx_off, int64_t total_ctx,
    const int64_t* __restrict__ sel_off, int64_t total_sel, const int32_t* __restrict__ ctx_pos0,
    int32_t* __restrict__ sel_idx, int32_t* __restrict__ sel_row, int32_t* __restrict__ sel_pos) {
  __shared__ uint32_t merged[kBins];
  __shared__ uint64_t wave_tot[kWaves];
  __shared__ uint32_t red_lo[kWaves], red_hi[kWaves];
  __shared__ uint32_t s_digit, s_k;

  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int64_t c0 = ctx_off[b], c1 = ctx_off[b + 1];
  c0 = min(max(c0, (int64_t)0), total_ctx);
  c1 = min(max(c1, c0), total_ctx);
  int64_t o0 = sel_off[b], o1 = sel_off[b + 1];
  o0 = min(max(o0, (int64_t)0), total_sel);
  o1 = min(max(o1, o0), total_sel);
  const int T = (int)(c1 - c0);
  const int N = (int)min((int64_t)T, o1 - o0);
  if (N <= 0) return;
  const float* s = score + c0;

  const int seg = (T + kThreads - 1) / kThreads;
  const int j0 = min(T, tid * seg), j1 = min(T, j0 + seg);
  const int cnt = j1 - j0;
  if (SEG > 0 && seg > SEG) return;          // launcher guarantees this cannot happen

  uint32_t keys[SEG > 0 ? SEG : 1];
  if (SEG > 0) {
    // a full, 16-byte aligned segment is read as vectors (a quarter of the memory instructions)
    if (SEG % 4 == 0 && cnt == SEG && ((reinterpret_cast<uintptr_t>(s + j0) & 15u) == 0)) {
#pragma unroll
      for (int i = 0; i < SEG / 4; ++i) {
        const float4 v = *reinterpret_cast<const float4*>(s + j0 + 4 * i);
        keys[4 * i + 0] = order_key(v.x);
        keys[4 * i + 1] = order_key(v.y);
        keys[4 * i + 2] = order_key(v.z);
        keys[4 * i + 3] = order_key(v.w);
      }
    } else {
#pragma unroll
      for (int i = 0; i < SEG; ++i) keys[i] = (i < cnt) ? order_key(s[j0 + i]) : 0u;
    }
  }
#define QCF_KEY(i) (SEG > 0 ? keys[i] : order_key(s[j0 + (i)]))
#define QCF_FOR_KEYS(i, ...)                                   \
  if (SEG > 0) {                                               \
    _Pragma("unroll") for (int i = 0; i < SEG; ++i) {          \
      if (i < cnt) { __VA_ARGS__ }                             \
    }                                                          \
  } else {                                                     \
    for (int i = 0; i < cnt; ++i) { __VA_ARGS__ }              \
  }

  const int base_pos = ctx_pos0 ? ctx_pos0[b] : 0;
  uint32_t tau = 0;       // key of the N-th largest score
  uint32_t k = (uint32_t)N;   // how many keys equal to tau are admitted

  if (N < T) {
    // range of the keys
    uint32_t lo = 0xffffffffu, hi = 0u;
    QCF_FOR_KEYS(i, { const uint32_t key = QCF_KEY(i); lo = min(lo, key); hi = max(hi, key); })
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
      hi = max(hi, (uint32_t)__shfl_xor((int)hi, d, 64));
    }
    if (lane == 0) { red_lo[wave] = lo; red_hi[wave] = hi; }
    for (int i = tid; i < kBins; i += kThreads) merged[i] = 0u;
    __syncthreads();
    lo = red_lo[0]; hi = red_hi[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) { lo = min(lo, red_lo[w]); hi = max(hi, red_hi[w]); }

    const uint32_t diff = lo ^ hi;
    int bits = diff ? 32 - __clz((int)diff) : 0;     // low bits in which keys may differ
    uint32_t prefix = (bits >= 32) ? 0u : (hi >> bits);   // common high part
    while (bits > 0) {
      const int w = min(kDigitBits, bits);
      const int shift = bits - w;
      const uint32_t mask = (1u << w) - 1u;
      // (merged[] was cleared before the loop and is cleared again by wave 0 after each pass)
      QCF_FOR_KEYS(i, {
        const uint32_t key = QCF_KEY(i);
        const uint32_t high = (bits >= 32) ? 0u : (key >> bits);
        if (high == prefix) atomicAdd(&merged[(key >> shift) & mask], 1u);
      })
      __syncthreads();
      if (wave == 0) {
        uint32_t c[kBinsPerLane];
        uint32_t tot = 0;
#pragma unroll
        for (int q = 0; q < kBinsPerLane; ++q) {
          c[q] = merged[kBinsPerLane * lane + q];
          tot += c[q];
          merged[kBinsPerLane * lane + q] = 0u;
        }
        uint32_t suffix = tot;               // sum over lanes >= this one
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const uint32_t o = __shfl_down(suffix, d, 64);
          if (lane + d < 64) suffix += o;
        }
        uint32_t above = suffix - tot;       // keys with a larger digit than this lane's bins
#pragma unroll
        for (int q = kBinsPerLane - 1; q >= 0; --q) {
          if (above < k && k <= above + c[q]) { s_digit = kBinsPerLane * lane + q; s_k = k - above; }
          above += c[q];
        }
      }
      __syncthreads();
      prefix = (prefix << w) | s_digit;
      k = s_k;
      bits = shift;
    }
    tau = prefix;
  }

  // compaction in index order
  uint32_t n_gt = 0, n_eq = 0;
  if (N < T) {
    QCF_FOR_KEYS(i, { const uint32_t key = QCF_KEY(i); n_gt += key > tau; n_eq += key == tau; })
  } else {
    n_gt = (uint32_t)cnt;
  }
  const uint64_t mine = ((uint64_t)n_eq << 32) | n_gt;
  const uint64_t incl = wave_incl_scan(mine, lane);
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint64_t before = incl - mine;
  for (int w = 0; w < wave; ++w) before += wave_tot[w];
  uint32_t gt_before = (uint32_t)before, eq_before = (uint32_t)(before >> 32);
  const int64_t out0 = o0;
#define QCF_EMIT(j, pos)                                            \
  {                                                                 \
    sel_idx[out0 + (pos)] = (j);                                    \
    if (sel_row) sel_row[out0 + (pos)] = (int32_t)(c0 + (j));       \
    if (sel_pos) sel_pos[out0 + (pos)] = base_pos + (j);            \
  }
  if (N < T) {
    QCF_FOR_KEYS(i, {
      const uint32_t key = QCF_KEY(i);
      const bool gt = key > tau, eq = key == tau;
      const uint32_t pos = gt_before + min(eq_before, k);
      if ((gt || (eq && eq_before < k)) && pos < (uint32_t)N) QCF_EMIT(j0 + i, pos)
      gt_before += gt;
      eq_before += eq;
    })
  } else {
    for (int i = 0; i < cnt; ++i) QCF_EMIT(j0 + i, gt_before + i)
  }
#undef QCF_EMIT
#undef QCF_KEY
#undef QCF_FOR_KEYS
}

}  // namespace

size_t select_workspace(int32_t, int64_t) { return 0; }

qcf_status launch_select(int32_t B, const float* score, const int64_t* ctx_off, int64_t total_ctx,
                         const int64_t* sel_off, int64_t total_sel, const int32_t* ctx_pos0,
                         int32_t* sel_idx, int32_t* sel_row, int32_t* sel_pos, void*, hipStream_t st) {
  const dim3 grid((unsigned)B), block(kThreads);
  // a request is never longer than total_ctx, which bounds the per-thread segment
  if (total_ctx <= 8 * kThreads)
    select_kernel<8><<<grid, block, 0, st>>>(score, ctx_off, total_ctx, sel_off, total_sel, ctx_pos0,
                                             sel_idx, sel_row, sel_pos);
  else if (total_ctx <= 32 * kThreads)
    select_kernel<32><<<grid, block, 0, st>>>(score, ctx_off, total_ctx, sel_off, total_sel, ctx_pos0,
                                              sel_idx, sel_row, sel_pos);
  else
    select_kernel<0><<<grid, block, 0, st>>>(score, ctx_off, total_ctx, sel_off, total_sel, ctx_pos0,
                                             sel_idx, sel_row, sel_pos);
  return check_launch("select");
}

}  // namespace qcf
