// Step 4: recompute Q/K/V of the selected tokens (Section 3.1 Phase 4 of the paper):
// [Q|K|V] = X_sel W_qkv^T, rotary embedding on Q and K at the tokens' absolute positions.
//
// The bf16 path is a 32x32x16-MFMA GEMM (both operands are contiguous along the contraction
// dimension) with a ring of LDS stages; an output tile is 128 columns wide, i.e. whole heads, so
// the rotary partner of every element is inside the tile and the embedding is applied in the
// epilogue, which forms the rotation itself: the angle pos * theta_i is taken in turns, with the
// frequency split in two floats and the product's rounding error recovered by a fused
// multiply-add (a plain float32 product would be off by 1e-3 rad at 8K positions), reduced to its
// fraction and handed to the hardware sine and cosine (inputs in turns, errors far below a bf16
// ulp).  Positions of 2^24 and more take the same steps in float64.
// The generic path (f32, or shapes the MFMA tiling does not cover) writes the raw product to
// the workspace and rotates it in a second kernel with a (cos, sin) table built from float64
// angles by a small table kernel.
// qcf_recompute_qkv_scatter: the epilogue of the MFMA path also stores the K and V rows to their rows of the
// fused cache (step 5 of the path, otherwise a kernel of its own).
#include <type_traits>
#include <utility>

#include "qcf_internal.h"

namespace qcf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ------------------------------------------------------------------ rotary table

__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t* __restrict__ pos, int64_t M, int D,
                                                         double neg2_over_d_log2base,
                                                         float2* __restrict__ cs) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int half = D / 2;
  if (gid >= M * half) return;
  const int64_t m = gid / half;
  const int i = (int)(gid - m * half);
  const double theta = exp2(neg2_over_d_log2base * (double)i);
  double sn, cn;
  sincos((double)pos[m] * theta, &sn, &cn);
  cs[gid] = make_float2((float)cn, (float)sn);
}

// ------------------------------------------------------------------ generic path

template <typename T>
__global__ __launch_bounds__(256) void qkv_gemm_generic(const T* __restrict__ x, int64_t x_rows,
                                                        const int32_t* __restrict__ gather, int64_t M,
                                                        const T* __restrict__ w, int Kdim, int Ntot,
                                                        float* __restrict__ y) {
  __shared__ float sA[16][65];
  __shared__ float sB[16][65];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int64_t m0 = (int64_t)blockIdx.x * 64;
  const int n0 = blockIdx.y * 64;
  float acc[4][4] = {};
  const int lr = tid >> 2;            // 0..63: tile row loaded by this thread
  const int lc = (tid & 3) * 4;       // 0,4,8,12: first k of its 4 elements
  int64_t arow = -1;
  if (m0 + lr < M) {
    const int64_t idx = gather ? (int64_t)gather[m0 + lr] : m0 + lr;
    if (idx >= 0 && idx < x_rows) arow = idx;
  }
  const int brow = (n0 + lr < Ntot) ? n0 + lr : -1;
  for (int k0 = 0; k0 < Kdim; k0 += 16) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int kk = k0 + lc + c;
      sA[lc + c][lr] = (arow >= 0 && kk < Kdim) ? Elem<T>::load(x + arow * Kdim + kk) : 0.f;
      sB[lc + c][lr] = (brow >= 0 && kk < Kdim) ? Elem<T>::load(w + (int64_t)brow * Kdim + kk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = sA[kk][ty * 4 + i]; bv[i] = sB[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < Ntot) y[m * Ntot + n] = acc[i][j];
    }
  }
}

// one thread per (row, head slot, rotary pair); V heads are copied
template <typename T>
__global__ __launch_bounds__(256) void qkv_rope_split_generic(const float* __restrict__ y, int64_t M,
                                                              const float2* __restrict__ cs, int H, int Hkv,
                                                              int D, int style, T* __restrict__ q,
                                                              T* __restrict__ k, T* __restrict__ v) {
  const int half = D / 2;
  const int heads = H + 2 * Hkv;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= M * heads * half) return;
  const int i = (int)(gid % half);
  const int hs = (int)((gid / half) % heads);
  const int64_t m = gid / ((int64_t)half * heads);
  const int ia = style == 0 ? i : 2 * i;
  const int ib = style == 0 ? i + half : 2 * i + 1;
  const float* src = y + m * (int64_t)heads * D + (int64_t)hs * D;
  const float a = src[ia], b = src[ib];
  T* dst;
  bool rot = true;
  if (hs < H) dst = q ? q + (m * H + hs) * D : nullptr;
  else if (hs < H + Hkv) dst = k ? k + (m * Hkv + (hs - H)) * D : nullptr;
  else { dst = v ? v + (m * Hkv + (hs - H - Hkv)) * D : nullptr; rot = false; }
  if (!dst) return;
  if (rot) {
    const float2 w = cs[m * half + i];
    Elem<T>::store(dst + ia, a * w.x - b * w.y);
    Elem<T>::store(dst + ib, b * w.x + a * w.y);
  } else {
    Elem<T>::store(dst + ia, a);
    Elem<T>::store(dst + ib, b);
  }
}

// out = y (+ residual), stored in the element type (generic path of the plain linear map)
template <typename T>
__global__ __launch_bounds__(256) void linear_finish_generic(const float* __restrict__ y, const T* residual,
                                                             int64_t n, T* out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float v = y[i];
  if (residual) v += Elem<T>::load(residual + i);
  Elem<T>::store(out + i, v);
}

// ------------------------------------------------------------------ RMSNorm and gated SiLU (HBM bound)

// One workgroup per row: every thread keeps its 16-byte vectors of the row in registers (up to kNormVecs),
// the sum of squares goes through the waves and LDS in a fixed order, then the row is scaled and stored.
constexpr int kNormVecs = 4;
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T* x, const T* __restrict__ weight, float eps, int cols,
                                                      T* out) {
  constexpr int VEC = Elem<T>::kVec;
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x;
  const T* xr = x + row * cols;
  const int n_vec = cols / VEC;
  u32x4 raw[kNormVecs];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < kNormVecs; ++i) {
    const int v = tid + i * 256;
    if (v < n_vec) {
      raw[i] = *reinterpret_cast<const u32x4*>(xr + v * VEC);
      float f[VEC];
      Vec16<T>::unpack(raw[i], f);
#pragma unroll
      for (int e = 0; e < VEC; ++e) ss += f[e] * f[e];
    }
  }
  for (int v = tid + kNormVecs * 256; v < n_vec; v += 256) {       // longer rows: the tail is read twice
    float f[VEC];
    Vec16<T>::unpack(*reinterpret_cast<const u32x4*>(xr + v * VEC), f);
#pragma unroll
    for (int e = 0; e < VEC; ++e) ss += f[e] * f[e];
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) ss += __shfl_xor(ss, d, 64);
  if (lane == 0) red[wave] = ss;
  __syncthreads();
  const float scale = rsqrtf(((red[0] + red[1]) + (red[2] + red[3])) / (float)cols + eps);
  T* orow = out + row * cols;
  auto emit = [&](int v, const u32x4& r) {
    float f[VEC], g[VEC];
    Vec16<T>::unpack(r, f);
    Vec16<T>::unpack(*reinterpret_cast<const u32x4*>(weight + v * VEC), g);
#pragma unroll
    for (int e = 0; e < VEC; ++e) f[e] = f[e] * scale * g[e];
    *reinterpret_cast<u32x4*>(orow + v * VEC) = Vec16<T>::pack(f);
  };
#pragma unroll
  for (int i = 0; i < kNormVecs; ++i) {
    const int v = tid + i * 256;
    if (v < n_vec) emit(v, raw[i]);
  }
  for (int v = tid + kNormVecs * 256; v < n_vec; v += 256) emit(v, *reinterpret_cast<const u32x4*>(xr + v * VEC));
}

// out[m, f] = silu(gate_up[m, f]) * gate_up[m, F + f]; one 16-byte output vector per thread
template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const T* __restrict__ gate_up, int64_t M, int F,
                                                     T* __restrict__ out) {
  constexpr int VEC = Elem<T>::kVec;
  const int per_row = F / VEC;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= M * per_row) return;
  const int64_t m = i / per_row;
  const int c = (int)(i - m * per_row) * VEC;
  float g[VEC], u[VEC];
  Vec16<T>::unpack(*reinterpret_cast<const u32x4*>(gate_up + m * 2 * F + c), g);
  Vec16<T>::unpack(*reinterpret_cast<const u32x4*>(gate_up + m * 2 * F + F + c), u);
#pragma unroll
  for (int e = 0; e < VEC; ++e) g[e] = g[e] / (1.f + __expf(-g[e])) * u[e];
  *reinterpret_cast<u32x4*>(out + m * F + c) = Vec16<T>::pack(g);
}

// ------------------------------------------------------------------ MFMA path (bf16)

constexpr int kBK = 64;                  // contraction elements per LDS stage (rows of 128 bytes)
constexpr int kBN = 128;                 // output columns per workgroup (whole heads)
constexpr int kCStride = kBN + 8;        // floats per row of the epilogue tile (rows 4 apart: 32 banks apart)
constexpr int kStages = 3;               // ring of LDS stages filled by asynchronous loads
constexpr size_t kRhoBytes = 64 * sizeof(float2);   // theta_i / (2 pi) of up to 64 rotary pairs, as (high, low) floats

struct QkvArgs {
  const bf16_t* x;
  const bf16_t* w;
  const int32_t* gather;
  const int32_t* pos;            // [M] absolute positions (rotary embedding; unused by the plain linear map)
  double neg2_over_d_log2base;   // theta_i = 2^(i * this)
  int64_t x_rows, M;
  int d_model, H, Hkv, D;
  int m_tiles, n_tiles;
  bf16_t* q;
  bf16_t* k;
  bf16_t* v;
  // plain linear map (qcf_linear): all H*D columns go to q without rotation; residual (may be NULL) is added
  int plain;
  const bf16_t* residual;
  // projection fused with the write-back: row m of the K and V tiles also goes to row dst_rows[m] of the fused
  // cache (rows outside [0, fused_rows) are skipped); all null / 0 otherwise
  int rows_over_xcds;            // workgroup order of the specialised kernel (see there)
  const int32_t* dst_rows;
  bf16_t* k_fused;
  bf16_t* v_fused;
  int64_t fused_rows;
};

template <int TM, int TN, int WGM, int WGN>
struct Tile {
  static constexpr int BM = 32 * TM * WGM;
  static constexpr int NTHR = 64 * WGM * WGN;
  static constexpr int NWAVE = WGM * WGN;
  static constexpr int A_LD = BM / 8 / NWAVE;             // 1 KB load instructions per wave and stage
  static constexpr int B_LD = kBN / 8 / NWAVE;
  static constexpr int STAGE = (BM + kBN) * kBK * 2;      // bytes per stage
  static constexpr size_t LDS_MAIN = (size_t)kStages * STAGE;
  static constexpr size_t LDS_EPI = (size_t)BM * kCStride * 4;
  static constexpr size_t RHO = LDS_MAIN > LDS_EPI ? LDS_MAIN : LDS_EPI;      // rotary frequencies (64 doubles) sit behind both
  static constexpr size_t LDS = RHO + kRhoBytes;
  static_assert(32 * TN * WGN == kBN, "a workgroup covers 128 output columns");
  static_assert((BM / 8) % NWAVE == 0 && (kBN / 8) % NWAVE == 0, "load split");
};

// Where a 128-column tile of the fused projection goes.
struct OutTile {
  bf16_t* out;
  bf16_t* fused;          // second destination, addressed through dst_rows (K and V tiles of the fused call)
  int out_cols, out_col0;
  bool rotate;
};
__device__ __forceinline__ OutTile out_tile_of(const QkvArgs& a, int col0) {
  const int q_cols = a.H * a.D, kv_cols = a.Hkv * a.D;
  OutTile o;
  o.rotate = !a.plain;
  o.fused = nullptr;
  if (col0 < q_cols) { o.out = a.q; o.out_cols = q_cols; o.out_col0 = col0; }
  else if (col0 < q_cols + kv_cols) { o.out = a.k; o.fused = a.k_fused; o.out_cols = kv_cols; o.out_col0 = col0 - q_cols; }
  else { o.out = a.v; o.fused = a.v_fused; o.out_cols = kv_cols; o.out_col0 = col0 - q_cols - kv_cols; o.rotate = false; }
  return o;
}

// Epilogue, first half: a wave drops its accumulators (32*TM rows from row_base, 32*TN columns from
// col_base) into the fp32 tile in LDS.
template <int TM, int TN>
__device__ __forceinline__ void acc_to_lds(float* sC, const floatx16 (&acc)[TM][TN], int row_base, int col_base,
                                           int lane) {
  const int hf = lane >> 5, l32 = lane & 31;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = row_base + i * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
        const int c = col_base + j * 32 + l32;
        sC[r * kCStride + c] = acc[i][j][v];
      }
}

// Rotary frequencies in turns per position, theta_i / (2 pi) = 2^(i * c) / (2 pi), for the d/2 pairs of a head:
// computed in float64 and kept as two floats, high + low (written by 64 threads before the barrier that precedes
// store_tile).
__device__ __forceinline__ void fill_rho(const QkvArgs& a, float2* sRho, int i) {
  if (i < a.D / 2) {
    const double rho = exp2(a.neg2_over_d_log2base * (double)i) * 0.15915494309189535;
    const float hi = (float)rho;
    sRho[i] = make_float2(hi, (float)(rho - (double)hi));
  }
}
// (cos, sin) of pos * theta for one pair.  The angle in turns is p * (hi + lo): the product p * hi is rounded, its
// error is exact in an FMA, and only the fraction of the rounded part matters, so the sum below is good to about
// 1e-7 of a turn for positions below 2^24 (exactly representable in a float).
__device__ __forceinline__ void rotary_factor(int32_t pos, float2 rho, float& c, float& sn) {
#pragma clang fp contract(off)          // the rounded product and its error term must stay two operations
  float fr;
  if (pos > -(1 << 24) && pos < (1 << 24)) {
    const float pf = (float)pos;
    const float t_hi = pf * rho.x;
    const float t_lo = __builtin_fmaf(pf, rho.y, __builtin_fmaf(pf, rho.x, -t_hi));
    fr = (t_hi - floorf(t_hi)) + t_lo;
  } else {
    const double turns = (double)pos * ((double)rho.x + (double)rho.y);
    fr = (float)(turns - floor(turns));
  }
  c = __builtin_amdgcn_cosf(fr);
  sn = __builtin_amdgcn_sinf(fr);
}

// Epilogue, second half (after a barrier): each thread takes the same 16 columns (8 rotary pairs) of
// BM*8/NTHR rows.  It first requests the gather indices and rotary factors of all its rows, then rotates
// and stores two 16-byte vectors per row.
// Column task tk (0..7) of a 128-column tile: 16 columns = 8 rotary pairs.  e0 / e1: first column of the two
// 8-column pieces; i0: index of the first pair inside its head.
template <int STYLE>
__device__ __forceinline__ void column_task(const QkvArgs& a, int tk, int& e0, int& e1, int& i0) {
  if (STYLE == 0) {
    const int per_head = a.D / 16;                     // tasks per head
    const int hd = tk / per_head;
    i0 = (tk - hd * per_head) * 8;
    e0 = hd * a.D + i0;
    e1 = e0 + a.D / 2;
  } else {
    e0 = tk * 16;
    e1 = e0 + 8;
    i0 = (e0 % a.D) / 2;
  }
}

template <int BM, int NTHR, int STYLE>
__device__ __forceinline__ void store_tile(const QkvArgs& a, const float* sC, const float2* sRho, int64_t m0,
                                           const OutTile& ot, int tid) {
  constexpr int NT = BM * 8 / NTHR;                    // rows per thread
  constexpr int RSTEP = NTHR / 8;                      // row distance between a thread's tasks
  static_assert(BM * 8 % NTHR == 0, "rows per thread");
  const int tk = tid & 7, r0 = tid >> 3;
  int e0, e1, i0;
  column_task<STYLE>(a, tk, e0, e1, i0);
  bool zero[NT];
  int32_t posv[NT];
  int64_t fdst[NT];                                    // row of the fused cache (-1: none)
  u32x4 w4[NT][2];                                     // the row's 16 residual values
  float2 rho[8];                                       // frequencies of this thread's 8 pairs, in turns per position
  if (ot.rotate) {
#pragma unroll
    for (int p = 0; p < 8; ++p) rho[p] = sRho[i0 + p];
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int64_t m = m0 + r0 + t * RSTEP;
    zero[t] = false;
    posv[t] = 0;
    fdst[t] = -1;
    if (m < a.M) {
      if (ot.fused) {
        const int64_t d = a.dst_rows[m];
        if (d >= 0 && d < a.fused_rows) fdst[t] = d;
      }
      if (a.gather) {                                  // an index outside x produces a zero row
        const int64_t idx = a.gather[m];
        zero[t] = idx < 0 || idx >= a.x_rows;
      }
      if (ot.rotate) {
        posv[t] = a.pos[m];
      } else if (a.residual) {
        const bf16_t* res = a.residual + m * ot.out_cols + ot.out_col0;
        w4[t][0] = *reinterpret_cast<const u32x4*>(res + e0);
        w4[t][1] = *reinterpret_cast<const u32x4*>(res + e1);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int r = r0 + t * RSTEP;
    const int64_t m = m0 + r;
    if (m >= a.M) continue;
    float f[16], o[16];
    const float* row = sC + r * kCStride;
    {
      const u32x4 c0 = *reinterpret_cast<const u32x4*>(row + e0), c1 = *reinterpret_cast<const u32x4*>(row + e0 + 4);
      const u32x4 c2 = *reinterpret_cast<const u32x4*>(row + e1), c3 = *reinterpret_cast<const u32x4*>(row + e1 + 4);
      Vec16<float>::unpack(c0, f); Vec16<float>::unpack(c1, f + 4);
      Vec16<float>::unpack(c2, f + 8); Vec16<float>::unpack(c3, f + 12);
    }
    if (zero[t]) {
#pragma unroll
      for (int p = 0; p < 16; ++p) f[p] = 0.f;
    }
    if (ot.rotate) {
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        float wx, wy;
        rotary_factor(posv[t], rho[p], wx, wy);
        const int ia = (STYLE == 0) ? p : 2 * p;
        const int ib = (STYLE == 0) ? p + 8 : 2 * p + 1;
        o[ia] = f[ia] * wx - f[ib] * wy;
        o[ib] = f[ib] * wx + f[ia] * wy;
      }
    } else if (a.residual) {
      float res[16];
      Vec16<bf16_t>::unpack(w4[t][0], res);
      Vec16<bf16_t>::unpack(w4[t][1], res + 8);
#pragma unroll
      for (int p = 0; p < 16; ++p) o[p] = f[p] + res[p];
    } else {
#pragma unroll
      for (int p = 0; p < 16; ++p) o[p] = f[p];
    }
    const u32x4 lo16 = Vec16<bf16_t>::pack(o), hi16 = Vec16<bf16_t>::pack(o + 8);
    bf16_t* dst = ot.out + m * ot.out_cols + ot.out_col0;
    *reinterpret_cast<u32x4*>(dst + e0) = lo16;
    *reinterpret_cast<u32x4*>(dst + e1) = hi16;
    if (fdst[t] >= 0) {
      bf16_t* fd = ot.fused + fdst[t] * ot.out_cols + ot.out_col0;
      *reinterpret_cast<u32x4*>(fd + e0) = lo16;
      *reinterpret_cast<u32x4*>(fd + e1) = hi16;
    }
  }
}

// Staged tiles have rows of 128 bytes (8 chunks of 16 bytes) without padding; chunk c of row r sits in
// slot c ^ ((r / 2) % 8), so the 16-byte fragment reads of 16 consecutive rows touch 16 different bank
// groups.  One load instruction of a wave fills 8 rows (1 KB): lane L fills slot L%8 of row L/8.
template <int TM, int TN, int WGM, int WGN, int STYLE>
__global__ __launch_bounds__(64 * WGM * WGN) void qkv_mfma_kernel(QkvArgs a) {
  using C = Tile<TM, TN, WGM, WGN>;
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int hf = lane >> 5, l32 = lane & 31;
  // consecutive workgroup ids land on different XCDs: all row tiles of a column tile share an XCD, so
  // the weight tile is fetched into one L2 only
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int m_tile = slot % a.m_tiles, n_tile = (slot / a.m_tiles) * 8 + xcd;
  if (n_tile >= a.n_tiles) return;
  const int64_t m0 = (int64_t)m_tile * C::BM;
  const int col0 = n_tile * kBN;

  const OutTile ot = out_tile_of(a, col0);
  if (!ot.out) return;

  // load instruction i of this wave covers tile rows 8*(wave + NWAVE*i) .. +7
  const int ld_r = lane >> 3;                                    // row inside the 8-row group
  const bf16_t* a_src[C::A_LD];                                  // per-lane source of chunk (lane%8)^swz at k = 0
#pragma unroll
  for (int i = 0; i < C::A_LD; ++i) {
    const int row = 8 * (wave + C::NWAVE * i) + ld_r;
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    const int64_t m = m0 + row;
    int64_t idx = 0;                                             // rows past M read row 0; never stored
    if (m < a.M) {
      idx = a.gather ? (int64_t)a.gather[m] : m;
      if (idx < 0 || idx >= a.x_rows) idx = 0;                   // stored as zeros in the epilogue
    }
    a_src[i] = a.x + idx * a.d_model + chunk * 8;
  }
  uint32_t b_off[C::B_LD];                                       // byte offset from w + col0 * d_model
#pragma unroll
  for (int i = 0; i < C::B_LD; ++i) {
    const int row = 8 * (wave + C::NWAVE * i) + ld_r;
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    b_off[i] = (uint32_t)row * (uint32_t)a.d_model * 2u + (uint32_t)chunk * 16u;
  }
  const char* b_base = reinterpret_cast<const char*>(a.w + (int64_t)col0 * a.d_model);
  auto issue = [&](int kt, int st) {
    unsigned char* sA = smem + (size_t)st * C::STAGE;
    unsigned char* sB = sA + C::BM * kBK * 2;
#pragma unroll
    for (int i = 0; i < C::A_LD; ++i) load_to_lds_addr(a_src[i] + (int64_t)kt * kBK, sA + (wave + C::NWAVE * i) * 1024);
#pragma unroll
    for (int i = 0; i < C::B_LD; ++i)
      load_to_lds(b_base + (int64_t)kt * kBK * 2, b_off[i], sB + (wave + C::NWAVE * i) * 1024);
  };

  // the same loads split in four parts (part p issues every 4th instruction), so that they can be spread
  // between the MFMAs of a k-tile
  auto issue_part = [&](int kt, int st, int part) {
    unsigned char* sA = smem + (size_t)st * C::STAGE;
    unsigned char* sB = sA + C::BM * kBK * 2;
#pragma unroll
    for (int i = 0; i < C::A_LD; ++i)
      if ((i & 3) == part) load_to_lds_addr_nf(a_src[i] + (int64_t)kt * kBK, sA + (wave + C::NWAVE * i) * 1024);
#pragma unroll
    for (int i = 0; i < C::B_LD; ++i)
      if ((i & 3) == part) load_to_lds_nf(b_base + (int64_t)kt * kBK * 2, b_off[i], sB + (wave + C::NWAVE * i) * 1024);
  };

  // fragment addresses inside a stage: row (32-row tile base + l32), chunk 2*ks + hf in slot
  // (2*ks + hf) ^ ((l32 / 2) % 8); the address of step ks is base ^ (32 * ks)
  const int swz = (l32 >> 1) & 7;
  const int fb0 = l32 * 128 + ((hf ^ (swz & 1)) * 16) + ((swz & 6) * 16);
  const int a_frag = wm * 32 * TM * 128 + fb0;
  const int b_frag = C::BM * kBK * 2 + wn * 32 * TN * 128 + fb0;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = floatx16{0};

  const int nk = a.d_model / kBK;
  issue(0, 0);
  if (nk > 1) issue(1, 1);
  for (int kt = 0; kt < nk; ++kt) {
    // every wave has at most two stages of its own loads in flight; wait for the older one
    if (kt + 1 < nk) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::A_LD + C::B_LD) : "memory");
    else __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                       // stage kt%3 is complete; stage (kt+2)%3 is free again
    const bool more = kt + 2 < nk;
    const int st_next = (kt + 2) % kStages;
    const unsigned char* stage = smem + (size_t)(kt % kStages) * C::STAGE;
    // fragments of step ks+1 are requested before the MFMAs of step ks are issued
    u32x4 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = *reinterpret_cast<const u32x4*>(stage + (a_frag + i * 32 * 128));
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = *reinterpret_cast<const u32x4*>(stage + (b_frag + j * 32 * 128));
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      if (ks + 1 < kBK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[(ks + 1) & 1][i] = *reinterpret_cast<const u32x4*>(stage + ((a_frag + i * 32 * 128) ^ (32 * (ks + 1))));
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[(ks + 1) & 1][j] = *reinterpret_cast<const u32x4*>(stage + ((b_frag + j * 32 * 128) ^ (32 * (ks + 1))));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        // a quarter of the next-but-one stage per k-step, requested while the matrix unit is busy
        if (i == TM / 2 && more) issue_part(kt + 2, st_next, ks);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[ks & 1][i]),
                                                               __builtin_bit_cast(bf16x8, bfr[ks & 1][j]), acc[i][j], 0, 0, 0);
      }
    }
  }
  __syncthreads();                         // all fragment reads done before the epilogue reuses the LDS

  // epilogue: the whole BM x 128 tile goes through LDS as fp32 (it fits in the ring's space)
  float* sC = reinterpret_cast<float*>(smem);
  float2* sRho = reinterpret_cast<float2*>(smem + C::RHO);
  if (ot.rotate && tid < 64) fill_rho(a, sRho, tid);
  acc_to_lds<TM, TN>(sC, acc, wm * 32 * TM, wn * 32 * TN, lane);
  __syncthreads();
  store_tile<C::BM, C::NTHR, STYLE>(a, sC, sRho, m0, ot, tid);
}

// ---- specialised variant for 256-row tiles (TM = 2) and 128-row tiles (TM = 1) ----------------------
// Four compute waves (one per SIMD, 32*TM x 128 outputs each) issue only fragment reads and MFMAs; four more
// waves only issue the asynchronous global-to-LDS loads.  A wave that issues such a load can stall on the
// memory pipeline's queue, and a stalled wave issues no MFMAs either: with the two roles in different
// waves the matrix unit keeps running meanwhile.
//
// Synchronisation, one barrier per k-tile (barrier number kt + 1 is crossed while tile kt is computed):
//   compute wave: steps 0..2 of tile kt, wait for its last fragment reads of stage kt%3, barrier,
//                 request the first fragments of tile kt+1, step 3 of tile kt;
//   load wave:    after barrier kt it requests tile kt+2 into stage (kt+2)%3 == (kt-1)%3 (free: every
//                 compute wave finished reading tile kt-1 before barrier kt), waits until its loads of
//                 tile kt+1 have landed, barrier.
template <int TM_>
struct WsTile {
  static constexpr int TM = TM_, TN = 4, NC = 4, NL = 4;          // compute waves stacked along M
  static constexpr int BM = 32 * TM * NC;                         // 256 (TM = 2) or 128 (TM = 1)
  static constexpr int NTHR = 64 * (NC + NL);
  static constexpr int A_LD = BM / 8 / NL;                        // 1 KB load instructions per load wave and stage
  static constexpr int B_LD = kBN / 8 / NL;
  static constexpr int STAGE = (BM + kBN) * kBK * 2;
  static constexpr size_t LDS_MAIN = (size_t)kStages * STAGE;
  static constexpr size_t LDS_EPI = (size_t)BM * kCStride * 4;
  static constexpr size_t RHO = LDS_MAIN > LDS_EPI ? LDS_MAIN : LDS_EPI;
  static constexpr size_t LDS = RHO + kRhoBytes;
  static_assert(32 * TN == kBN, "a compute wave covers the 128 output columns");
};

template <int TM_, int STYLE>
__global__ __launch_bounds__(WsTile<TM_>::NTHR) void qkv_ws_kernel(QkvArgs a) {
  using C = WsTile<TM_>;
  constexpr int TM = C::TM, TN = C::TN;
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hf = lane >> 5, l32 = lane & 31;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;        // same workgroup order as above
  int m_tile = slot % a.m_tiles, n_tile = (slot / a.m_tiles) * 8 + xcd;
  if (a.rows_over_xcds) {          // many row tiles: row tiles are dealt to the XCDs, column tiles run side by side
    m_tile = (slot / a.n_tiles) * 8 + xcd;
    n_tile = slot % a.n_tiles;
  }
  if (n_tile >= a.n_tiles || m_tile >= a.m_tiles) return;
  const int64_t m0 = (int64_t)m_tile * C::BM;
  const int col0 = n_tile * kBN;
  const OutTile ot = out_tile_of(a, col0);
  if (!ot.out) return;
  const int nk = a.d_model / kBK;
  float* sC = reinterpret_cast<float*>(smem);
  float2* sRho = reinterpret_cast<float2*>(smem + C::RHO);

  if (wave >= C::NC) {
    // ---------------- load wave lw: instruction i covers tile rows 8*(lw + NL*i) .. +7
    const int lw = wave - C::NC;
    const int ld_r = lane >> 3;
    uint32_t a_off[C::A_LD];                                     // byte offset from x (x is below 4 GiB here)
#pragma unroll
    for (int i = 0; i < C::A_LD; ++i) {
      const int row = 8 * (lw + C::NL * i) + ld_r;
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      const int64_t m = m0 + row;
      int64_t idx = 0;                                           // rows past M read row 0; never stored
      if (m < a.M) {
        idx = a.gather ? (int64_t)a.gather[m] : m;
        if (idx < 0 || idx >= a.x_rows) idx = 0;                 // stored as zeros in the epilogue
      }
      a_off[i] = (uint32_t)idx * (uint32_t)a.d_model * 2u + (uint32_t)chunk * 16u;
    }
    const char* a_base = reinterpret_cast<const char*>(a.x);
    uint32_t b_off[C::B_LD];
#pragma unroll
    for (int i = 0; i < C::B_LD; ++i) {
      const int row = 8 * (lw + C::NL * i) + ld_r;
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      b_off[i] = (uint32_t)row * (uint32_t)a.d_model * 2u + (uint32_t)chunk * 16u;
    }
    const char* b_base = reinterpret_cast<const char*>(a.w + (int64_t)col0 * a.d_model);
    auto issue = [&](int kt) {
      unsigned char* sA = smem + (size_t)(kt % kStages) * C::STAGE;
      unsigned char* sB = sA + C::BM * kBK * 2;
#pragma unroll
      for (int i = 0; i < C::B_LD; ++i)
        load_to_lds(b_base + (int64_t)kt * kBK * 2, b_off[i], sB + (lw + C::NL * i) * 1024);
#pragma unroll
      for (int i = 0; i < C::A_LD; ++i)
        load_to_lds(a_base + (int64_t)kt * kBK * 2, a_off[i], sA + (lw + C::NL * i) * 1024);
    };
    issue(0);
    if (nk > 1) {
      issue(1);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::A_LD + C::B_LD) : "memory");
    } else {
      __builtin_amdgcn_s_waitcnt(0);
    }
    __syncthreads();                                             // barrier 0: tile 0 has landed
    for (int kt = 0; kt < nk; ++kt) {
      if (kt + 2 < nk) {
        issue(kt + 2);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::A_LD + C::B_LD) : "memory");
      } else {
        __builtin_amdgcn_s_waitcnt(0);
      }
      __syncthreads();                                           // barrier kt + 1: tile kt + 1 has landed
    }
    if (ot.rotate && lw == 0) fill_rho(a, sRho, lane);           // (behind the ring: no stage is touched)
    __syncthreads();                                             // the accumulators are in LDS
  } else {
    // ---------------- compute wave: rows 64*wave .. +63 of the tile, all 128 columns
    __builtin_amdgcn_s_setprio(2);                               // its instructions go first when both roles are ready
    const int swz = (l32 >> 1) & 7;
    const int fb0 = l32 * 128 + ((hf ^ (swz & 1)) * 16) + ((swz & 6) * 16);
    const int a_frag = wave * 32 * TM * 128 + fb0;
    const int b_frag = C::BM * kBK * 2 + fb0;
    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = floatx16{0};
    u32x4 af[2][TM], bfr[2][TN];
    auto fetch = [&](const unsigned char* stage, int ks, int buf) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[buf][i] = *reinterpret_cast<const u32x4*>(stage + ((a_frag + i * 32 * 128) ^ (32 * ks)));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[buf][j] = *reinterpret_cast<const u32x4*>(stage + ((b_frag + j * 32 * 128) ^ (32 * ks)));
    };
    auto mfmas = [&](int buf) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[buf][i]),
                                                               __builtin_bit_cast(bf16x8, bfr[buf][j]), acc[i][j], 0, 0, 0);
    };
    // issue order of one k-step: every fragment read sits behind an MFMA, so that the matrix unit is
    // already busy while the read is issued
    auto interleave = [&]() {
      constexpr int kPairs = TM * TN < TM + TN ? TM * TN : TM + TN;
#pragma unroll
      for (int q = 0; q < kPairs; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);       // one LDS read
      }
      if (TM * TN > kPairs) __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - kPairs, 0);
      if (TM + TN > kPairs) __builtin_amdgcn_sched_group_barrier(0x100, TM + TN - kPairs, 0);
    };
    __syncthreads();                                             // barrier 0
    fetch(smem, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
      const unsigned char* stage = smem + (size_t)(kt % kStages) * C::STAGE;
#pragma unroll
      for (int ks = 0; ks < 3; ++ks) {
        fetch(stage, ks + 1, (ks + 1) & 1);
        mfmas(ks & 1);
        interleave();
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");         // the last fragments of this stage are in registers
      __syncthreads();                                           // barrier kt + 1
      // (after the last tile this re-reads the current stage; the values are not used)
      fetch(smem + (size_t)((kt + 1 < nk ? kt + 1 : kt) % kStages) * C::STAGE, 0, 0);
      mfmas(1);
      interleave();
    }
    __builtin_amdgcn_s_setprio(0);
    acc_to_lds<TM, TN>(sC, acc, wave * 32 * TM, 0, lane);
    __syncthreads();
  }
  store_tile<C::BM, C::NTHR, STYLE>(a, sC, sRho, m0, ot, tid);
}

// 256-row or 128-row tiles (both load/compute-split)?  Both run one workgroup per compute unit, so
// the launch takes (rounds of workgroups) x (time of one workgroup); the per-k-tile and fixed costs are the
// measured ones of the two kernels on MI355X (microseconds).
bool prefer_256_rows(int64_t M, int n_col_tiles, int K) {
  const int cus = compute_unit_count();
  const double k_tiles = (double)K / kBK;
  const int64_t wg256 = ((M + 255) / 256) * n_col_tiles, wg128 = ((M + 127) / 128) * n_col_tiles;
  const double t256 = (double)((wg256 + cus - 1) / cus) * (0.8 * k_tiles + 15.0);
  const double t128 = (double)((wg128 + cus - 1) / cus) * (0.47 * k_tiles + 12.0);
  return t256 < t128;
}

bool use_mfma(const qcf_layer_desc& L) {
  return L.dtype == QCF_DTYPE_BF16 && L.d_model % kBK == 0 && (L.n_kv_heads * L.head_dim) % kBN == 0;
}

size_t cs_bytes(const qcf_layer_desc& L, int64_t M) {
  return align_up((size_t)M * (L.head_dim / 2) * sizeof(float2), 256);
}

template <int TM, int TN, int WGM, int WGN>
qcf_status run_mfma(const qcf_layer_desc& L, const QkvArgs& a_in, hipStream_t st) {
  using C = Tile<TM, TN, WGM, WGN>;
  const int64_t mt = (a_in.M + C::BM - 1) / C::BM;
  const int nt = (L.n_q_heads + 2 * L.n_kv_heads) * L.head_dim / kBN;
  const int64_t n_wg = mt * ((nt + 7) / 8) * 8;
  if (mt > 0x7fffffff || n_wg > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "qkv: grid too large");
  const dim3 grid((unsigned)n_wg), block(C::NTHR);
  QkvArgs a = a_in;
  a.m_tiles = (int)mt;
  a.n_tiles = nt;
  static std::atomic<uint64_t> lds_ok[2];
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&qkv_mfma_kernel<TM, TN, WGM, WGN, 0>), C::LDS, lds_ok[0]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&qkv_mfma_kernel<TM, TN, WGM, WGN, 1>), C::LDS, lds_ok[1]));
  if (L.rope_style == 0) qkv_mfma_kernel<TM, TN, WGM, WGN, 0><<<grid, block, C::LDS, st>>>(a);
  else qkv_mfma_kernel<TM, TN, WGM, WGN, 1><<<grid, block, C::LDS, st>>>(a);
  return check_launch("qkv gemm");
}

template <int TM>
qcf_status run_ws(const qcf_layer_desc& L, const QkvArgs& a_in, hipStream_t st) {
  using C = WsTile<TM>;
  const int64_t mt = (a_in.M + C::BM - 1) / C::BM;
  const int nt = (L.n_q_heads + 2 * L.n_kv_heads) * L.head_dim / kBN;
  // Workgroup order.  Few row tiles: all row tiles of a column tile share an XCD, so a weight tile is fetched into
  // one L2 only and the XCD's concurrent workgroups share the row tiles of x.  Many row tiles: an XCD's concurrent
  // workgroups would all belong to one column tile and x would be streamed once per column tile (6 times at 48
  // column tiles); then the row tiles are dealt to the XCDs instead, a row tile of x stays in L2 and the weights
  // are streamed once per row tile (measured at 73 row tiles: 1127 -> 945 us, at 20: 964 -> 912 us).
  const bool rows_over_xcds = mt >= 16;
  const int64_t n_wg = rows_over_xcds ? ((mt + 7) / 8) * 8 * nt : mt * ((nt + 7) / 8) * 8;
  if (mt > 0x7fffffff || n_wg > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "qkv: grid too large");
  const dim3 grid((unsigned)n_wg), block(C::NTHR);
  QkvArgs a = a_in;
  a.m_tiles = (int)mt;
  a.n_tiles = nt;
  a.rows_over_xcds = rows_over_xcds ? 1 : 0;
  static std::atomic<uint64_t> lds_ok[2];
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&qkv_ws_kernel<TM, 0>), C::LDS, lds_ok[0]));
  QCF_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(&qkv_ws_kernel<TM, 1>), C::LDS, lds_ok[1]));
  if (L.rope_style == 0) qkv_ws_kernel<TM, 0><<<grid, block, C::LDS, st>>>(a);
  else qkv_ws_kernel<TM, 1><<<grid, block, C::LDS, st>>>(a);
  return check_launch("qkv gemm");
}

}  // namespace

qcf_status launch_rope_table(const int32_t* pos, int64_t M, int head_dim, double base, float2* cs,
                             hipStream_t st) {
  const int64_t n = M * (head_dim / 2);
  const int64_t blocks = (n + 255) / 256;
  if (blocks > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "rope table: too many rows");
  rope_table_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(pos, M, head_dim,
                                                                -2.0 / (double)head_dim * std::log2(base), cs);
  return check_launch("rope table");
}

size_t qkv_workspace(const qcf_layer_desc& L, int64_t M) {
  if (use_mfma(L)) return 0;                       // the GEMM's epilogue forms the rotary factors itself
  return cs_bytes(L, M) + align_up((size_t)M * (L.n_q_heads + 2 * L.n_kv_heads) * L.head_dim * sizeof(float), 256);
}

qcf_status launch_qkv(const qcf_layer_desc& L, const void* x, int64_t x_rows, const int32_t* gather,
                      int64_t M, const void* w, const int32_t* pos, void* q, void* k, void* v,
                      const int32_t* dst_rows, void* k_fused, void* v_fused, int64_t fused_rows, void* ws,
                      hipStream_t st) {
  const int H = L.n_q_heads, Hkv = L.n_kv_heads, D = L.head_dim;
  const int Ntot = (H + 2 * Hkv) * D;
  if (use_mfma(L)) {
    QkvArgs a;
    a.x = static_cast<const bf16_t*>(x);
    a.w = static_cast<const bf16_t*>(w);
    a.gather = gather;
    a.pos = pos;
    a.neg2_over_d_log2base = -2.0 / (double)D * std::log2(L.rope_base);
    a.x_rows = x_rows;
    a.M = M;
    a.d_model = L.d_model; a.H = H; a.Hkv = Hkv; a.D = D;
    a.m_tiles = 0; a.n_tiles = 0; a.rows_over_xcds = 0;
    a.q = static_cast<bf16_t*>(q); a.k = static_cast<bf16_t*>(k); a.v = static_cast<bf16_t*>(v);
    a.plain = 0; a.residual = nullptr;
    a.dst_rows = dst_rows; a.k_fused = static_cast<bf16_t*>(k_fused); a.v_fused = static_cast<bf16_t*>(v_fused);
    a.fused_rows = fused_rows;
    const bool big = prefer_256_rows(M, Ntot / kBN, L.d_model);
    // (the specialised kernels address x with 32-bit byte offsets)
    const bool ws_ok = (uint64_t)x_rows * (uint64_t)L.d_model * 2u < (1ull << 32);
    if (big && ws_ok) return run_ws<2>(L, a, st);
    if (big) return run_mfma<2, 4, 4, 1>(L, a, st);
    if (ws_ok) return run_ws<1>(L, a, st);
    return run_mfma<2, 2, 2, 2>(L, a, st);
  }
  float2* cs = static_cast<float2*>(ws);
  QCF_TRY(launch_rope_table(pos, M, L.head_dim, L.rope_base, cs, st));
  float* y = reinterpret_cast<float*>(static_cast<char*>(ws) + cs_bytes(L, M));
  const int64_t mb = (M + 63) / 64;
  const int nb = (Ntot + 63) / 64;
  const int64_t rope_blocks = (M * (H + 2 * Hkv) * (D / 2) + 255) / 256;
  if (mb > 0x7fffffff || nb > 65535 || rope_blocks > 0x7fffffff)
    return fail(QCF_ERR_UNSUPPORTED, "qkv: grid too large");
  const dim3 grid((unsigned)mb, (unsigned)nb), block(256);
  if (L.dtype == QCF_DTYPE_BF16) {
    qkv_gemm_generic<bf16_t><<<grid, block, 0, st>>>(static_cast<const bf16_t*>(x), x_rows, gather, M,
                                                     static_cast<const bf16_t*>(w), L.d_model, Ntot, y);
    QCF_TRY_LAUNCH("qkv gemm");
    qkv_rope_split_generic<bf16_t><<<dim3((unsigned)rope_blocks), dim3(256), 0, st>>>(
        y, M, cs, H, Hkv, D, L.rope_style, static_cast<bf16_t*>(q), static_cast<bf16_t*>(k),
        static_cast<bf16_t*>(v));
  } else {
    qkv_gemm_generic<float><<<grid, block, 0, st>>>(static_cast<const float*>(x), x_rows, gather, M,
                                                    static_cast<const float*>(w), L.d_model, Ntot, y);
    QCF_TRY_LAUNCH("qkv gemm");
    qkv_rope_split_generic<float><<<dim3((unsigned)rope_blocks), dim3(256), 0, st>>>(
        y, M, cs, H, Hkv, D, L.rope_style, static_cast<float*>(q), static_cast<float*>(k),
        static_cast<float*>(v));
  }
  QCF_TRY_LAUNCH("qkv rope");
  if (dst_rows) return launch_scatter(L, k, v, dst_rows, M, k_fused, v_fused, fused_rows, st);   // (k, v given: checked by the caller)
  return QCF_OK;
}

// ---- plain linear map, RMSNorm, gated SiLU (rest of the layer for the recomputed rows) -----------------

static bool linear_uses_mfma(const qcf_layer_desc& L, int32_t K, int32_t N) {
  return L.dtype == QCF_DTYPE_BF16 && K % kBK == 0 && N % kBN == 0;
}

size_t linear_workspace(const qcf_layer_desc& L, int64_t M, int32_t K, int32_t N) {
  if (linear_uses_mfma(L, K, N)) return 0;
  return align_up((size_t)M * N * sizeof(float), 256);
}

qcf_status launch_linear(const qcf_layer_desc& L, const void* x, int64_t M, int32_t K, const void* w, int32_t N,
                         const void* residual, void* out, void* ws, hipStream_t st) {
  if (linear_uses_mfma(L, K, N)) {
    // the projection GEMM with one "query" output of N / 128 heads of 128 columns and no rotation
    qcf_layer_desc LL = L;
    LL.d_model = K; LL.n_q_heads = N / kBN; LL.n_kv_heads = 0; LL.head_dim = kBN; LL.rope_style = 0;
    QkvArgs a;
    a.x = static_cast<const bf16_t*>(x);
    a.w = static_cast<const bf16_t*>(w);
    a.gather = nullptr;
    a.pos = nullptr;
    a.neg2_over_d_log2base = 0.0;
    a.x_rows = M;
    a.M = M;
    a.d_model = K; a.H = N / kBN; a.Hkv = 0; a.D = kBN;
    a.m_tiles = 0; a.n_tiles = 0; a.rows_over_xcds = 0;
    a.q = static_cast<bf16_t*>(out); a.k = nullptr; a.v = nullptr;
    a.plain = 1;
    a.residual = static_cast<const bf16_t*>(residual);
    a.dst_rows = nullptr; a.k_fused = nullptr; a.v_fused = nullptr; a.fused_rows = 0;
    const bool big = prefer_256_rows(M, N / kBN, K);
    const bool ws_ok = (uint64_t)M * (uint64_t)K * 2u < (1ull << 32);
    if (big && ws_ok) return run_ws<2>(LL, a, st);
    if (big) return run_mfma<2, 4, 4, 1>(LL, a, st);
    if (ws_ok) return run_ws<1>(LL, a, st);
    return run_mfma<2, 2, 2, 2>(LL, a, st);
  }
  float* y = static_cast<float*>(ws);
  const int64_t mb = (M + 63) / 64;
  const int nb = (N + 63) / 64;
  const int64_t n = M * N;
  if (mb > 0x7fffffff || nb > 65535 || (n + 255) / 256 > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "linear: grid too large");
  const dim3 grid((unsigned)mb, (unsigned)nb), block(256);
  if (L.dtype == QCF_DTYPE_BF16) {
    qkv_gemm_generic<bf16_t><<<grid, block, 0, st>>>(static_cast<const bf16_t*>(x), M, nullptr, M,
                                                     static_cast<const bf16_t*>(w), K, N, y);
    QCF_TRY_LAUNCH("linear gemm");
    linear_finish_generic<bf16_t><<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(
        y, static_cast<const bf16_t*>(residual), n, static_cast<bf16_t*>(out));
  } else {
    qkv_gemm_generic<float><<<grid, block, 0, st>>>(static_cast<const float*>(x), M, nullptr, M,
                                                    static_cast<const float*>(w), K, N, y);
    QCF_TRY_LAUNCH("linear gemm");
    linear_finish_generic<float><<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(
        y, static_cast<const float*>(residual), n, static_cast<float*>(out));
  }
  return check_launch("linear finish");
}

qcf_status launch_rmsnorm(const qcf_layer_desc& L, const void* x, const void* weight, double eps, int64_t M,
                          int32_t cols, void* out, hipStream_t st) {
  if (M > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "rmsnorm: too many rows");
  const dim3 grid((unsigned)M), block(256);
  if (L.dtype == QCF_DTYPE_BF16)
    rmsnorm_kernel<bf16_t><<<grid, block, 0, st>>>(static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(weight),
                                                   (float)eps, cols, static_cast<bf16_t*>(out));
  else
    rmsnorm_kernel<float><<<grid, block, 0, st>>>(static_cast<const float*>(x), static_cast<const float*>(weight),
                                                  (float)eps, cols, static_cast<float*>(out));
  return check_launch("rmsnorm");
}

qcf_status launch_swiglu(const qcf_layer_desc& L, const void* gate_up, int64_t M, int32_t F, void* out,
                         hipStream_t st) {
  const int vec = 16 / elem_size(L.dtype);
  const int64_t blocks = (M * (F / vec) + 255) / 256;
  if (blocks > 0x7fffffff) return fail(QCF_ERR_UNSUPPORTED, "swiglu: too many elements");
  if (L.dtype == QCF_DTYPE_BF16)
    swiglu_kernel<bf16_t><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<const bf16_t*>(gate_up), M, F,
                                                                        static_cast<bf16_t*>(out));
  else
    swiglu_kernel<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<const float*>(gate_up), M, F,
                                                                       static_cast<float*>(out));
  return check_launch("swiglu");
}

}  // namespace qcf
