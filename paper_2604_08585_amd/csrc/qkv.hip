// Step 4: recompute Q/K/V of the selected tokens (Section 3.1 Phase 4 of the paper):
// [Q|K|V] = X_sel W_qkv^T, rotary embedding on Q and K at the tokens' absolute positions.
//
// A small table kernel writes (cos, sin)(pos_m * theta_i) from float64 angles.  The bf16 path
// is a 32x32x16-MFMA GEMM (both operands are contiguous along the contraction dimension) with
// LDS double buffering; an output tile is 128 columns wide, i.e. whole heads, so the rotary
// partner of every element is inside the tile and the embedding is applied in the epilogue.
// The generic path (f32, or shapes the MFMA tiling does not cover) writes the raw product to
// the workspace and rotates it in a second kernel.
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

// ------------------------------------------------------------------ MFMA path (bf16)

constexpr int kBK = 64;                  // contraction elements per LDS stage
constexpr int kLdsStride = kBK + 8;      // bf16 elements per staged row (16-byte pad)
constexpr int kBN = 128;                 // output columns per workgroup (whole heads)
constexpr int kCStride = kBN + 4;        // floats per row of the epilogue slab

struct QkvArgs {
  const bf16_t* x;
  const bf16_t* w;
  const int32_t* gather;
  const float2* cs;
  int64_t x_rows, M;
  int d_model, H, Hkv, D;
  bf16_t* q;
  bf16_t* k;
  bf16_t* v;
};

template <int TM, int TN, int WGM, int WGN>
struct Tile {
  static constexpr int BM = 32 * TM * WGM;
  static constexpr int NTHR = 64 * WGM * WGN;
  static constexpr int A_CH = BM * (kBK / 8) / NTHR;     // 16-byte chunks per thread and stage
  static constexpr int B_CH = kBN * (kBK / 8) / NTHR;
  static constexpr int STAGE = (BM + kBN) * kLdsStride;   // bf16 elements per stage
  static constexpr size_t LDS_MAIN = (size_t)2 * STAGE * 2;
  static constexpr size_t LDS_EPI = (size_t)32 * TM * kCStride * 4;
  static constexpr size_t LDS = LDS_MAIN > LDS_EPI ? LDS_MAIN : LDS_EPI;
  static_assert(32 * TN * WGN == kBN, "a workgroup covers 128 output columns");
  static_assert(BM * (kBK / 8) % NTHR == 0 && kBN * (kBK / 8) % NTHR == 0, "chunk split");
};

template <int TM, int TN, int WGM, int WGN, int STYLE>
__global__ __launch_bounds__(64 * WGM * WGN) void qkv_mfma_kernel(QkvArgs a) {
  using C = Tile<TM, TN, WGM, WGN>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sbase = reinterpret_cast<bf16_t*>(smem);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int64_t m0 = (int64_t)blockIdx.x * C::BM;
  const int col0 = blockIdx.y * kBN;

  // which output does this column tile belong to
  const int q_cols = a.H * a.D, kv_cols = a.Hkv * a.D;
  bf16_t* out;
  int out_cols, out_col0;
  bool rotate = true;
  if (col0 < q_cols) { out = a.q; out_cols = q_cols; out_col0 = col0; }
  else if (col0 < q_cols + kv_cols) { out = a.k; out_cols = kv_cols; out_col0 = col0 - q_cols; }
  else { out = a.v; out_cols = kv_cols; out_col0 = col0 - q_cols - kv_cols; rotate = false; }
  if (!out) return;

  int64_t a_off[C::A_CH], b_off[C::B_CH];
#pragma unroll
  for (int i = 0; i < C::A_CH; ++i) {
    const int chunk = tid + i * C::NTHR;
    const int row = chunk >> 3, c = chunk & 7;
    a_off[i] = -1;
    const int64_t m = m0 + row;
    if (m < a.M) {
      const int64_t idx = a.gather ? (int64_t)a.gather[m] : m;
      if (idx >= 0 && idx < a.x_rows) a_off[i] = idx * a.d_model + c * 8;
    }
  }
#pragma unroll
  for (int i = 0; i < C::B_CH; ++i) {
    const int chunk = tid + i * C::NTHR;
    const int row = chunk >> 3, c = chunk & 7;
    b_off[i] = (int64_t)(col0 + row) * a.d_model + c * 8;
  }
  u32x4 ra[C::A_CH], rb[C::B_CH];
  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < C::A_CH; ++i) {
      ra[i] = u32x4{0u, 0u, 0u, 0u};
      if (a_off[i] >= 0) ra[i] = *reinterpret_cast<const u32x4*>(a.x + a_off[i] + (int64_t)kt * kBK);
    }
#pragma unroll
    for (int i = 0; i < C::B_CH; ++i)
      rb[i] = *reinterpret_cast<const u32x4*>(a.w + b_off[i] + (int64_t)kt * kBK);
  };
  auto swrite = [&](int st) {
    bf16_t* sA = sbase + st * C::STAGE;
    bf16_t* sB = sA + C::BM * kLdsStride;
#pragma unroll
    for (int i = 0; i < C::A_CH; ++i) {
      const int chunk = tid + i * C::NTHR;
      *reinterpret_cast<u32x4*>(sA + (chunk >> 3) * kLdsStride + (chunk & 7) * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < C::B_CH; ++i) {
      const int chunk = tid + i * C::NTHR;
      *reinterpret_cast<u32x4*>(sB + (chunk >> 3) * kLdsStride + (chunk & 7) * 8) = rb[i];
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = floatx16{0};

  const int nk = a.d_model / kBK;
  gload(0);
  swrite(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) gload(kt + 1);
    const bf16_t* sA = sbase + (kt & 1) * C::STAGE;
    const bf16_t* sB = sA + C::BM * kLdsStride;
    const bf16_t* pa = sA + (wm * 32 * TM + (lane & 31)) * kLdsStride + 8 * (lane >> 5);
    const bf16_t* pb = sB + (wn * 32 * TN + (lane & 31)) * kLdsStride + 8 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(pa + i * 32 * kLdsStride + ks * 16));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(pb + j * 32 * kLdsStride + ks * 16));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) swrite((kt + 1) & 1);
    __syncthreads();
  }

  // epilogue: one slab of 32*TM rows at a time goes through LDS as fp32, then every thread
  // rotates 8 pairs (or copies 16 values) and stores two 16-byte vectors.
  float* sC = reinterpret_cast<float*>(smem);
  constexpr int SLAB = 32 * TM;
  const int half = a.D / 2;
  for (int slab = 0; slab < WGM; ++slab) {
    if (wm == slab) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int r = i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            const int c = wn * 32 * TN + j * 32 + (lane & 31);
            sC[r * kCStride + c] = acc[i][j][v];
          }
    }
    __syncthreads();
    for (int task = tid; task < SLAB * 8; task += C::NTHR) {
      const int r = task >> 3, tk = task & 7;
      const int64_t m = m0 + slab * SLAB + r;
      if (m >= a.M) continue;
      int e0, e1, i0;
      if (STYLE == 0) {
        const int per_head = a.D / 16;               // tasks per head
        const int hd = tk / per_head;
        i0 = (tk - hd * per_head) * 8;
        e0 = hd * a.D + i0;
        e1 = e0 + half;
      } else {
        e0 = tk * 16;
        e1 = e0 + 8;
        i0 = (e0 % a.D) / 2;
      }
      float f[16], o[16];
      const float* row = sC + r * kCStride;
#pragma unroll
      for (int p = 0; p < 8; ++p) { f[p] = row[e0 + p]; f[8 + p] = row[e1 + p]; }
      if (rotate) {
        const float2* my = a.cs + m * half + i0;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const float2 w = my[p];
          const int ia = (STYLE == 0) ? p : 2 * p;
          const int ib = (STYLE == 0) ? p + 8 : 2 * p + 1;
          o[ia] = f[ia] * w.x - f[ib] * w.y;
          o[ib] = f[ib] * w.x + f[ia] * w.y;
        }
      } else {
#pragma unroll
        for (int p = 0; p < 16; ++p) o[p] = f[p];
      }
      bf16_t* dst = out + m * out_cols + out_col0;
      *reinterpret_cast<u32x4*>(dst + e0) = Vec16<bf16_t>::pack(o);
      *reinterpret_cast<u32x4*>(dst + e1) = Vec16<bf16_t>::pack(o + 8);
    }
    __syncthreads();
  }
}

bool use_mfma(const qcf_layer_desc& L) {
  return L.dtype == QCF_DTYPE_BF16 && L.d_model % kBK == 0 && (L.n_kv_heads * L.head_dim) % kBN == 0;
}

size_t cs_bytes(const qcf_layer_desc& L, int64_t M) {
  return align_up((size_t)M * (L.head_dim / 2) * sizeof(float2), 256);
}

template <int TM, int TN, int WGM, int WGN>
qcf_status run_mfma(const qcf_layer_desc& L, const QkvArgs& a, hipStream_t st) {
  using C = Tile<TM, TN, WGM, WGN>;
  const int64_t mt = (a.M + C::BM - 1) / C::BM;
  const int nt = (L.n_q_heads + 2 * L.n_kv_heads) * L.head_dim / kBN;
  if (mt > 0x7fffffff || nt > 65535) return fail(QCF_ERR_UNSUPPORTED, "qkv: grid too large");
  const dim3 grid((unsigned)mt, (unsigned)nt), block(C::NTHR);
  static bool attr_done = false;
  if (!attr_done) {
    QCF_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(&qkv_mfma_kernel<TM, TN, WGM, WGN, 0>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS), "qkv attr"));
    QCF_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(&qkv_mfma_kernel<TM, TN, WGM, WGN, 1>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS), "qkv attr"));
    attr_done = true;
  }
  if (L.rope_style == 0) qkv_mfma_kernel<TM, TN, WGM, WGN, 0><<<grid, block, C::LDS, st>>>(a);
  else qkv_mfma_kernel<TM, TN, WGM, WGN, 1><<<grid, block, C::LDS, st>>>(a);
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
  size_t bytes = cs_bytes(L, M);
  if (!use_mfma(L))
    bytes += align_up((size_t)M * (L.n_q_heads + 2 * L.n_kv_heads) * L.head_dim * sizeof(float), 256);
  return bytes;
}

qcf_status launch_qkv(const qcf_layer_desc& L, const void* x, int64_t x_rows, const int32_t* gather,
                      int64_t M, const void* w, const int32_t* pos, void* q, void* k, void* v, void* ws,
                      hipStream_t st) {
  float2* cs = static_cast<float2*>(ws);
  QCF_TRY(launch_rope_table(pos, M, L.head_dim, L.rope_base, cs, st));
  const int H = L.n_q_heads, Hkv = L.n_kv_heads, D = L.head_dim;
  const int Ntot = (H + 2 * Hkv) * D;
  if (use_mfma(L)) {
    QkvArgs a;
    a.x = static_cast<const bf16_t*>(x);
    a.w = static_cast<const bf16_t*>(w);
    a.gather = gather;
    a.cs = cs;
    a.x_rows = x_rows;
    a.M = M;
    a.d_model = L.d_model; a.H = H; a.Hkv = Hkv; a.D = D;
    a.q = static_cast<bf16_t*>(q); a.k = static_cast<bf16_t*>(k); a.v = static_cast<bf16_t*>(v);
    // 256-row tiles when they still give every compute unit a workgroup, else 128-row tiles
    const int64_t tiles256 = ((M + 255) / 256) * (Ntot / kBN);
    if (tiles256 >= 200) return run_mfma<2, 4, 4, 1>(L, a, st);
    return run_mfma<2, 2, 2, 2>(L, a, st);
  }
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
  return check_launch("qkv rope");
}

}  // namespace qcf
