// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <algorithm>
#include <cmath>
#include <atomic>

#include "qcf.h"

namespace qcf {

// ---- host-side error reporting ------------------------------------------------
qcf_status fail(qcf_status s, const char* fmt, ...);
qcf_status check_hip(hipError_t e, const char* what);
qcf_status check_launch(const char* what);

#define QCF_TRY(expr)                 \
  do {                                \
    qcf_status _s = (expr);           \
    if (_s != QCF_OK) return _s;      \
  } while (0)
#define QCF_TRY_LAUNCH(what) QCF_TRY(::qcf::check_launch(what))

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Raises a kernel's dynamic-LDS limit, once per device and kernel (`done` is a bit mask over device ids kept by
// the caller, one per kernel; a repeated call from another thread is harmless).
qcf_status allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done);
// Compute units of the device that was current at the first call (256 if none could be asked).
int compute_unit_count();
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int elem_size(int dtype) { return dtype == QCF_DTYPE_BF16 ? 2 : 4; }

// 16-byte and 8-byte register vectors (native vector types, so they live in registers)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4 r = {a, b, c, d};
  return r;
}

// ---- storage types --------------------------------------------------------------
typedef uint16_t bf16_t;   // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(static_cast<uint32_t>(v) << 16);
}
// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kVec = 4;   // elements per 16-byte access
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 16-byte vector <-> float unpacking
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  __device__ static __forceinline__ void unpack(const u32x4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static __forceinline__ u32x4 pack(const float* f) {
    return mk4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                      __float_as_uint(f[3]));
  }
};
template <> struct Vec16<bf16_t> {
  __device__ static __forceinline__ void unpack(const u32x4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static __forceinline__ u32x4 pack(const float* f) {
    return mk4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                      pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
  }
};

// ---- gfx950 helpers shared by the MFMA kernels ---------------------------------------
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round-to-nearest-even in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  const floatx2_t f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ uint32_t lds_offset_of(const void* lds) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(const_cast<void*>(lds));
}

// 16 bytes per lane from global memory straight into LDS: lane L lands at lds + 16*L (lds is
// wave-uniform).  Issued through inline assembly so that the compiler does not count these among the
// loads it waits for before unrelated LDS reads: callers wait for them themselves
// (__builtin_amdgcn_s_waitcnt(0)) before the barrier that publishes the tile.  M0 (the LDS base of
// such a load) is saved and restored around the instruction.
// Form 1: wave-uniform 64-bit base in scalar registers plus a 32-bit byte offset per lane.
__device__ __forceinline__ void load_to_lds(const void* base, uint32_t lane_off, void* lds) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((int)lds_offset_of(lds));
  const uint64_t b = (uint64_t)(uintptr_t)base;
  // the builtin returns a signed int: widen through uint32_t, or a low half >= 2^31 would smear ones
  // over the high half of the address
  const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32)) << 32) |
                      (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(lane_off), "s"(sb), "s"(lds_addr)
               : "memory");
}
// Form 1 with the LDS destination given as a byte address (wave-uniform).
__device__ __forceinline__ void load_to_lds_at(const void* base, uint32_t lane_off, uint32_t lds_addr_in) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((int)lds_addr_in);
  const uint64_t b = (uint64_t)(uintptr_t)base;
  const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32)) << 32) |
                      (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(lane_off), "s"(sb), "s"(lds_addr)
               : "memory");
}
// Form 2: a full 64-bit address per lane.
__device__ __forceinline__ void load_to_lds_addr(const void* gptr, void* lds) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((int)lds_offset_of(lds));
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(gptr), "s"(lds_addr)
               : "memory");
}

// The same two forms without the compiler-level memory fence: ordinary LDS accesses may be scheduled
// across them (for loops that interleave these loads with fragment reads of another stage and order
// everything with their own waits and barriers).
// Form 1.
__device__ __forceinline__ void load_to_lds_nf(const void* base, uint32_t lane_off, void* lds) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((int)lds_offset_of(lds));
  const uint64_t b = (uint64_t)(uintptr_t)base;
  // the builtin returns a signed int: widen through uint32_t, or a low half >= 2^31 would smear ones
  // over the high half of the address
  const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32)) << 32) |
                      (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(lane_off), "s"(sb), "s"(lds_addr)
               :);
}
// Form 2.
__device__ __forceinline__ void load_to_lds_addr_nf(const void* gptr, void* lds) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((int)lds_offset_of(lds));
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(gptr), "s"(lds_addr)
               :);
}

// ---- launchers (one per translation unit) --------------------------------------
// Each returns QCF_OK or an error after enqueueing on `st`; arguments were validated
// by the entry points in api.hip.

size_t rerope_workspace(const qcf_layer_desc& L, int32_t n_chunks, int64_t total_rows);
qcf_status launch_rerope(const qcf_layer_desc& L, const qcf_chunk* chunks, int32_t n_chunks,
                         int64_t total_rows, void* kf, void* vf, void* ws, hipStream_t st);

// host-side validation shared by the two scoring entry points; *empty = nothing to do
qcf_status check_score_args(const qcf_layer_desc* desc, int32_t B, const void* q_probe,
                            const int64_t* probe_off_dev, int64_t total_probe, const void* k_fused,
                            const int64_t* ctx_off_dev, int64_t total_ctx, const int32_t* probe_limit_dev,
                            float* score, bool* empty);
size_t score_workspace(const qcf_layer_desc& L, int32_t B, int64_t total_probe, int64_t total_ctx);
qcf_status launch_score(const qcf_layer_desc& L, int32_t B, const void* q, const int64_t* probe_off,
                        int64_t total_probe, const void* k, const int64_t* ctx_off, int64_t total_ctx,
                        const int32_t* probe_limit, float* score, float alpha, float beta, void* ws, hipStream_t st);

size_t select_workspace(int32_t B, int64_t total_ctx);
qcf_status launch_select(int32_t B, const float* score, const int64_t* ctx_off, int64_t total_ctx,
                         const int64_t* sel_off, int64_t total_sel, const int32_t* ctx_pos0,
                         int32_t* sel_idx, int32_t* sel_row, int32_t* sel_pos, void* ws,
                         hipStream_t st);

size_t qkv_workspace(const qcf_layer_desc& L, int64_t M);
// dst_rows / k_fused / v_fused (all or none): the K/V rows are also written to rows dst_rows[m] of the fused cache
qcf_status launch_qkv(const qcf_layer_desc& L, const void* x, int64_t x_rows, const int32_t* gather,
                      int64_t M, const void* w, const int32_t* pos, void* q, void* k, void* v,
                      const int32_t* dst_rows, void* k_fused, void* v_fused, int64_t fused_rows,
                      void* ws, hipStream_t st);

qcf_status launch_scatter(const qcf_layer_desc& L, const void* k_new, const void* v_new,
                          const int32_t* rows, int64_t M, void* kf, void* vf, int64_t total_rows,
                          hipStream_t st);

qcf_status launch_gather(const qcf_layer_desc& L, const void* k_src, const void* v_src, const int32_t* rows,
                         int64_t M, int64_t src_rows, void* k_out, void* v_out, hipStream_t st);
qcf_status launch_key_norm(const qcf_layer_desc& L, const void* k, int64_t rows, float* norm, hipStream_t st);

size_t attn_workspace(const qcf_layer_desc& L, int32_t B, int64_t total_sel, int64_t total_ctx);
qcf_status launch_attn(const qcf_layer_desc& L, int32_t B, const void* q, const int32_t* sel_pos,
                       const int64_t* sel_off, int64_t total_sel, const void* k, const void* v,
                       const int64_t* ctx_off, int64_t total_ctx, const int32_t* ctx_pos0, void* o,
                       float* lse, void* ws, hipStream_t st);

size_t linear_workspace(const qcf_layer_desc& L, int64_t M, int32_t K, int32_t N);
qcf_status launch_linear(const qcf_layer_desc& L, const void* x, int64_t M, int32_t K, const void* w, int32_t N,
                         const void* residual, void* out, void* ws, hipStream_t st);
qcf_status launch_rmsnorm(const qcf_layer_desc& L, const void* x, const void* weight, double eps, int64_t M,
                          int32_t cols, void* out, hipStream_t st);
qcf_status launch_swiglu(const qcf_layer_desc& L, const void* gate_up, int64_t M, int32_t F, void* out,
                         hipStream_t st);

// rotary table shared by rerope and qkv: cs[m * (d/2) + i] = (cos, sin)(angle_m * theta_i),
// angles taken in float64.  `pos` gives one integer per row.
qcf_status launch_rope_table(const int32_t* pos, int64_t M, int head_dim, double base, float2* cs,
                             hipStream_t st);

}  // namespace qcf
