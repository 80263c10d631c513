// Shared host/device helpers for the stage-shard kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tm_stage.h"

namespace tmk {

// ---- error reporting (host) -------------------------------------------------
int fail(int code, const char *fmt, ...);   // records the message for tm_last_error(), returns code
int check_launch(const char *what);         // hipGetLastError() -> TM_ELAUNCH
// Name of the (main) kernel the most recent launcher on this thread enqueued; read by the stage
// profiler to attribute event timings.  Points at a string with static storage.
extern thread_local const char *g_last_kernel;

// ---- storage types -----------------------------------------------------------
typedef __bf16 bf16;

template <typename T> struct Vec;            // 16-byte vector of T
template <> struct Vec<float> {
  static constexpr int N = 4;
  float v[4];
};
template <> struct Vec<bf16> {
  static constexpr int N = 8;
  bf16 v[8];
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }  // round to nearest even

template <typename T> __device__ __forceinline__ void load_vec(const T *p, float (&out)[Vec<T>::N]) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  union { u32x4 raw; Vec<T> v; } u;
  u.raw = *reinterpret_cast<const u32x4 *>(p);
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) out[i] = to_f32(u.v.v[i]);
}
template <typename T> __device__ __forceinline__ void store_vec(T *p, const float (&in)[Vec<T>::N]) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  union { u32x4 raw; Vec<T> v; } u;
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) u.v.v[i] = from_f32<T>(in[i]);
  *reinterpret_cast<u32x4 *>(p) = u.raw;
}

// ---- buffer-descriptor access: reads past `bytes` return zero, writes past it are dropped, so
// ragged edges need no branches (a branch around a load keeps the compiler from batching loads) ----
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}
template <typename T> __device__ __forceinline__ void buf_load_vec(rsrc_t r, uint32_t byte_off, float (&out)[Vec<T>::N]) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  union { u32x4 raw; Vec<T> v; } u;
  u.raw = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0));
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) out[i] = to_f32(u.v.v[i]);
}
template <typename T> __device__ __forceinline__ void buf_store_vec(rsrc_t r, uint32_t byte_off, const float (&in)[Vec<T>::N]) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef unsigned int v4u32 __attribute__((__vector_size__(16)));
  union { u32x4 raw; Vec<T> v; } u;
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) u.v.v[i] = from_f32<T>(in[i]);
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u32, u.raw), r, byte_off, 0, 0);
}

// ---- reductions ---------------------------------------------------------------
constexpr int kWave = 64;

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
  return x;
}

// Sum of two values over a block of NT threads (NT a multiple of 64).  Every thread gets the
// result; the order of additions is fixed, so results are reproducible.  `red` holds 2*NT/64 floats.
template <int NT> __device__ __forceinline__ void block_sum2(float &a, float &b, float *red) {
  constexpr int NW = NT / kWave;
  a = wave_sum(a);
  b = wave_sum(b);
  const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
  __syncthreads();  // protects `red` against the previous use
  if (l == 0) {
    red[w] = a;
    red[NW + w] = b;
  }
  __syncthreads();
  float sa = 0.f, sb = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    sa += red[i];
    sb += red[NW + i];
  }
  a = sa;
  b = sb;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Adam over flat arrays (elementwise.hip): one sweep at full HBM rate.
int adam_launch(int64_t n, float *p, float *g, float *m, float *v, void *p_bf16, const tm_adam_hparams_t *hp, int64_t step,
                hipStream_t s);
int adam_launch_segments(int n_seg, const int64_t *first, const int64_t *count, float *p, float *g, float *m, float *v,
                         void *p_bf16, const tm_adam_hparams_t *hp, int64_t step, hipStream_t s);

}  // namespace tmk
