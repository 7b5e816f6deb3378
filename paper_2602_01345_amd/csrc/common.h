// Device-side helpers shared by the gfx950 kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define NOVA_WAVE 64

typedef __bf16 bf16_t;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// element load/store with widening to fp32 (T = float or bf16_t)
template <typename T> __device__ __forceinline__ float ld_f32(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void st_f32(T* p, float v) { *p = (T)v; }

// 16-byte vector of T as fp32 lanes
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  f32x4 v;
  __device__ __forceinline__ void load(const float* p) { v = *reinterpret_cast<const f32x4*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<f32x4*>(p) = v; }
  __device__ __forceinline__ float get(int i) const { return v[i]; }
  __device__ __forceinline__ void set(int i, float x) { v[i] = x; }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  bf16x8 v;
  __device__ __forceinline__ void load(const bf16_t* p) { v = *reinterpret_cast<const bf16x8*>(p); }
  __device__ __forceinline__ void store(bf16_t* p) const { *reinterpret_cast<bf16x8*>(p) = v; }
  __device__ __forceinline__ float get(int i) const { return (float)v[i]; }
  __device__ __forceinline__ void set(int i, float x) { v[i] = (bf16_t)x; }
};

// Per-image keep counts (the reduction ratios of Sec. 3.3, "Dual-Linkage Acceleration", are per instance): the
// kept rows of image b are slots [0, k_b) of its kpitch-row segment, and it holds its own number of prior K/V rows.
// Null pointers mean "uniform": every image keeps kpitch rows / holds P prior rows.  Values are clamped, so a
// count the host never saw cannot send a kernel out of bounds.
__device__ __forceinline__ int image_count(const int32_t* __restrict__ k_rows, int b, int kpitch) {
  if (!k_rows) return kpitch;
  const int v = k_rows[b];
  return v < 0 ? 0 : (v > kpitch ? kpitch : v);
}
__device__ __forceinline__ int image_prior(const int32_t* __restrict__ kv_rows, int b, int P) {
  if (!kv_rows) return P;
  const int v = kv_rows[b];
  return v < 0 ? 0 : (v > P ? P : v);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, NOVA_WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, NOVA_WAVE));
  return v;
}
