// Device-side helpers for gfx950 (wave64) kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace jpp {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// 16-byte chunk of storage elements: 4 floats or 8 bf16.
template <typename T> struct Chunk;
template <> struct Chunk<float> {
  static constexpr int N = 4;
  f32x4 v;
  __device__ float get(int i) const { return v[i]; }
  __device__ void set(int i, float f) { v[i] = f; }
};
template <> struct Chunk<bf16> {
  static constexpr int N = 8;
  bf16x8 v;
  __device__ float get(int i) const { return (float)v[i]; }
  __device__ void set(int i, float f) { v[i] = (bf16)f; }  // round to nearest even
};

template <typename T>
__device__ inline Chunk<T> load_chunk(const T* p) {
  Chunk<T> c;
  c.v = *reinterpret_cast<const decltype(c.v)*>(p);
  return c;
}
template <typename T>
__device__ inline void store_chunk(T* p, const Chunk<T>& c) {
  *reinterpret_cast<decltype(c.v)*>(p) = c.v;
}

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ inline T from_f32(float x);
template <> __device__ inline float from_f32<float>(float x) { return x; }
template <> __device__ inline bf16 from_f32<bf16>(float x) { return (bf16)x; }

// Makes LDS writes of this wave's lanes visible to its other lanes (waves run their LDS
// operations in order; the fences keep the compiler from moving accesses across).
__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Sum over the 64 lanes of a wave; every lane gets the result.
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// Sum over a workgroup of NW waves through LDS (`red` holds at least NW floats per
// concurrent reduction).  All threads must call; all get the result.  The fixed
// shuffle pattern and the fixed wave order make the result independent of timing.
template <int NW>
__device__ inline float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) t += red[i];
  return t;
}
template <int NW>
__device__ inline float block_max(float v, float* red) {
  v = wave_max(v);
  const int w = threadIdx.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) t = fmaxf(t, red[i]);
  return t;
}

}  // namespace jpp
