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

// GeLU in its two forms and their derivatives (erf form: a = h Phi(h), a' = Phi(h) + h phi(h);
// tanh form: 0.5 h (1 + tanh(k0 (h + k1 h^3)))).  One definition for the element-wise kernels
// and for the GEMM epilogues that apply them, so that both give the same bits.
__device__ inline float gelu_erf(float h) { return 0.5f * h * (1.f + erff(h * 0.70710678118654752f)); }
__device__ inline float gelu_erf_grad(float h) {
  const float cdf = 0.5f * (1.f + erff(h * 0.70710678118654752f));
  const float pdf = 0.3989422804014327f * __expf(-0.5f * h * h);
  return cdf + h * pdf;
}
// The same two for bf16 storage, whose rounding (2^-9) hides a cumulative-normal error of
// 2e-7: Phi(h) without a branch or a division.  The upper tail 1 - Phi(u), u = |h|, equals
// 0.5 * 2^(u Q(u)); Q is the degree-8 least-squares fit at Chebyshev nodes of
// log2(erfc(u / sqrt 2)) / u on [0, 5.7] (normal_tail_fit.py prints the coefficients and the
// error of this fp32 evaluation: |Phi| 2.2e-7, |h Phi| 4.5e-7 over [-8, 8]).  Beyond 5.7 the
// tail is below 2^-26 and Phi rounds to 0 or 1, so u is clamped there.
__device__ inline float normal_cdf_fit(float h) {
  const float u = fminf(fabsf(h), 5.7f);
  float q = 1.206639126e-07f;
  q = fmaf(q, u, -3.104290045e-06f);
  q = fmaf(q, u, 3.136583473e-05f);
  q = fmaf(q, u, -1.292686939e-04f);
  q = fmaf(q, u, -2.939080587e-04f);
  q = fmaf(q, u, 7.268518209e-03f);
  q = fmaf(q, u, -5.261694267e-02f);
  q = fmaf(q, u, -4.591840208e-01f);
  q = fmaf(q, u, -1.151105404e+00f);
  const float tail2 = __builtin_amdgcn_exp2f(q * u);          // 2 (1 - Phi(u))
  return 0.5f + copysignf(0.5f - 0.5f * tail2, h);
}
__device__ inline float gelu_erf_fit(float h) { return h * normal_cdf_fit(h); }
__device__ inline float gelu_erf_grad_fit(float h) {
  // phi(h) = 2^(-h^2 log2(e) / 2) / sqrt(2 pi)
  const float pdf = 0.3989422804014327f * __builtin_amdgcn_exp2f(-0.72134752044448170f * h * h);
  return fmaf(h, pdf, normal_cdf_fit(h));
}
// storage-type dispatch: T = float keeps erff, T = bf16 takes the fit
template <typename T> __device__ inline float gelu_erf_of(float h) { return gelu_erf(h); }
template <> __device__ inline float gelu_erf_of<bf16>(float h) { return gelu_erf_fit(h); }
template <typename T> __device__ inline float gelu_erf_grad_of(float h) { return gelu_erf_grad(h); }
template <> __device__ inline float gelu_erf_grad_of<bf16>(float h) { return gelu_erf_grad_fit(h); }
__device__ inline float gelu_tanh(float h) {
  const float u = 0.7978845608028654f * (h + 0.044715f * h * h * h);
  return 0.5f * h * (1.f + tanhf(u));
}
__device__ inline float gelu_tanh_grad(float h) {
  const float u = 0.7978845608028654f * (h + 0.044715f * h * h * h);
  const float th = tanhf(u);
  const float du = 0.7978845608028654f * (1.f + 3.f * 0.044715f * h * h);
  return 0.5f * (1.f + th) + 0.5f * h * (1.f - th * th) * du;
}

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
