// Causal self-attention, generic version: any head_dim that is a multiple of the 16-byte
// chunk and at most 256, any sequence length, fp32 or bf16 storage, all math in fp32 on the
// vector ALUs.  It is the path of the all-fp32 mode and the fallback for head sizes the MFMA
// kernels do not cover; it is not a performance path.
//
// Per batch element b and query head h (kv head g = h / (Hq/Hkv)):
//   S[t,u] = q_t . k_u / sqrt(hd) for u <= t;  P = softmax_u(S);  O_t = sum_u P[t,u] v_u
//   lse[t] = log sum_u exp(S[t,u])
// Backward, with D_t = dO_t . O_t:
//   dP[t,u] = dO_t . v_u;  dS = P * (dP - D_t);
//   dq_t = sum_u dS[t,u] k_u / sqrt(hd);  dk_u = sum_t dS[t,u] q_t / sqrt(hd);  dv_u = sum_t P[t,u] dO_t
// dk and dv of a shared kv head sum over the group's query heads in ascending order.  One
// wavefront owns one output row, so no floating-point atomics are needed.
#include "device_utils.h"
#include "internal.h"

namespace jpp {

namespace {

constexpr int kRowsPerBlock = 4;  // one wave per row
constexpr int kMaxHd = 256;
constexpr int kEPerLane = kMaxHd / kWave;

template <typename T>
__device__ inline float dot_row(const float* __restrict__ a_lds, const T* __restrict__ row, int hd) {
  constexpr int N = Chunk<T>::N;
  float s = 0.f;
  for (int c = 0; c < hd / N; ++c) {
    const Chunk<T> v = load_chunk(row + c * N);
#pragma unroll
    for (int e = 0; e < N; ++e) s += a_lds[c * N + e] * v.get(e);
  }
  return s;
}

template <typename T>
__global__ __launch_bounds__(kRowsPerBlock* kWave) void attn_fwd_generic_kernel(
    const T* __restrict__ qkv, T* __restrict__ out, float* __restrict__ lse, int seq, int Hq, int Hkv, int hd) {
  __shared__ float qs[kRowsPerBlock][kMaxHd];
  __shared__ float ps[kRowsPerBlock][kWave];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int t = blockIdx.x * kRowsPerBlock + w;
  const int h = blockIdx.y, b = blockIdx.z;
  if (t >= seq) return;  // whole wave exits together; no block-level barrier is used below
  const int g = h / (Hq / Hkv);
  const int ld = (Hq + 2 * Hkv) * hd;
  const float scale = rsqrtf((float)hd);
  const T* qrow = qkv + ((size_t)b * seq + t) * ld + (size_t)h * hd;
  const T* kbase = qkv + (size_t)b * seq * ld + (size_t)(Hq + g) * hd;
  const T* vbase = kbase + (size_t)Hkv * hd;
  for (int e = lane; e < hd; e += kWave) qs[w][e] = to_f32(qrow[e]);
  wave_lds_sync();
  float m = -INFINITY, l = 0.f, o[kEPerLane] = {};
  for (int u0 = 0; u0 <= t; u0 += kWave) {
    const int u = u0 + lane;
    float s = -INFINITY;
    if (u <= t) s = scale * dot_row<T>(qs[w], kbase + (size_t)u * ld, hd);
    const float mnew = fmaxf(m, wave_max(s));
    const float p = (u <= t) ? __expf(s - mnew) : 0.f;
    const float alpha = __expf(m - mnew);
    l = l * alpha + wave_sum(p);
    m = mnew;
    wave_lds_sync();
    ps[w][lane] = p;
    wave_lds_sync();
    const int nu = min(kWave, t - u0 + 1);
#pragma unroll
    for (int i = 0; i < kEPerLane; ++i) o[i] *= alpha;
    for (int j = 0; j < nu; ++j) {
      const float pj = ps[w][j];
      const T* vrow = vbase + (size_t)(u0 + j) * ld;
#pragma unroll
      for (int i = 0; i < kEPerLane; ++i) {
        const int e = lane + i * kWave;
        if (e < hd) o[i] += pj * to_f32(vrow[e]);
      }
    }
  }
  T* orow = out + ((size_t)b * seq + t) * ((size_t)Hq * hd) + (size_t)h * hd;
  const float inv = 1.f / l;
#pragma unroll
  for (int i = 0; i < kEPerLane; ++i) {
    const int e = lane + i * kWave;
    if (e < hd) orow[e] = from_f32<T>(o[i] * inv);
  }
  if (lane == 0) lse[((size_t)b * Hq + h) * seq + t] = m + __logf(l);
}

// dq rows and D = rowsum(dO * O); one wave per (b, h, t).
template <typename T>
__global__ __launch_bounds__(kRowsPerBlock* kWave) void attn_bwd_dq_generic_kernel(
    const T* __restrict__ qkv, const T* __restrict__ out, const float* __restrict__ lse,
    const T* __restrict__ dout, T* __restrict__ dqkv, float* __restrict__ delta, int seq, int Hq, int Hkv,
    int hd) {
  __shared__ float qs[kRowsPerBlock][kMaxHd];
  __shared__ float dos[kRowsPerBlock][kMaxHd];
  __shared__ float ds_s[kRowsPerBlock][kWave];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int t = blockIdx.x * kRowsPerBlock + w;
  const int h = blockIdx.y, b = blockIdx.z;
  if (t >= seq) return;
  const int g = h / (Hq / Hkv);
  const int ld = (Hq + 2 * Hkv) * hd;
  const float scale = rsqrtf((float)hd);
  const size_t tok = (size_t)b * seq + t;
  const T* qrow = qkv + tok * ld + (size_t)h * hd;
  const T* orow = out + tok * ((size_t)Hq * hd) + (size_t)h * hd;
  const T* dorow = dout + tok * ((size_t)Hq * hd) + (size_t)h * hd;
  const T* kbase = qkv + (size_t)b * seq * ld + (size_t)(Hq + g) * hd;
  const T* vbase = kbase + (size_t)Hkv * hd;
  float dpart = 0.f;
  for (int e = lane; e < hd; e += kWave) {
    qs[w][e] = to_f32(qrow[e]);
    const float d = to_f32(dorow[e]);
    dos[w][e] = d;
    dpart += d * to_f32(orow[e]);
  }
  const float D = wave_sum(dpart);
  const float L = lse[((size_t)b * Hq + h) * seq + t];
  if (lane == 0) delta[((size_t)b * Hq + h) * seq + t] = D;
  wave_lds_sync();
  float dq[kEPerLane] = {};
  for (int u0 = 0; u0 <= t; u0 += kWave) {
    const int u = u0 + lane;
    float ds = 0.f;
    if (u <= t) {
      const float s = scale * dot_row<T>(qs[w], kbase + (size_t)u * ld, hd);
      const float p = __expf(s - L);
      const float dp = dot_row<T>(dos[w], vbase + (size_t)u * ld, hd);
      ds = p * (dp - D);
    }
    wave_lds_sync();
    ds_s[w][lane] = ds;
    wave_lds_sync();
    const int nu = min(kWave, t - u0 + 1);
    for (int j = 0; j < nu; ++j) {
      const float dj = ds_s[w][j];
      const T* krow = kbase + (size_t)(u0 + j) * ld;
#pragma unroll
      for (int i = 0; i < kEPerLane; ++i) {
        const int e = lane + i * kWave;
        if (e < hd) dq[i] += dj * to_f32(krow[e]);
      }
    }
  }
  T* dqrow = dqkv + tok * ld + (size_t)h * hd;
#pragma unroll
  for (int i = 0; i < kEPerLane; ++i) {
    const int e = lane + i * kWave;
    if (e < hd) dqrow[e] = from_f32<T>(dq[i] * scale);
  }
}

// dk and dv rows; one wave per (b, kv head g, key u).
template <typename T>
__global__ __launch_bounds__(kRowsPerBlock* kWave) void attn_bwd_dkv_generic_kernel(
    const T* __restrict__ qkv, const float* __restrict__ lse, const T* __restrict__ dout,
    const float* __restrict__ delta, T* __restrict__ dqkv, int seq, int Hq, int Hkv, int hd) {
  __shared__ float ks[kRowsPerBlock][kMaxHd];
  __shared__ float vs[kRowsPerBlock][kMaxHd];
  __shared__ float p_s[kRowsPerBlock][kWave];
  __shared__ float ds_s[kRowsPerBlock][kWave];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int u = blockIdx.x * kRowsPerBlock + w;
  const int g = blockIdx.y, b = blockIdx.z;
  if (u >= seq) return;
  const int group = Hq / Hkv;
  const int ld = (Hq + 2 * Hkv) * hd;
  const int ldo = Hq * hd;
  const float scale = rsqrtf((float)hd);
  const size_t tok_u = (size_t)b * seq + u;
  const T* krow = qkv + tok_u * ld + (size_t)(Hq + g) * hd;
  const T* vrow = krow + (size_t)Hkv * hd;
  for (int e = lane; e < hd; e += kWave) { ks[w][e] = to_f32(krow[e]); vs[w][e] = to_f32(vrow[e]); }
  wave_lds_sync();
  float dk[kEPerLane] = {}, dv[kEPerLane] = {};
  for (int hh = 0; hh < group; ++hh) {
    const int h = g * group + hh;
    const float* lrow = lse + ((size_t)b * Hq + h) * seq;
    const float* drow = delta + ((size_t)b * Hq + h) * seq;
    for (int t0 = u; t0 < seq; t0 += kWave) {
      const int t = t0 + lane;
      float p = 0.f, ds = 0.f;
      if (t < seq) {
        const size_t tok = (size_t)b * seq + t;
        const float s = scale * dot_row<T>(ks[w], qkv + tok * ld + (size_t)h * hd, hd);
        p = __expf(s - lrow[t]);
        const float dp = dot_row<T>(vs[w], dout + tok * ldo + (size_t)h * hd, hd);
        ds = p * (dp - drow[t]);
      }
      wave_lds_sync();
      p_s[w][lane] = p;
      ds_s[w][lane] = ds;
      wave_lds_sync();
      const int nt = min(kWave, seq - t0);
      for (int j = 0; j < nt; ++j) {
        const float pj = p_s[w][j], dj = ds_s[w][j];
        const size_t tok = (size_t)b * seq + t0 + j;
        const T* qrow = qkv + tok * ld + (size_t)h * hd;
        const T* dorow = dout + tok * ldo + (size_t)h * hd;
#pragma unroll
        for (int i = 0; i < kEPerLane; ++i) {
          const int e = lane + i * kWave;
          if (e < hd) { dv[i] += pj * to_f32(dorow[e]); dk[i] += dj * to_f32(qrow[e]); }
        }
      }
    }
  }
  T* dkrow = dqkv + tok_u * ld + (size_t)(Hq + g) * hd;
  T* dvrow = dkrow + (size_t)Hkv * hd;
#pragma unroll
  for (int i = 0; i < kEPerLane; ++i) {
    const int e = lane + i * kWave;
    if (e < hd) { dkrow[e] = from_f32<T>(dk[i] * scale); dvrow[e] = from_f32<T>(dv[i]); }
  }
}

}  // namespace

hipError_t launch_attention_fwd_generic(int dtype, const AttnDesc& a, hipStream_t s) {
  dim3 grid((a.seq + kRowsPerBlock - 1) / kRowsPerBlock, a.Hq, a.mb);
  if (dtype == JPP_BF16)
    attn_fwd_generic_kernel<bf16><<<grid, kRowsPerBlock * kWave, 0, s>>>((const bf16*)a.qkv, (bf16*)a.out, a.lse,
                                                                         a.seq, a.Hq, a.Hkv, a.hd);
  else
    attn_fwd_generic_kernel<float><<<grid, kRowsPerBlock * kWave, 0, s>>>((const float*)a.qkv, (float*)a.out,
                                                                          a.lse, a.seq, a.Hq, a.Hkv, a.hd);
  return hipGetLastError();
}

hipError_t launch_attention_bwd_generic(int dtype, const AttnDesc& a, hipStream_t s) {
  dim3 gq((a.seq + kRowsPerBlock - 1) / kRowsPerBlock, a.Hq, a.mb);
  dim3 gk((a.seq + kRowsPerBlock - 1) / kRowsPerBlock, a.Hkv, a.mb);
  if (dtype == JPP_BF16) {
    attn_bwd_dq_generic_kernel<bf16><<<gq, kRowsPerBlock * kWave, 0, s>>>(
        (const bf16*)a.qkv, (const bf16*)a.out, a.lse, (const bf16*)a.dout, (bf16*)a.dqkv, a.delta, a.seq, a.Hq,
        a.Hkv, a.hd);
    attn_bwd_dkv_generic_kernel<bf16><<<gk, kRowsPerBlock * kWave, 0, s>>>(
        (const bf16*)a.qkv, a.lse, (const bf16*)a.dout, a.delta, (bf16*)a.dqkv, a.seq, a.Hq, a.Hkv, a.hd);
  } else {
    attn_bwd_dq_generic_kernel<float><<<gq, kRowsPerBlock * kWave, 0, s>>>(
        (const float*)a.qkv, (const float*)a.out, a.lse, (const float*)a.dout, (float*)a.dqkv, a.delta, a.seq,
        a.Hq, a.Hkv, a.hd);
    attn_bwd_dkv_generic_kernel<float><<<gk, kRowsPerBlock * kWave, 0, s>>>(
        (const float*)a.qkv, a.lse, (const float*)a.dout, a.delta, (float*)a.dqkv, a.seq, a.Hq, a.Hkv, a.hd);
  }
  return hipGetLastError();
}

}  // namespace jpp
