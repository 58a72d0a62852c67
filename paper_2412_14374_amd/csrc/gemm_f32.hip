// fp32 GEMM for the all-fp32 storage mode (small parity configuration; not a performance
// path).  C[M,N] (op)= sum_k A(m,k) B(n,k) (+bias[n]) (+residual[m,n]) with arbitrary
// sizes and either operand stored k-major; plain FMA accumulation in ascending k.
#include "device_utils.h"
#include "internal.h"

namespace jpp {

namespace {

constexpr int BM = 64, BN = 64, BK = 16, NT = 256;

__global__ __launch_bounds__(NT) void gemm_f32_kernel(int M, int N, int K, const float* __restrict__ A, int lda,
                                                      int a_ks, const float* __restrict__ B, int ldb, int b_ks,
                                                      float* __restrict__ C, int ldc, int out_mode,
                                                      const float* __restrict__ bias,
                                                      const float* __restrict__ residual) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < BM * BK / NT; ++i) {
      const int e = threadIdx.x + NT * i;
      int mm, kk;
      if (a_ks) { mm = e % BM; kk = e / BM; } else { kk = e % BK; mm = e / BK; }
      const int gm = m0 + mm, gk = k0 + kk;
      float v = 0.f;
      if (gm < M && gk < K) v = a_ks ? A[(size_t)gk * lda + gm] : A[(size_t)gm * lda + gk];
      As[kk][mm] = v;
    }
#pragma unroll
    for (int i = 0; i < BN * BK / NT; ++i) {
      const int e = threadIdx.x + NT * i;
      int nn, kk;
      if (b_ks) { nn = e % BN; kk = e / BN; } else { kk = e % BK; nn = e / BK; }
      const int gn = n0 + nn, gk = k0 + kk;
      float v = 0.f;
      if (gn < N && gk < K) v = b_ks ? B[(size_t)gk * ldb + gn] : B[(size_t)gn * ldb + gk];
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      float v = acc[i][j];
      if (bias) v += bias[gn];
      if (residual) v += residual[(size_t)gm * ldc + gn];
      float* c = C + (size_t)gm * ldc + gn;
      if (out_mode == OUT_ACC_F32) *c += v; else *c = v;
    }
  }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmDesc& g, hipStream_t s) {
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM);
  gemm_f32_kernel<<<grid, NT, 0, s>>>(g.M, g.N, g.K, (const float*)g.A, g.lda, g.a_kstrided ? 1 : 0,
                                      (const float*)g.B, g.ldb, g.b_kstrided ? 1 : 0, (float*)g.C, g.ldc,
                                      g.out_mode, (const float*)g.bias, (const float*)g.residual);
  return hipGetLastError();
}

}  // namespace jpp
