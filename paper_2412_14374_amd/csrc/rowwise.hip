// Bandwidth-bound kernels of the stage: norms, activations, RoPE, bias/gain gradients,
// cross-entropy, zero fill.  All are written for 64-wide wavefronts with 16-byte
// accesses per lane and deterministic (fixed-order) reductions; math is fp32.
//
// The paper defines none of these operations (its Evaluation section only names the
// GPT-3 and Llama 2 model families); the formulas are the standard ones and are stated
// next to each kernel.
#include <cmath>

#include <type_traits>
#include <utility>

#include "device_utils.h"
#include "internal.h"

namespace jpp {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

// Reduces two values at once over a workgroup of NW waves.
template <int NW = kWaves>
__device__ inline void block_sum2(float& a, float& b, float* red /* >= 2*NW */) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int w = threadIdx.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) { red[w] = a; red[NW + w] = b; }
  __syncthreads();
  float ta = 0.f, tb = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) { ta += red[i]; tb += red[NW + i]; }
  a = ta; b = tb;
}

// Reduces NV values at once over a workgroup of NW waves (one pass through LDS for all of them);
// for a value, the same order of additions as block_sum2.
template <int NV, int NW>
__device__ inline void block_sum_many(float (&v)[NV], float* red /* >= NV*NW */) {
#pragma unroll
  for (int q = 0; q < NV; ++q) v[q] = wave_sum(v[q]);
  const int w = threadIdx.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) {
#pragma unroll
    for (int q = 0; q < NV; ++q) red[q * NW + w] = v[q];
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += red[q * NW + i];
    v[q] = t;
  }
}

// ---------------------------------------------------------------------------------------
// Norm forward.  LayerNorm: y = (x - mean) * rstd * gamma + beta, rstd = 1/sqrt(var + eps),
// biased variance.  RMSNorm: y = x * rstd * gamma, rstd = 1/sqrt(mean(x^2) + eps).
// One workgroup per row; the row stays in registers between the statistics and the
// normalisation, so x is read once.  stats[2r] = mean (0 for RMSNorm), stats[2r+1] = rstd.
template <typename T, int MAXC>
__global__ __launch_bounds__(kThreads) void norm_fwd_kernel(const T* __restrict__ x,
                                                            const T* __restrict__ gamma,
                                                            const T* __restrict__ beta,
                                                            T* __restrict__ y, float* __restrict__ stats,
                                                            int d, float eps, int norm) {
  __shared__ float red[2 * kWaves];
  constexpr int N = Chunk<T>::N;
  const int nchunks = d / N;
  const size_t base = (size_t)blockIdx.x * d;
  // Every load is unconditional (a chunk index beyond the row reads the row's last chunk
  // instead, and its values are not used): loads inside the `c < nchunks` branches would each be
  // waited for before the next is issued.
  Chunk<T> xs[MAXC];
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    xs[j] = load_chunk(x + base + (size_t)(c < nchunks ? c : nchunks - 1) * N);
  }
  // gain and offset are requested behind the row: they arrive during the reductions
  Chunk<T> gs[MAXC], bs[MAXC];
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    const size_t o = (size_t)(c < nchunks ? c : nchunks - 1) * N;
    gs[j] = load_chunk(gamma + o);
    if (beta != nullptr) bs[j] = load_chunk(beta + o);
  }
  float s = 0.f, ss = 0.f;
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    if (c < nchunks) {
#pragma unroll
      for (int e = 0; e < N; ++e) { const float v = xs[j].get(e); s += v; ss += v * v; }
    }
  }
  float mean = 0.f, rstd;
  const float inv_d = 1.f / (float)d;
  if (norm == JPP_LAYERNORM) {
    float dummy = 0.f;
    block_sum2(s, dummy, red);
    mean = s * inv_d;
    float v2 = 0.f;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
      const int c = threadIdx.x + j * kThreads;
      if (c < nchunks) {
#pragma unroll
        for (int e = 0; e < N; ++e) { const float t = xs[j].get(e) - mean; v2 += t * t; }
      }
    }
    dummy = 0.f;
    block_sum2(v2, dummy, red);
    rstd = rsqrtf(v2 * inv_d + eps);
  } else {
    float dummy = 0.f;
    block_sum2(ss, dummy, red);
    rstd = rsqrtf(ss * inv_d + eps);
  }
  if (threadIdx.x == 0) { stats[2 * (size_t)blockIdx.x] = mean; stats[2 * (size_t)blockIdx.x + 1] = rstd; }
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    if (c < nchunks) {
      Chunk<T> o;
      if (beta != nullptr) {
#pragma unroll
        for (int e = 0; e < N; ++e) o.set(e, (xs[j].get(e) - mean) * rstd * gs[j].get(e) + bs[j].get(e));
      } else {
#pragma unroll
        for (int e = 0; e < N; ++e) o.set(e, (xs[j].get(e) - mean) * rstd * gs[j].get(e));
      }
      store_chunk(y + base + (size_t)c * N, o);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Norm backward.  With xhat = (x - mean) * rstd and dxhat = dy * gamma:
//   LayerNorm: dx = rstd * (dxhat - mean_d(dxhat) - xhat * mean_d(dxhat * xhat))
//   RMSNorm:   dx = rstd * (dxhat - xhat * mean_d(dxhat * xhat))
//   dgamma = sum_rows dy * xhat,  dbeta = sum_rows dy.
// dx_add (optional) is added to dx (the residual branch's cotangent).
// A workgroup owns the rows {b, b + nblk, ...}; it keeps per-column partial sums of
// dgamma/dbeta in registers and writes them to partial[b, :]; a second kernel adds the
// nblk partials in ascending order into the fp32 gradient (no atomics).
// NT threads per workgroup.  The narrow form (256 threads, up to 8 chunks per thread) fetches
// dx_add when a row is processed; the wide form (512 threads, for rows of 1024 chunks and more)
// has the registers to fetch it with the row, one row ahead, so that nothing a row needs is
// still on its way when the row's turn comes.  A turn of a workgroup is R of its rows (the next
// R in its ascending order), reduced together in one pass through LDS: narrow rows, whose single
// row would leave a compute unit with a few KB of loads in flight, take R = 2 or 4.
// FAST != 0: the row is exactly MAXC * NT chunks and every workgroup has only full turns
// (rows a multiple of R * gridDim.x), dx_add is absent (1) or present (2): nothing is predicated
// and no branch stands between a load and its use, so the compiler counts the accesses in
// flight instead of waiting for all of them (stores included) at every join.
template <typename T, int MAXC, int NT = kThreads, bool WIDE = false, int R = 1, int FAST = 0>
__global__ __launch_bounds__(NT) void norm_bwd_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const float* __restrict__ stats,
    const T* __restrict__ dy, const T* __restrict__ dx_add, T* __restrict__ dx,
    float* __restrict__ partial_g, float* __restrict__ partial_b, int rows, int d, int norm) {
  constexpr int NW = NT / kWave;
  __shared__ float red[2 * R * NW];
  constexpr int N = Chunk<T>::N;
  const int nchunks = d / N;
  const float inv_d = 1.f / (float)d;
  float pg[MAXC][N], pb[MAXC][N];
  Chunk<T> gs[MAXC];
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * NT;
    if (FAST || c < nchunks) gs[j] = load_chunk(gamma + (size_t)c * N);
#pragma unroll
    for (int e = 0; e < N; ++e) { pg[j][e] = 0.f; pb[j][e] = 0.f; }
  }
  // One turn's operands in registers.  The next turn of this workgroup is fetched while the
  // current one is reduced and written, so a turn costs one memory latency, not three.
  struct Turn { Chunk<T> xs[R][MAXC], ds[R][MAXC], as[R][WIDE ? MAXC : 1]; float mean[R], rstd[R]; };
  const int stride = gridDim.x;
  // row i of the turn that starts at row r0
  auto row_of = [&](int r0, int i) { return r0 + i * stride; };
  auto fetch = [&](int r0, Turn& w) {
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int r = row_of(r0, i);
      if (FAST || r < rows) {
        const size_t base = (size_t)r * d;
        w.mean[i] = stats[2 * (size_t)r];
        w.rstd[i] = stats[2 * (size_t)r + 1];
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
          const int c = threadIdx.x + j * NT;
          if (FAST || c < nchunks) {
            w.xs[i][j] = load_chunk(x + base + (size_t)c * N);
            w.ds[i][j] = load_chunk(dy + base + (size_t)c * N);
            if constexpr (WIDE) {
              if (FAST ? FAST == 2 : dx_add != nullptr) w.as[i][j] = load_chunk(dx_add + base + (size_t)c * N);
            }
          }
        }
      }
    }
  };
  auto process = [&](int r0, const Turn& w) {
    // the tensor added to the result is only needed after the reduction: its latency hides there
    Chunk<T> as[R][MAXC];
    if constexpr (WIDE) {
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int j = 0; j < MAXC; ++j) as[i][j] = w.as[i][j];
    } else if (FAST ? FAST == 2 : dx_add != nullptr) {
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const int r = row_of(r0, i);
        if (FAST || r < rows) {
#pragma unroll
          for (int j = 0; j < MAXC; ++j) {
            const int c = threadIdx.x + j * NT;
            if (FAST || c < nchunks) as[i][j] = load_chunk(dx_add + (size_t)r * d + (size_t)c * N);
          }
        }
      }
    }
    float sums[2 * R];
#pragma unroll
    for (int i = 0; i < R; ++i) {
      float s1 = 0.f, s2 = 0.f;
      if (FAST || row_of(r0, i) < rows) {
        const float mean = w.mean[i], rstd = w.rstd[i];
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
          const int c = threadIdx.x + j * NT;
          if (FAST || c < nchunks) {
#pragma unroll
            for (int e = 0; e < N; ++e) {
              const float xh = (w.xs[i][j].get(e) - mean) * rstd;
              const float dv = w.ds[i][j].get(e);
              const float dxh = dv * gs[j].get(e);
              s1 += dxh;
              s2 += dxh * xh;
              pg[j][e] += dv * xh;
              pb[j][e] += dv;
            }
          }
        }
      }
      sums[2 * i] = s1;
      sums[2 * i + 1] = s2;
    }
    block_sum_many<2 * R, NW>(sums, red);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int r = row_of(r0, i);
      if (FAST || r < rows) {
        const float mean = w.mean[i], rstd = w.rstd[i];
        const float m1 = (norm == JPP_LAYERNORM) ? sums[2 * i] * inv_d : 0.f;
        const float m2 = sums[2 * i + 1] * inv_d;
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
          const int c = threadIdx.x + j * NT;
          if (FAST || c < nchunks) {
            Chunk<T> o;
#pragma unroll
            for (int e = 0; e < N; ++e) {
              const float xh = (w.xs[i][j].get(e) - mean) * rstd;
              const float dxh = w.ds[i][j].get(e) * gs[j].get(e);
              float v = rstd * (dxh - m1 - xh * m2);
              if (FAST ? FAST == 2 : dx_add != nullptr) v += as[i][j].get(e);
              o.set(e, v);
            }
            store_chunk(dx + (size_t)r * d + (size_t)c * N, o);
          }
        }
      }
    }
  };
  const int turn = R * stride;   // rows between the first rows of two turns of a workgroup
  if constexpr (MAXC > 6) {
    // two rows of this width do not fit the register file: one at a time
    Turn a;
    for (int r = blockIdx.x; r < rows; r += turn) {
      fetch(r, a);
      process(r, a);
    }
  } else {
    Turn a, b;
    int r = blockIdx.x;
    if (r < rows) fetch(r, a);
    while (r < rows) {
      int nxt = r + turn;
      if (nxt < rows) fetch(nxt, b);
      process(r, a);
      r = nxt;
      if (r >= rows) break;
      nxt = r + turn;
      if (nxt < rows) fetch(nxt, a);
      process(r, b);
      r = nxt;
    }
  }
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * NT;
    if (FAST || c < nchunks) {
      const size_t o = (size_t)blockIdx.x * d + (size_t)c * N;
#pragma unroll
      for (int e = 0; e < N; ++e) {
        partial_g[o + e] = pg[j][e];
        if (partial_b != nullptr) partial_b[o + e] = pb[j][e];
      }
    }
  }
}

// g[col] += sum_b partial[b, col].  32 columns x 8 row groups per workgroup: group q adds the
// partial rows q, q+8, ... in ascending order, then the 8 group sums are added in ascending
// order: a fixed association, independent of timing.  A launch with gridDim.y = 2 finishes a
// second (partial2, g2) pair of the same shape in its y = 1 workgroups.
constexpr int kFinCols = 32, kFinGroups = kThreads / kFinCols;
__global__ __launch_bounds__(kThreads) void colreduce_finish_kernel(const float* __restrict__ partial,
                                                                    int nblk, int n, float* __restrict__ g,
                                                                    const float* __restrict__ partial2 = nullptr,
                                                                    float* __restrict__ g2 = nullptr) {
  __shared__ float red[kFinGroups][kFinCols];
  if (blockIdx.y == 1) { partial = partial2; g = g2; }
  const int c = threadIdx.x % kFinCols, q = threadIdx.x / kFinCols;
  const int col = blockIdx.x * kFinCols + c;
  float acc = 0.f;
  if (col < n) {
#pragma unroll 8
    for (int b = q; b < nblk; b += kFinGroups) acc += partial[(size_t)b * n + col];
  }
  red[q][c] = acc;
  __syncthreads();
  if (q == 0 && col < n) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < kFinGroups; ++i) t += red[i][c];
    g[col] += t;
  }
}

// partial[b, col] = sum over rows {b, b + nblk, ...} of dy[r, col]
template <typename T>
__global__ __launch_bounds__(kThreads) void colsum_partial_kernel(const T* __restrict__ dy, int ld, int rows,
                                                                  int n, float* __restrict__ partial) {
  constexpr int N = Chunk<T>::N;
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c * N >= n) return;
  float acc[N];
#pragma unroll
  for (int e = 0; e < N; ++e) acc[e] = 0.f;
  // four of the thread's rows are requested before the first is added (the additions keep
  // their order, so the sums are the same bits as with one row at a time)
  constexpr int kAhead = 4;
  const int step = gridDim.y;
  for (int r = blockIdx.y; r < rows; r += kAhead * step) {
    Chunk<T> v[kAhead];
#pragma unroll
    for (int j = 0; j < kAhead; ++j)
      if (r + j * step < rows) v[j] = load_chunk(dy + (size_t)(r + j * step) * ld + (size_t)c * N);
#pragma unroll
    for (int j = 0; j < kAhead; ++j)
      if (r + j * step < rows) {
#pragma unroll
        for (int e = 0; e < N; ++e) acc[e] += v[j].get(e);
      }
  }
#pragma unroll
  for (int e = 0; e < N; ++e) partial[(size_t)blockIdx.y * n + (size_t)c * N + e] = acc[e];
}

// ---------------------------------------------------------------------------------------
// Activations.  GeLU (erf form): a = h * Phi(h), Phi the standard normal CDF;
// a' = Phi(h) + h * phi(h).  Tanh form: 0.5 h (1 + tanh(k0 (h + k1 h^3))).
// SwiGLU on h = [gate | up]: a = silu(gate) * up, silu(t) = t * sigmoid(t),
// silu'(t) = sigmoid(t) * (1 + t * (1 - sigmoid(t))).
__device__ inline float sigmoidf(float t) { return 1.f / (1.f + __expf(-t)); }

// A thread owns one 16-byte column chunk and walks the rows kActRows at a time: the loads of
// the rows of one step are all issued before the first is used, and no index is divided.
constexpr int kActRows = 4;

template <typename T, int ACT>
__global__ __launch_bounds__(kThreads) void act_fwd_kernel(const T* __restrict__ h, T* __restrict__ a,
                                                           int rows, int f) {
  constexpr int N = Chunk<T>::N;
  const int c = blockIdx.x * kThreads + threadIdx.x;   // chunk of the output row
  if (c * N >= f) return;
  const size_t hld = ACT == JPP_SWIGLU ? 2 * (size_t)f : (size_t)f;
  for (int r0 = blockIdx.y * kActRows; r0 < rows; r0 += gridDim.y * kActRows) {
    Chunk<T> v[kActRows], u[kActRows];
#pragma unroll
    for (int j = 0; j < kActRows; ++j) {
      if (r0 + j < rows) {
        v[j] = load_chunk(h + (size_t)(r0 + j) * hld + (size_t)c * N);
        if (ACT == JPP_SWIGLU) u[j] = load_chunk(h + (size_t)(r0 + j) * hld + f + (size_t)c * N);
      }
    }
#pragma unroll
    for (int j = 0; j < kActRows; ++j) {
      if (r0 + j < rows) {
        Chunk<T> o;
#pragma unroll
        for (int e = 0; e < N; ++e) {
          const float t = v[j].get(e);
          if (ACT == JPP_SWIGLU) o.set(e, t * sigmoidf(t) * u[j].get(e));
          else if (ACT == JPP_GELU) o.set(e, gelu_erf_of<T>(t));
          else o.set(e, gelu_tanh(t));
        }
        store_chunk(a + (size_t)(r0 + j) * f + (size_t)c * N, o);
      }
    }
  }
}

template <typename T, int ACT>
__global__ __launch_bounds__(kThreads) void act_bwd_kernel(const T* __restrict__ h, const T* __restrict__ da,
                                                           T* __restrict__ dh, int rows, int f) {
  constexpr int N = Chunk<T>::N;
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c * N >= f) return;
  const size_t hld = ACT == JPP_SWIGLU ? 2 * (size_t)f : (size_t)f;
  for (int r0 = blockIdx.y * kActRows; r0 < rows; r0 += gridDim.y * kActRows) {
    Chunk<T> d[kActRows], v[kActRows], u[kActRows];
#pragma unroll
    for (int j = 0; j < kActRows; ++j) {
      if (r0 + j < rows) {
        d[j] = load_chunk(da + (size_t)(r0 + j) * f + (size_t)c * N);
        v[j] = load_chunk(h + (size_t)(r0 + j) * hld + (size_t)c * N);
        if (ACT == JPP_SWIGLU) u[j] = load_chunk(h + (size_t)(r0 + j) * hld + f + (size_t)c * N);
      }
    }
#pragma unroll
    for (int j = 0; j < kActRows; ++j) {
      if (r0 + j < rows) {
        T* out = dh + (size_t)(r0 + j) * hld + (size_t)c * N;
        if (ACT == JPP_SWIGLU) {
          Chunk<T> og, ou;
#pragma unroll
          for (int e = 0; e < N; ++e) {
            const float t = v[j].get(e), sg = sigmoidf(t), dv = d[j].get(e);
            og.set(e, dv * u[j].get(e) * sg * (1.f + t * (1.f - sg)));
            ou.set(e, dv * t * sg);
          }
          store_chunk(out, og);
          store_chunk(out + f, ou);
        } else {
          Chunk<T> o;
#pragma unroll
          for (int e = 0; e < N; ++e)
            o.set(e, d[j].get(e) * (ACT == JPP_GELU ? gelu_erf_grad_of<T>(v[j].get(e)) : gelu_tanh_grad(v[j].get(e))));
          store_chunk(out, o);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// RoPE.  Element j < hd/2 of a head is paired with element j + hd/2; the pair at sequence
// position p is rotated by angle(p, j) = p * theta^(-2j/hd).  The table holds
// (cos, sin) as fp32, computed in double precision.  The inverse rotation is the backward.
__global__ void rope_table_kernel(float* __restrict__ table, int seq, int hd, double theta) {
  const int half = hd / 2;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= seq * half) return;
  const int p = idx / half, j = idx - p * half;
  const double inv = pow(theta, -2.0 * (double)j / (double)hd);
  const double ang = (double)p * inv;
  table[2 * (size_t)idx] = (float)cos(ang);
  table[2 * (size_t)idx + 1] = (float)sin(ang);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void rope_kernel(T* __restrict__ qkv, const float* __restrict__ table,
                                                        int tokens, int seq, int heads, int hd, int ld,
                                                        float sign) {
  constexpr int N = Chunk<T>::N;
  const int half = hd / 2;
  const int cph = half / N;  // chunk pairs per head
  const size_t total = (size_t)tokens * heads * cph;
  for (size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * kThreads) {
    const int c = (int)(idx % cph);
    const size_t th = idx / cph;
    const int head = (int)(th % heads);
    const size_t tok = th / heads;
    const int pos = (int)(tok % seq);
    T* p = qkv + tok * ld + (size_t)head * hd + (size_t)c * N;
    Chunk<T> a = load_chunk(p), b = load_chunk(p + half);
    Chunk<T> oa, ob;
#pragma unroll
    for (int e = 0; e < N; ++e) {
      const size_t ti = 2 * ((size_t)pos * half + (size_t)c * N + e);
      const float cs = table[ti], sn = sign * table[ti + 1];
      const float av = a.get(e), bv = b.get(e);
      oa.set(e, av * cs - bv * sn);
      ob.set(e, av * sn + bv * cs);
    }
    store_chunk(p, oa);
    store_chunk(p + half, ob);
  }
}

// ---------------------------------------------------------------------------------------
// Mean-token cross-entropy from fp32 logits.  Per row r: lse = log sum_v exp(z_v);
// row_loss[r] = lse - z[target]; dz = (exp(z - lse) - onehot(target)) / rows.
// One workgroup per row; the row is read three times (max, sum, gradient), the last two
// mostly from L2.
template <typename T>
__global__ __launch_bounds__(kThreads) void cross_entropy_kernel(const float* __restrict__ z,
                                                                 const int32_t* __restrict__ targets,
                                                                 T* __restrict__ dz, float* __restrict__ row_loss,
                                                                 int rows, int vocab) {
  __shared__ float red[kWaves];
  const size_t base = (size_t)blockIdx.x * vocab;
  float m = -INFINITY;
  for (int v = threadIdx.x; v < vocab; v += kThreads) m = fmaxf(m, z[base + v]);
  m = block_max<kWaves>(m, red);
  float s = 0.f;
  for (int v = threadIdx.x; v < vocab; v += kThreads) s += __expf(z[base + v] - m);
  s = block_sum<kWaves>(s, red);
  const float lse = m + __logf(s);
  const int tgt = targets[blockIdx.x];
  // An id outside [0, vocab) cannot be indexed: its row reports NaN instead of reading out of bounds.
  const bool tgt_ok = (unsigned)tgt < (unsigned)vocab;
  if (threadIdx.x == 0) row_loss[blockIdx.x] = tgt_ok ? lse - z[base + tgt] : NAN;
  const float inv_rows = 1.f / (float)rows;
  for (int v = threadIdx.x; v < vocab; v += kThreads) {
    float p = __expf(z[base + v] - lse);
    if (v == tgt) p -= 1.f;
    dz[base + v] = from_f32<T>(p * inv_rows);
  }
}

// The same with the row held in registers: one workgroup of NT threads per row, every thread CH
// chunks of four logits (chunk j of thread t is chunk t + j * NT of the row), so the fp32 logits
// are read once, by 16-byte loads that are all in flight together, instead of three times.
// For vocab a multiple of 4 with (CH - 1) * NT < vocab / 4 <= CH * NT: only a thread's last
// chunk can lie beyond the row's end, every other load and store is unconditional.
template <typename T, int CH, int NT, int kMinWaves>
__global__ __launch_bounds__(NT, kMinWaves) void cross_entropy_reg_kernel(const float* __restrict__ z,
                                                                          const int32_t* __restrict__ targets,
                                                                          T* __restrict__ dz,
                                                                          float* __restrict__ row_loss, int rows,
                                                                          int vocab) {
  constexpr int NW = NT / kWave;
  __shared__ float red[NW];
  typedef T T4 __attribute__((ext_vector_type(4)));
  const float* zr = z + (size_t)blockIdx.x * vocab;
  T* dzr = dz + (size_t)blockIdx.x * vocab;
  const bool last_ok = (int)threadIdx.x + (CH - 1) * NT < vocab / 4;
  f32x4 x[CH];
#pragma unroll
  for (int j = 0; j < CH - 1; ++j) x[j] = *reinterpret_cast<const f32x4*>(zr + (threadIdx.x + j * NT) * 4);
  x[CH - 1] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};   // exp(-inf - m) adds nothing to the sum
  if (last_ok) x[CH - 1] = *reinterpret_cast<const f32x4*>(zr + (threadIdx.x + (CH - 1) * NT) * 4);
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < CH; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) m = fmaxf(m, x[j][e]);
  m = block_max<NW>(m, red);
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < CH; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) s += __expf(x[j][e] - m);
  s = block_sum<NW>(s, red);
  const float lse = m + __logf(s);
  const int tgt = targets[blockIdx.x];
  // An id outside [0, vocab) cannot be indexed: its row reports NaN instead of reading out of bounds.
  const bool tgt_ok = (unsigned)tgt < (unsigned)vocab;
  if (threadIdx.x == 0) row_loss[blockIdx.x] = tgt_ok ? lse - zr[tgt] : NAN;
  const float inv_rows = 1.f / (float)rows;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int c = threadIdx.x + j * NT;
    T4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float p = __expf(x[j][e] - lse);
      if (c * 4 + e == tgt) p -= 1.f;
      o[e] = from_f32<T>(p * inv_rows);
    }
    if (j < CH - 1 || last_ok) *reinterpret_cast<T4*>(dzr + c * 4) = o;
  }
}

// loss = (1/rows) * sum_r row_loss[r]; one workgroup, fixed order.
__global__ __launch_bounds__(kThreads) void mean_rows_kernel(const float* __restrict__ row_loss, int rows,
                                                             float* __restrict__ loss) {
  __shared__ float red[kWaves];
  float s = 0.f;
  for (int r = threadIdx.x; r < rows; r += kThreads) s += row_loss[r];
  s = block_sum<kWaves>(s, red);
  if (threadIdx.x == 0) *loss = s / (float)rows;
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(u32x4* __restrict__ p, size_t n16) {
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += (size_t)gridDim.x * kThreads)
    p[i] = z;
}

// ---- parameter update after gradient accumulation (Section 3.1: apply_gradient) -----------
// Four consecutive elements per thread.  SGD works on the stored parameters; AdamW keeps fp32
// master weights and moments and rounds the master weights into the storage type.
template <typename T>
__global__ __launch_bounds__(kThreads) void sgd_kernel(T* __restrict__ w, const float* __restrict__ g, size_t n4,
                                                       float lr, float wd) {
  typedef T T4 __attribute__((ext_vector_type(4)));
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    const f32x4 gv = reinterpret_cast<const f32x4*>(g)[i];
    T4 wv = reinterpret_cast<T4*>(w)[i];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x = (float)wv[e];
      wv[e] = (T)(x - lr * (gv[e] + wd * x));
    }
    reinterpret_cast<T4*>(w)[i] = wv;
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void adamw_kernel(T* __restrict__ w, float* __restrict__ master,
                                                         float* __restrict__ m, float* __restrict__ v,
                                                         const float* __restrict__ g, size_t n4, float lr, float b1,
                                                         float b2, float eps, float wd, float c1, float c2) {
  typedef T T4 __attribute__((ext_vector_type(4)));
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    const f32x4 gv = reinterpret_cast<const f32x4*>(g)[i];
    f32x4 mv = reinterpret_cast<f32x4*>(m)[i], vv = reinterpret_cast<f32x4*>(v)[i];
    f32x4 x = reinterpret_cast<f32x4*>(master)[i];
    T4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      mv[e] = b1 * mv[e] + (1.f - b1) * gv[e];
      vv[e] = b2 * vv[e] + (1.f - b2) * gv[e] * gv[e];
      const float mh = mv[e] * c1, vh = vv[e] * c2;      // c1 = 1 / (1 - b1^t), c2 = 1 / (1 - b2^t)
      x[e] = x[e] - lr * (mh / (sqrtf(vh) + eps) + wd * x[e]);
      out[e] = (T)x[e];
    }
    reinterpret_cast<f32x4*>(m)[i] = mv;
    reinterpret_cast<f32x4*>(v)[i] = vv;
    reinterpret_cast<f32x4*>(master)[i] = x;
    reinterpret_cast<T4*>(w)[i] = out;
  }
}

// master <- (float) w
template <typename T>
__global__ __launch_bounds__(kThreads) void widen_kernel(const T* __restrict__ w, float* __restrict__ master, size_t n4) {
  typedef T T4 __attribute__((ext_vector_type(4)));
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    const T4 wv = reinterpret_cast<const T4*>(w)[i];
    f32x4 x;
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = (float)wv[e];
    reinterpret_cast<f32x4*>(master)[i] = x;
  }
}

// Token embedding, forward: row t of x is row tok[t] of the table E [vocab, d] (an id outside
// [0, vocab) gives a zero row).  One workgroup per token, 16-byte chunks.
template <typename T>
__global__ __launch_bounds__(kThreads) void embed_fwd_kernel(const int32_t* __restrict__ tok, const T* __restrict__ E,
                                                             T* __restrict__ x, int d, int vocab) {
  const int t = blockIdx.x;
  const int id = tok[t];
  const int n16 = d * (int)sizeof(T) / 16;
  const u32x4* src = reinterpret_cast<const u32x4*>(E + (size_t)id * d);
  u32x4* dst = reinterpret_cast<u32x4*>(x + (size_t)t * d);
  if (id >= 0 && id < vocab) {   // the row is only addressed when the id is inside the table
    for (int c = threadIdx.x; c < n16; c += kThreads) dst[c] = src[c];
  } else {
    for (int c = threadIdx.x; c < n16; c += kThreads) dst[c] = u32x4{0u, 0u, 0u, 0u};
  }
}

// Token embedding, backward: G[id] += sum over the positions t with tok[t] == id, in
// ascending t, of dx[t].  One workgroup per position; the workgroup of an id's first
// occurrence does all the work for that id, every other one leaves at once, so each row of G
// has a single writer and a fixed order of additions (no float atomics).  The positions of
// the id are first marked in a bitmap in LDS (rows bits, dynamic), then walked in order.
template <typename T>
__global__ __launch_bounds__(kThreads) void embed_bwd_kernel(const int32_t* __restrict__ tok, const T* __restrict__ dx,
                                                             float* __restrict__ G, int rows, int d, int vocab) {
  constexpr int kCols = 8;   // columns per thread and pass
  extern __shared__ uint32_t marks[];
  __shared__ int seen_before;
  const int t = blockIdx.x;
  const int id = tok[t];
  if (id < 0 || id >= vocab) return;
  const int nwords = (rows + 31) / 32;
  for (int w = threadIdx.x; w < nwords; w += kThreads) marks[w] = 0u;
  if (threadIdx.x == 0) seen_before = 0;
  __syncthreads();
  for (int u = threadIdx.x; u < rows; u += kThreads) {
    if (tok[u] != id) continue;
    if (u < t) seen_before = 1;   // every writer writes the same value
    else atomicOr(&marks[u >> 5], 1u << (u & 31));
  }
  __syncthreads();
  if (seen_before) return;
  for (int c0 = threadIdx.x * kCols; c0 < d; c0 += kThreads * kCols) {
    float acc[kCols];
#pragma unroll
    for (int e = 0; e < kCols; ++e) acc[e] = 0.f;
    for (int w = t >> 5; w < nwords; ++w) {
      uint32_t m = marks[w];
      while (m) {
        const int u = w * 32 + __builtin_ctz(m);
        m &= m - 1;
        const T* r = dx + (size_t)u * d + c0;
#pragma unroll
        for (int e = 0; e < kCols; ++e)
          if (c0 + e < d) acc[e] += to_f32(r[e]);
      }
    }
    float* g = G + (size_t)id * d + c0;
#pragma unroll
    for (int e = 0; e < kCols; ++e)
      if (c0 + e < d) g[e] += acc[e];
  }
}

// The final addition of Section 3's loop-commuting rewrite for a weight used by two stages:
// both partial gradients become their sum.
__global__ __launch_bounds__(kThreads) void tied_sum_kernel(float* __restrict__ a, float* __restrict__ b, size_t n4) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    const f32x4 s = reinterpret_cast<f32x4*>(a)[i] + reinterpret_cast<f32x4*>(b)[i];
    reinterpret_cast<f32x4*>(a)[i] = s;
    reinterpret_cast<f32x4*>(b)[i] = s;
  }
}

inline int grid_for(size_t items) {
  size_t g = (items + kThreads - 1) / kThreads;
  const size_t cap = 256 * 16;  // 16 workgroups per CU
  return (int)(g < 1 ? 1 : (g > cap ? cap : g));
}

template <typename T>
int pick_maxc(int d) {
  const int nchunks = d / Chunk<T>::N;
  const int per = (nchunks + kThreads - 1) / kThreads;
  return per <= 1 ? 1 : per <= 2 ? 2 : per <= 4 ? 4 : per <= 6 ? 6 : 8;
}

template <typename T>
hipError_t norm_fwd_t(int norm, int rows, int d, float eps, const void* x, const void* gamma,
                      const void* beta, void* y, float* stats, hipStream_t s) {
  const T* xp = (const T*)x; const T* gp = (const T*)gamma; const T* bp = (const T*)beta; T* yp = (T*)y;
  switch (pick_maxc<T>(d)) {
    case 1: norm_fwd_kernel<T, 1><<<rows, kThreads, 0, s>>>(xp, gp, bp, yp, stats, d, eps, norm); break;
    case 2: norm_fwd_kernel<T, 2><<<rows, kThreads, 0, s>>>(xp, gp, bp, yp, stats, d, eps, norm); break;
    case 4: norm_fwd_kernel<T, 4><<<rows, kThreads, 0, s>>>(xp, gp, bp, yp, stats, d, eps, norm); break;
    case 6: norm_fwd_kernel<T, 6><<<rows, kThreads, 0, s>>>(xp, gp, bp, yp, stats, d, eps, norm); break;
    default: norm_fwd_kernel<T, 8><<<rows, kThreads, 0, s>>>(xp, gp, bp, yp, stats, d, eps, norm); break;
  }
  return hipGetLastError();
}

template <typename T>
hipError_t norm_bwd_t(int norm, int rows, int d, const void* x, const void* gamma, const float* stats,
                      const void* dy, const void* dx_add, void* dx, float* g_gamma, float* g_beta,
                      float* partial, hipStream_t s) {
  const int nblk = colreduce_blocks(rows);
  float* pg = partial;
  float* pb = (norm == JPP_LAYERNORM && g_beta) ? partial + (size_t)nblk * d : nullptr;
  const T* xp = (const T*)x; const T* gp = (const T*)gamma; const T* dyp = (const T*)dy;
  const T* ap = (const T*)dx_add; T* dxp = (T*)dx;
  // wide form: rows of 1024 chunks and more whose two rows in flight fit the registers
  // (24 elements per thread and row: bf16 up to 12288 columns, fp32 up to 8192)
  const int nchunks = d / Chunk<T>::N;
  const int per = (nchunks + 511) / 512;
  auto go = [&](auto maxc, auto nt, auto wide, auto r) {
    constexpr int MAXC = decltype(maxc)::value, NT = decltype(nt)::value, R = decltype(r)::value;
    constexpr bool WIDE = decltype(wide)::value;
    // the unpredicated forms: narrow bf16 rows (the wide forms have no registers to spare for
    // what the scheduler then keeps in flight; the fp32 path is the parity path)
    if constexpr (std::is_same<T, bf16>::value && !WIDE && MAXC <= 2) {
      if (nchunks == MAXC * NT && rows % (R * nblk) == 0) {
        if (ap)
          norm_bwd_kernel<T, MAXC, NT, WIDE, R, 2><<<nblk, NT, 0, s>>>(xp, gp, stats, dyp, ap, dxp, pg, pb, rows, d, norm);
        else
          norm_bwd_kernel<T, MAXC, NT, WIDE, R, 1><<<nblk, NT, 0, s>>>(xp, gp, stats, dyp, ap, dxp, pg, pb, rows, d, norm);
        return;
      }
    }
    norm_bwd_kernel<T, MAXC, NT, WIDE, R, 0><<<nblk, NT, 0, s>>>(xp, gp, stats, dyp, ap, dxp, pg, pb, rows, d, norm);
  };
  using std::integral_constant;
  typedef integral_constant<int, 512> W512;
  typedef integral_constant<int, kThreads> W256;
  typedef integral_constant<int, 1> One;
  if (nchunks >= 1024 && per * Chunk<T>::N <= 24) {
    if (per <= 2) go(integral_constant<int, 2>{}, W512{}, std::true_type{}, One{});
    else if (per == 3) go(integral_constant<int, 3>{}, W512{}, std::true_type{}, One{});
    else go(integral_constant<int, 4>{}, W512{}, std::true_type{}, One{});
  } else
  switch (pick_maxc<T>(d)) {
    case 1: go(integral_constant<int, 1>{}, W256{}, std::false_type{}, integral_constant<int, 4>{}); break;
    case 2: go(integral_constant<int, 2>{}, W256{}, std::false_type{}, integral_constant<int, 2>{}); break;
    case 4: go(integral_constant<int, 4>{}, W256{}, std::false_type{}, One{}); break;
    case 6: go(integral_constant<int, 6>{}, W256{}, std::false_type{}, One{}); break;
    default: go(integral_constant<int, 8>{}, W256{}, std::false_type{}, One{}); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int fin = (d + kFinCols - 1) / kFinCols;
  colreduce_finish_kernel<<<dim3(fin, pb ? 2 : 1), kThreads, 0, s>>>(pg, nblk, d, g_gamma, pb, g_beta);
  return hipGetLastError();
}

}  // namespace

bool norm_shape_ok(int dtype, int d) {
  const int n = dtype == JPP_BF16 ? 8 : 4;
  return d > 0 && d % n == 0 && d / n <= kThreads * kNormMaxChunksPerThread;
}

int colreduce_blocks(int rows) { return rows < 256 ? rows : 256; }

hipError_t launch_norm_fwd(int dtype, int norm, int rows, int d, float eps, const void* x, const void* gamma,
                           const void* beta, void* y, float* stats, hipStream_t s) {
  if (norm == JPP_RMSNORM) beta = nullptr;
  return dtype == JPP_BF16 ? norm_fwd_t<bf16>(norm, rows, d, eps, x, gamma, beta, y, stats, s)
                           : norm_fwd_t<float>(norm, rows, d, eps, x, gamma, beta, y, stats, s);
}

hipError_t launch_norm_bwd(int dtype, int norm, int rows, int d, const void* x, const void* gamma,
                           const float* stats, const void* dy, const void* dx_add, void* dx, float* g_gamma,
                           float* g_beta, float* partial, hipStream_t s) {
  return dtype == JPP_BF16
             ? norm_bwd_t<bf16>(norm, rows, d, x, gamma, stats, dy, dx_add, dx, g_gamma, g_beta, partial, s)
             : norm_bwd_t<float>(norm, rows, d, x, gamma, stats, dy, dx_add, dx, g_gamma, g_beta, partial, s);
}

hipError_t launch_bias_grad(int dtype, int rows, int n, const void* dy, int ld, float* g, float* partial,
                            hipStream_t s) {
  const int nblk = colreduce_blocks(rows);
  const int N = dtype == JPP_BF16 ? 8 : 4;
  const int chunks = n / N;
  dim3 grid((chunks + kThreads - 1) / kThreads, nblk);
  if (dtype == JPP_BF16)
    colsum_partial_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)dy, ld, rows, n, partial);
  else
    colsum_partial_kernel<float><<<grid, kThreads, 0, s>>>((const float*)dy, ld, rows, n, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  colreduce_finish_kernel<<<(n + kFinCols - 1) / kFinCols, kThreads, 0, s>>>(partial, nblk, n, g);
  return hipGetLastError();
}

namespace {
// x: 256 chunks of a row per workgroup; y: as many row groups as keep about 16 workgroups per CU
dim3 act_grid(int dtype, int rows, int f) {
  const int N = dtype == JPP_BF16 ? 8 : 4;
  const int gx = (f / N + kThreads - 1) / kThreads;
  int gy = (rows + kActRows - 1) / kActRows;
  const int cap = (256 * 16 + gx - 1) / gx;
  if (gy > cap) gy = cap;
  return dim3(gx, gy < 1 ? 1 : gy);
}

template <typename T>
void act_fwd_t(int act, int rows, int f, const void* h, void* a, dim3 grid, hipStream_t s) {
  const T* hp = (const T*)h; T* ap = (T*)a;
  if (act == JPP_SWIGLU) act_fwd_kernel<T, JPP_SWIGLU><<<grid, kThreads, 0, s>>>(hp, ap, rows, f);
  else if (act == JPP_GELU) act_fwd_kernel<T, JPP_GELU><<<grid, kThreads, 0, s>>>(hp, ap, rows, f);
  else act_fwd_kernel<T, JPP_GELU_TANH><<<grid, kThreads, 0, s>>>(hp, ap, rows, f);
}

template <typename T>
void act_bwd_t(int act, int rows, int f, const void* h, const void* da, void* dh, dim3 grid, hipStream_t s) {
  const T* hp = (const T*)h; const T* dp = (const T*)da; T* op = (T*)dh;
  if (act == JPP_SWIGLU) act_bwd_kernel<T, JPP_SWIGLU><<<grid, kThreads, 0, s>>>(hp, dp, op, rows, f);
  else if (act == JPP_GELU) act_bwd_kernel<T, JPP_GELU><<<grid, kThreads, 0, s>>>(hp, dp, op, rows, f);
  else act_bwd_kernel<T, JPP_GELU_TANH><<<grid, kThreads, 0, s>>>(hp, dp, op, rows, f);
}
}  // namespace

hipError_t launch_act_fwd(int dtype, int act, int rows, int f, const void* h, void* a, hipStream_t s) {
  const dim3 grid = act_grid(dtype, rows, f);
  if (dtype == JPP_BF16) act_fwd_t<bf16>(act, rows, f, h, a, grid, s);
  else act_fwd_t<float>(act, rows, f, h, a, grid, s);
  return hipGetLastError();
}

hipError_t launch_act_bwd(int dtype, int act, int rows, int f, const void* h, const void* da, void* dh,
                          hipStream_t s) {
  const dim3 grid = act_grid(dtype, rows, f);
  if (dtype == JPP_BF16) act_bwd_t<bf16>(act, rows, f, h, da, dh, grid, s);
  else act_bwd_t<float>(act, rows, f, h, da, dh, grid, s);
  return hipGetLastError();
}

hipError_t launch_rope_table(float* table, int seq, int hd, float theta, hipStream_t s) {
  const int n = seq * (hd / 2);
  rope_table_kernel<<<(n + 255) / 256, 256, 0, s>>>(table, seq, hd, (double)theta);
  return hipGetLastError();
}

hipError_t launch_rope(int dtype, int mb, int seq, int Hq, int Hkv, int hd, void* qkv, const float* table,
                       bool inverse, hipStream_t s) {
  const int N = dtype == JPP_BF16 ? 8 : 4;
  const int heads = Hq + Hkv;  // q heads followed by k heads are contiguous in the fused tensor
  const int ld = (Hq + 2 * Hkv) * hd;
  const int tokens = mb * seq;
  const int grid = grid_for((size_t)tokens * heads * (hd / 2 / N));
  const float sign = inverse ? -1.f : 1.f;
  if (dtype == JPP_BF16)
    rope_kernel<bf16><<<grid, kThreads, 0, s>>>((bf16*)qkv, table, tokens, seq, heads, hd, ld, sign);
  else
    rope_kernel<float><<<grid, kThreads, 0, s>>>((float*)qkv, table, tokens, seq, heads, hd, ld, sign);
  return hipGetLastError();
}

// Launches cross_entropy_reg_kernel<T, per, NT, MW> for per in 1..sizeof...(I); false if per is not among them.
template <int NT, int MW, int... I>
static bool launch_ce_reg(std::integer_sequence<int, I...>, int per, int dtype, int rows, int vocab, const float* z,
                          const int32_t* targets, void* dz, float* row_loss, hipStream_t s) {
  auto go = [&](auto ch) {
    constexpr int CH = decltype(ch)::value;
    if (dtype == JPP_BF16)
      cross_entropy_reg_kernel<bf16, CH, NT, MW><<<rows, NT, 0, s>>>(z, targets, (bf16*)dz, row_loss, rows, vocab);
    else
      cross_entropy_reg_kernel<float, CH, NT, MW><<<rows, NT, 0, s>>>(z, targets, (float*)dz, row_loss, rows, vocab);
    return true;
  };
  return ((per == I + 1 && go(std::integral_constant<int, I + 1>{})) || ...);
}

hipError_t launch_cross_entropy(int dtype, int rows, int vocab, const float* z, const int32_t* targets,
                                void* dz, float* row_loss, float* loss, hipStream_t s) {
  const int chunks = vocab / 4;   // chunks of four logits
  const int per512 = (chunks + 511) / 512, per1024 = (chunks + 1023) / 1024;
  if (vocab % 4 == 0 && vocab > 0 && per512 <= 25) {
    // 512 threads hold a row in at most 100 registers each: two rows are resident per compute unit
    // (4 waves per SIMD, 128 registers per lane), so one row's loads overlap the other's stores
    launch_ce_reg<512, 4>(std::make_integer_sequence<int, 25>{}, per512, dtype, rows, vocab, z, targets, dz, row_loss,
                          s);
  } else if (vocab % 4 == 0 && vocab > 0 && per1024 <= 16) {
    // one row per compute unit in the registers of 1024 threads
    launch_ce_reg<1024, 1>(std::make_integer_sequence<int, 16>{}, per1024, dtype, rows, vocab, z, targets, dz,
                           row_loss, s);
  } else if (dtype == JPP_BF16) {
    cross_entropy_kernel<bf16><<<rows, kThreads, 0, s>>>(z, targets, (bf16*)dz, row_loss, rows, vocab);
  } else {
    cross_entropy_kernel<float><<<rows, kThreads, 0, s>>>(z, targets, (float*)dz, row_loss, rows, vocab);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  mean_rows_kernel<<<1, kThreads, 0, s>>>(row_loss, rows, loss);
  return hipGetLastError();
}

hipError_t launch_sgd(int dtype, void* w, const float* g, size_t n, float lr, float wd, hipStream_t s) {
  const size_t n4 = n / 4;   // parameter buffers are padded to multiples of 8 elements
  if (dtype == JPP_BF16) sgd_kernel<bf16><<<grid_for(n4), kThreads, 0, s>>>((bf16*)w, g, n4, lr, wd);
  else sgd_kernel<float><<<grid_for(n4), kThreads, 0, s>>>((float*)w, g, n4, lr, wd);
  return hipGetLastError();
}

hipError_t launch_adamw(int dtype, void* w, float* master, float* m, float* v, const float* g, size_t n, float lr,
                        float b1, float b2, float eps, float wd, int step, hipStream_t s) {
  const size_t n4 = n / 4;
  // bias corrections in double on the host: 1 - b^t loses digits in fp32 for b close to 1
  const float c1 = (float)(1.0 / (1.0 - pow((double)b1, step))), c2 = (float)(1.0 / (1.0 - pow((double)b2, step)));
  if (dtype == JPP_BF16)
    adamw_kernel<bf16><<<grid_for(n4), kThreads, 0, s>>>((bf16*)w, master, m, v, g, n4, lr, b1, b2, eps, wd, c1, c2);
  else
    adamw_kernel<float><<<grid_for(n4), kThreads, 0, s>>>((float*)w, master, m, v, g, n4, lr, b1, b2, eps, wd, c1, c2);
  return hipGetLastError();
}

hipError_t launch_widen(int dtype, const void* w, float* master, size_t n, hipStream_t s) {
  const size_t n4 = n / 4;
  if (dtype == JPP_BF16) widen_kernel<bf16><<<grid_for(n4), kThreads, 0, s>>>((const bf16*)w, master, n4);
  else widen_kernel<float><<<grid_for(n4), kThreads, 0, s>>>((const float*)w, master, n4);
  return hipGetLastError();
}

hipError_t launch_embed_fwd(int dtype, int rows, int d, int vocab, const int32_t* tok, const void* E, void* x,
                            hipStream_t s) {
  if (dtype == JPP_BF16) embed_fwd_kernel<bf16><<<rows, kThreads, 0, s>>>(tok, (const bf16*)E, (bf16*)x, d, vocab);
  else embed_fwd_kernel<float><<<rows, kThreads, 0, s>>>(tok, (const float*)E, (float*)x, d, vocab);
  return hipGetLastError();
}

hipError_t launch_embed_bwd(int dtype, int rows, int d, int vocab, const int32_t* tok, const void* dx, float* G,
                            hipStream_t s) {
  const size_t lds = (size_t)((rows + 31) / 32) * sizeof(uint32_t);
  if (lds > 48 * 1024) return hipErrorInvalidValue;   // 393216 tokens per microbatch
  if (dtype == JPP_BF16) embed_bwd_kernel<bf16><<<rows, kThreads, lds, s>>>(tok, (const bf16*)dx, G, rows, d, vocab);
  else embed_bwd_kernel<float><<<rows, kThreads, lds, s>>>(tok, (const float*)dx, G, rows, d, vocab);
  return hipGetLastError();
}

hipError_t launch_tied_sum(float* a, float* b, size_t n, hipStream_t s) {
  const size_t n4 = n / 4;
  tied_sum_kernel<<<grid_for(n4), kThreads, 0, s>>>(a, b, n4);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;  // callers pass 16-byte multiples (arena regions are 256-byte aligned)
  if (n16 == 0) return hipSuccess;
  fill_zero_kernel<<<grid_for(n16), kThreads, 0, s>>>((u32x4*)p, n16);
  return hipGetLastError();
}

}  // namespace jpp
