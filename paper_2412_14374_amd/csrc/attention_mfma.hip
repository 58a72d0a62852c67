// Fused causal self-attention on the gfx950 matrix cores, bf16 storage, head_dim 128.
//
// Definition (per batch element b, query head h, kv head g = h / (Hq/Hkv)):
//   S[t,u] = q_t . k_u / sqrt(hd) for u <= t;  P = softmax_u(S);  O_t = sum_u P[t,u] v_u
//   lse[t] = log sum_u exp(S[t,u])
//   backward, D_t = dO_t . O_t:  dP = dO V^T;  dS = P * (dP - D);  dV = P^T dO;
//   dQ = dS K / sqrt(hd);  dK = dS^T Q / sqrt(hd); dK, dV of a shared kv head sum over the
//   group's query heads in ascending order.
// The paper names no attention algorithm (it calls a vendor library); this is the
// online-softmax formulation with the probabilities recomputed from lse in the backward.
//
// Everything is computed "transposed": the MFMA output tile has the softmax row (one query,
// or one key in the dK/dV kernel) along the LANE axis, so that
//  * row maxima / sums need one cross-lane exchange (lanes l and l+32 share a row),
//  * the probabilities sit in exactly the register layout the next MFMA wants as its
//    B operand, so P never moves between lanes or through LDS,
//  * the per-row rescale of the output accumulator is a per-lane scalar multiply.
// The k index of an MFMA may be permuted freely as long as both operands agree; the B
// operand taken from an accumulator holds, per 16 keys, keys {0-3, 8-11} in lanes 0-31 and
// {4-7, 12-15} in lanes 32-63, so transposed operand tiles are stored in LDS with that
// order inside each group of 16 and are read with one 16-byte load per lane.
//
// Determinism: the backward uses two kernels (one owns dK/dV rows, one owns dQ rows);
// nothing is accumulated with atomics.
#include "device_utils.h"
#include "internal.h"

namespace jpp {

namespace {

constexpr int HD = 128;
constexpr int kThreads = 256;
constexpr uint32_t kOOB = 0x7FFFFFFFu;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int kTileBytes = 64 * HD * 2;
constexpr f32x16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // a 64-row tile of one head: 16 KiB in either layout

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, long long bytes) {
  const uint32_t n = bytes > 0x7FFFFF00LL ? 0x7FFFFF00u : (bytes < 0 ? 0u : (uint32_t)bytes);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)n, 0x00020000);
}

__device__ inline int swz7(int row) { return (row ^ (row >> 3)) & 7; }

// 2^x by the hardware instruction alone (arguments here are <= 0 or masked; results below the
// normal range flush to zero, which is what the sums want).  The library exp2f wraps the same
// instruction in range scaling that triples its cost.
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- tile staging ------------------------------------------------------------------------
// "Row" tile: [64 rows][128 d], 256 bytes per row (one line of the 64 x 4-byte LDS banks), 16-byte
// chunk c stored at c ^ (row & 15): 16 consecutive rows reading the same logical chunk hit 16
// different bank quads.
// Filled HBM -> LDS directly: each wave instruction fills 4 rows (1 KiB) in lane order.
// `base` points at (row 0, d 0) of the tile in global memory, `ld` is the row pitch in
// elements, rows >= valid read as zero.
__device__ inline void load_row_tile(char* tile, const bf16* base, int ld, int valid, long long bytes_left) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
  const auto rs = make_rsrc(base, bytes_left);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int blk = wave * 4 + i;               // 4-row block index, 16 per tile
    const int row = blk * 4 + (lane >> 4);
    const int c = (lane & 15) ^ (row & 15);
    const uint32_t off = row < valid ? (uint32_t)(row * ld + c * 8) * 2u : kOOB;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(tile + blk * 1024), 16, (int)off, 0, 0, 0);
  }
}

// "Transposed" tile: [128 d][64 rows], 128 bytes per d, rows permuted inside each group of 16
// (bits 2 and 3 of the row index swapped), 16-byte chunk c stored at c ^ swz7(d).
// A thread loads 4 rows x 8 d (four 16-byte loads) into registers; from there the block is
// written as four 16-byte chunks of a row tile (store_rows) or, transposed in registers, as
// eight 8-byte runs of 4 rows of a transposed tile (store).  Issuing the loads of the next
// tile before the current one is multiplied hides the memory latency behind the MFMAs.
struct TransposedStage {
  u32x4 regs[4];
  __device__ inline void issue(const bf16* base, int ld, int valid, long long bytes_left) {
    const auto rs = make_rsrc(base, bytes_left);
    const int db = threadIdx.x & 15, rg = threadIdx.x >> 4;  // d block (8 wide), row group (4 rows)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = rg * 4 + j;
      const uint32_t off = row < valid ? (uint32_t)(row * ld + db * 8) * 2u : kOOB;
      regs[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
    }
  }
  __device__ inline void store_rows(char* tile) const {
    const int db = threadIdx.x & 15, rg = threadIdx.x >> 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = rg * 4 + j;
      *reinterpret_cast<u32x4*>(tile + row * 256 + ((db ^ (row & 15)) << 4)) = regs[j];
    }
  }
  __device__ inline void store(char* tile) const {
    const int db = threadIdx.x & 15, rg = threadIdx.x >> 4;
    const int o16 = (rg & 3) * 4;                               // row offset inside its group of 16
    const int pos16 = (o16 & 3) | ((o16 & 8) >> 1) | ((o16 & 4) << 1);
    const int chunk = (rg >> 2) * 2 + (pos16 >> 3);
    const int half8 = (pos16 >> 2) & 1;
#pragma unroll
    for (int dd = 0; dd < 8; ++dd) {
      const int w = dd >> 1;
      const uint32_t sel = (dd & 1) ? 0x07060302u : 0x05040100u;
      u32x2 v;
      v[0] = __builtin_amdgcn_perm(regs[1][w], regs[0][w], sel);
      v[1] = __builtin_amdgcn_perm(regs[3][w], regs[2][w], sel);
      const int d = db * 8 + dd;
      *reinterpret_cast<u32x2*>(tile + d * 128 + ((chunk ^ swz7(d)) << 4) + half8 * 8) = v;
    }
  }
};

// A operand from a row tile: rows mt*32 + l32, k = d chunk (2*kd + half).
__device__ inline bf16x8 row_frag(const char* tile, int mt, int kd, int l32, int half) {
  const int row = mt * 32 + l32;
  return *reinterpret_cast<const bf16x8*>(tile + row * 256 + (((kd * 2 + half) ^ (row & 15)) << 4));
}
// A operand from a transposed tile: rows (d) dt*32 + l32, k = the 16 tile-rows of step s in
// the permuted order described above.
__device__ inline bf16x8 trans_frag(const char* tile, int dt, int s, int l32, int half) {
  const int d = dt * 32 + l32;
  return *reinterpret_cast<const bf16x8*>(tile + d * 128 + (((s * 2 + half) ^ swz7(d)) << 4));
}
// B operand straight from global memory: row `row` (zero if not valid), d = 16*kd + 8*half ..
__device__ inline bf16x8 global_frag(const bf16* base, int ld, int row, bool valid, int kd, int half) {
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16)0.f;
  if (!valid) return z;
  return *reinterpret_cast<const bf16x8*>(base + (size_t)row * ld + kd * 16 + half * 8);
}
// B operand for k-step s2 (0 or 1) of a 32-row accumulator tile: registers 8*s2 .. 8*s2+7.
__device__ inline bf16x8 acc_frag(const f32x16& a, int s2) {
  bf16x8 p;
#pragma unroll
  for (int e = 0; e < 8; ++e) p[e] = (bf16)a[8 * s2 + e];
  return p;
}

// ---- forward -------------------------------------------------------------------------------
// One workgroup: 128 queries of one (b, h); wave w owns queries [32w, 32w+32).  KV tiles of 64.
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv,
                                                                 bf16* __restrict__ out,
                                                                 float* __restrict__ lse, int seq, int Hq,
                                                                 int Hkv, long long total_bytes) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * kTileBytes];
  char* k_tile = lds;
  char* vt_tile = lds + kTileBytes;
  // Heaviest blocks first over the whole launch (a late query block visits the most key
  // tiles): the block index is the slow grid dimension, (head, batch) the fast one, so the
  // launch ends with its shortest workgroups instead of a few long ones.
  const int qb = gridDim.y - 1 - blockIdx.y;
  const int h = blockIdx.x % Hq, b = blockIdx.x / Hq;
  const int g = h / (Hq / Hkv);
  const int ld = (Hq + 2 * Hkv) * HD;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, l32 = lane & 31, half = lane >> 5;
  const int q0 = qb * 128, qw0 = q0 + wave * 32;
  const size_t tok0 = (size_t)b * seq;
  const bf16* qbase = qkv + tok0 * ld + (size_t)h * HD;
  const bf16* kbase = qkv + tok0 * ld + (size_t)(Hq + g) * HD;
  const bf16* vbase = kbase + (size_t)Hkv * HD;
  const float sl2 = rsqrtf((float)HD) * kLog2e;

  bf16x8 qf[8];
  const int qrow = qw0 + l32;
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) qf[kd] = global_frag(qbase, ld, qrow, qrow < seq, kd, half);

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int q_end = min(q0 + 128, seq);      // keys needed: 0 .. q_end-1
  const int n_tiles = (q_end + 63) / 64;
  TransposedStage ks, vs;
  auto fetch = [&](int t) {
    const int kv0 = t * 64;
    const long long left_k = total_bytes - (long long)((kbase + (size_t)kv0 * ld) - qkv) * 2;
    ks.issue(kbase + (size_t)kv0 * ld, ld, seq - kv0, left_k);
    vs.issue(vbase + (size_t)kv0 * ld, ld, seq - kv0, left_k - (long long)Hkv * HD * 2);
  };
  fetch(0);
  for (int t = 0; t < n_tiles; ++t) {
    const int kv0 = t * 64;
    __syncthreads();                          // every wave is done with the previous tile
    ks.store_rows(k_tile);
    vs.store(vt_tile);
    __syncthreads();
    if (t + 1 < n_tiles) fetch(t + 1);        // in flight while this tile is multiplied
    if (kv0 > qw0 + 31) continue;             // every key of this tile is in this wave's future
    f32x16 s[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(k_tile, i, 0, l32, half), qf[0], kZero16, 0, 0, 0);
#pragma unroll
    for (int kd = 1; kd < 8; ++kd)
#pragma unroll
      for (int i = 0; i < 2; ++i)
        s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(k_tile, i, kd, l32, half), qf[kd], s[i], 0, 0, 0);
    // s[i][r] = q(qw0 + l32) . k(kv0 + 32 i + 8 (r/4) + 4 half + r%4), unscaled
    if (kv0 + 63 > qw0) {                     // only tiles that cross the diagonal need the mask
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
          if (key > qrow) s[i][r] = -INFINITY;
        }
    }
    float mx = s[0][0];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = __builtin_fmaxf(mx, s[i][r]);
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
    // the scale is positive, so it commutes with the maximum; m is kept in scaled log2 units
    const float mnew = __builtin_fmaxf(m, mx * sl2);   // finite: key kv0 <= qw0 + 31 and key 0 <= any query
    const float alpha = fast_exp2(m - mnew);
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(__builtin_fmaf(s[i][r], sl2, -mnew));
        s[i][r] = p;
        psum += p;
      }
    l = l * alpha + psum;
    m = mnew;
    if (__any(alpha != 1.f)) {                // late tiles rarely move the maximum
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    }
#pragma unroll
    for (int sk = 0; sk < 4; ++sk) {
      const bf16x8 pf = acc_frag(s[sk >> 1], sk & 1);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trans_frag(vt_tile, dt, sk, l32, half), pf, o[dt], 0, 0, 0);
    }
  }
  const float ltot = l + __shfl_xor(l, 32, 64);
  if (qrow < seq) {
    const float inv = 1.f / ltot;
    bf16* orow = out + (tok0 + qrow) * ((size_t)Hq * HD) + (size_t)h * HD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[dt][4 * gq + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + dt * 32 + 8 * gq + 4 * half) = v;
      }
    if (half == 0) lse[((size_t)b * Hq + h) * seq + qrow] = (m + log2f(ltot)) * kLn2;
  }
}

// ---- backward: D = rowsum(dO * O) ----------------------------------------------------------
__global__ __launch_bounds__(kThreads) void attn_delta_kernel(const bf16* __restrict__ out,
                                                              const bf16* __restrict__ dout,
                                                              float* __restrict__ delta, int mb, int seq, int Hq) {
  // 16 lanes per (token, head) row of 128 elements
  const size_t idx = (size_t)blockIdx.x * (kThreads / 16) + threadIdx.x / 16;
  const size_t rows = (size_t)mb * seq * Hq;
  const int sub = threadIdx.x & 15;
  float acc = 0.f;
  if (idx < rows) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(out + idx * HD + sub * 8);
    const bf16x8 d = *reinterpret_cast<const bf16x8*>(dout + idx * HD + sub * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)d[e];
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (idx < rows && sub == 0) {
    const size_t tok = idx / Hq;
    const int h = (int)(idx % Hq);
    const size_t b = tok / seq, t = tok % seq;
    delta[(b * Hq + h) * seq + t] = acc;
  }
}

// ---- backward: dK, dV ----------------------------------------------------------------------
// One workgroup: 128 keys of one (b, kv head); wave w owns keys [32w, 32w+32).  For every query
// head of the group (ascending) and every 64-query tile at or below the diagonal:
//   S = Q K^T, dP = dO V^T  (A = Q / dO row tiles from LDS, B = K / V fragments in registers)
//   P = exp(S/sqrt(hd) - lse), dS = P (dP - D)
//   dV^T += dO^T P,  dK^T += Q^T dS  (A = transposed tiles from LDS, B = P / dS from registers)
// With `partial` (grouped-query attention with a scratch buffer) a workgroup handles ONE query
// head (grid x = query heads x batch) and stores its unscaled fp32 dK and dV rows to
// partial[(b * Hq + h) * seq + key][0..127] and, mb * Hq * seq rows further, the dV rows; the
// group's heads are then summed in ascending order by attn_bwd_dkv_reduce_kernel.  Without
// it a workgroup walks the whole group of its kv head itself (grid x = kv heads x batch).
__global__ __launch_bounds__(kThreads) void attn_bwd_dkv_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16* __restrict__ dqkv, int seq, int Hq, int Hkv, long long qkv_bytes,
    long long dout_bytes, float* __restrict__ partial, long long partial_dv_offset) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];
  __shared__ float lse_s[64], delta_s[64];
  char* q_tile = lds;
  char* do_tile = lds + kTileBytes;
  char* qt_tile = lds + 2 * kTileBytes;
  char* dot_tile = lds + 3 * kTileBytes;
  // early key blocks (most query tiles) first
  const int kb = blockIdx.y;
  const int heads_x = partial ? Hq : Hkv;
  const int hx = blockIdx.x % heads_x, b = blockIdx.x / heads_x;
  const int group = Hq / Hkv;
  const int g = partial ? hx / group : hx;
  const int hh_first = partial ? hx % group : 0, hh_end = partial ? hh_first + 1 : group;
  const int ld = (Hq + 2 * Hkv) * HD, ldo = Hq * HD;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, l32 = lane & 31, half = lane >> 5;
  const int k0 = kb * 128, kw0 = k0 + wave * 32;
  const size_t tok0 = (size_t)b * seq;
  const bf16* kbase = qkv + tok0 * ld + (size_t)(Hq + g) * HD;
  const bf16* vbase = kbase + (size_t)Hkv * HD;
  const float scale = rsqrtf((float)HD);
  const float sl2 = scale * kLog2e;

  bf16x8 kf[8], vf[8];
  const int krow = kw0 + l32;
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) {
    kf[kd] = global_frag(kbase, ld, krow, krow < seq, kd, half);
    vf[kd] = global_frag(vbase, ld, krow, krow < seq, kd, half);
  }
  f32x16 dk[4], dv[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }

  const int first_tile = k0 / 64;
  const int n_tiles = (seq + 63) / 64;
  for (int hh = hh_first; hh < hh_end; ++hh) {
    const int h = g * group + hh;
    const bf16* qbase = qkv + tok0 * ld + (size_t)h * HD;
    const bf16* dobase = dout + tok0 * ldo + (size_t)h * HD;
    const float* lrow = lse + ((size_t)b * Hq + h) * seq;
    const float* drow = delta + ((size_t)b * Hq + h) * seq;
    for (int t = first_tile; t < n_tiles; ++t) {
      const int qt0 = t * 64;
      __syncthreads();
      const long long left_q = qkv_bytes - (long long)((qbase + (size_t)qt0 * ld) - qkv) * 2;
      const long long left_do = dout_bytes - (long long)((dobase + (size_t)qt0 * ldo) - dout) * 2;
      load_row_tile(q_tile, qbase + (size_t)qt0 * ld, ld, seq - qt0, left_q);
      load_row_tile(do_tile, dobase + (size_t)qt0 * ldo, ldo, seq - qt0, left_do);
      TransposedStage sq, sd;
      sq.issue(qbase + (size_t)qt0 * ld, ld, seq - qt0, left_q);
      sd.issue(dobase + (size_t)qt0 * ldo, ldo, seq - qt0, left_do);
      if (threadIdx.x < 64) {
        const int q = qt0 + threadIdx.x;
        lse_s[threadIdx.x] = q < seq ? lrow[q] * kLog2e : INFINITY;  // +inf makes P = 0 beyond the end
        delta_s[threadIdx.x] = q < seq ? drow[q] : 0.f;
      }
      sq.store(qt_tile);
      sd.store(dot_tile);
      __syncthreads();
      if (qt0 + 63 < kw0) continue;            // every query of this tile precedes this wave's keys
      f32x16 s[2], dp[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(q_tile, i, 0, l32, half), kf[0], kZero16, 0, 0, 0);
        dp[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(do_tile, i, 0, l32, half), vf[0], kZero16, 0, 0, 0);
      }
#pragma unroll
      for (int kd = 1; kd < 8; ++kd)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(q_tile, i, kd, l32, half), kf[kd], s[i], 0, 0, 0);
          dp[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(do_tile, i, kd, l32, half), vf[kd], dp[i], 0, 0, 0);
        }
      // s[i][r]: query qt0 + 32 i + 8 (r/4) + 4 half + r%4, key kw0 + l32
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int ql = 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
          s[i][r] = fast_exp2(__builtin_fmaf(s[i][r], sl2, -lse_s[ql]));
        }
      if (qt0 < kw0 + 31) {                    // only tiles that cross the diagonal need the mask
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int ql = 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
            if (qt0 + ql < krow) s[i][r] = 0.f;
          }
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int ql = 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
          dp[i][r] = s[i][r] * (dp[i][r] - delta_s[ql]);
        }
#pragma unroll
      for (int sk = 0; sk < 4; ++sk) {
        const bf16x8 pf = acc_frag(s[sk >> 1], sk & 1);
        const bf16x8 dsf = acc_frag(dp[sk >> 1], sk & 1);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trans_frag(dot_tile, dt, sk, l32, half), pf, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trans_frag(qt_tile, dt, sk, l32, half), dsf, dk[dt], 0, 0, 0);
        }
      }
    }
  }
  if (partial) {
    if (krow < seq) {
      float* pk = partial + (((size_t)b * Hq + hx) * seq + krow) * HD;
      float* pv = pk + partial_dv_offset;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          f32x4 a, c;
#pragma unroll
          for (int e = 0; e < 4; ++e) { a[e] = dk[dt][4 * gq + e]; c[e] = dv[dt][4 * gq + e]; }
          *reinterpret_cast<f32x4*>(pk + dt * 32 + 8 * gq + 4 * half) = a;
          *reinterpret_cast<f32x4*>(pv + dt * 32 + 8 * gq + 4 * half) = c;
        }
    }
    return;
  }
  if (krow < seq) {
    bf16* dkrow = dqkv + (tok0 + krow) * ld + (size_t)(Hq + g) * HD;
    bf16* dvrow = dkrow + (size_t)Hkv * HD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 a, c;
#pragma unroll
        for (int e = 0; e < 4; ++e) { a[e] = (bf16)(dk[dt][4 * gq + e] * scale); c[e] = (bf16)dv[dt][4 * gq + e]; }
        *reinterpret_cast<bf16x4*>(dkrow + dt * 32 + 8 * gq + 4 * half) = a;
        *reinterpret_cast<bf16x4*>(dvrow + dt * 32 + 8 * gq + 4 * half) = c;
      }
  }
}

// Sums the per-query-head partial dK / dV rows of a kv head in ascending head order, scales dK
// and rounds into the gradient tensor.  One thread per (token, kv head, 4 columns).
__global__ __launch_bounds__(kThreads) void attn_bwd_dkv_reduce_kernel(const float* __restrict__ partial,
                                                                       long long partial_dv_offset,
                                                                       bf16* __restrict__ dqkv, int mb, int seq, int Hq,
                                                                       int Hkv) {
  const int group = Hq / Hkv;
  const int ld = (Hq + 2 * Hkv) * HD;
  const float scale = rsqrtf((float)HD);
  const size_t total = (size_t)mb * seq * Hkv * (HD / 4);
  for (size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += (size_t)gridDim.x * kThreads) {
    const int c4 = (int)(idx % (HD / 4));
    const int g = (int)((idx / (HD / 4)) % Hkv);
    const size_t tok = idx / ((size_t)(HD / 4) * Hkv);      // b * seq + t
    const size_t b = tok / seq, t = tok % seq;
    f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    for (int hh = 0; hh < group; ++hh) {
      const float* pk = partial + ((b * Hq + (size_t)(g * group + hh)) * seq + t) * HD + c4 * 4;
      sk += *reinterpret_cast<const f32x4*>(pk);
      sv += *reinterpret_cast<const f32x4*>(pk + partial_dv_offset);
    }
    bf16x4 ok, ov;
#pragma unroll
    for (int e = 0; e < 4; ++e) { ok[e] = (bf16)(sk[e] * scale); ov[e] = (bf16)sv[e]; }
    bf16* row = dqkv + tok * ld + (size_t)(Hq + g) * HD + c4 * 4;
    *reinterpret_cast<bf16x4*>(row) = ok;
    *reinterpret_cast<bf16x4*>(row + (size_t)Hkv * HD) = ov;
  }
}

// ---- backward: dQ --------------------------------------------------------------------------
// One workgroup: 128 queries of one (b, h); wave w owns queries [32w, 32w+32).  KV tiles of 64:
//   S^T = K Q^T, dP^T = V dO^T (A = K / V row tiles from LDS, B = Q / dO fragments in registers)
//   dS^T = P^T (dP^T - D);  dQ^T += K^T dS^T (A = transposed K tile)
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16* __restrict__ dqkv, int seq, int Hq, int Hkv, long long qkv_bytes) {
  __shared__ __attribute__((aligned(1024))) char lds[3 * kTileBytes];
  char* k_tile = lds;
  char* v_tile = lds + kTileBytes;
  char* kt_tile = lds + 2 * kTileBytes;
  const int qb = gridDim.y - 1 - blockIdx.y;   // heaviest first, as in the forward kernel
  const int h = blockIdx.x % Hq, b = blockIdx.x / Hq;
  const int g = h / (Hq / Hkv);
  const int ld = (Hq + 2 * Hkv) * HD, ldo = Hq * HD;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, l32 = lane & 31, half = lane >> 5;
  const int q0 = qb * 128, qw0 = q0 + wave * 32;
  const size_t tok0 = (size_t)b * seq;
  const bf16* qbase = qkv + tok0 * ld + (size_t)h * HD;
  const bf16* dobase = dout + tok0 * ldo + (size_t)h * HD;
  const bf16* kbase = qkv + tok0 * ld + (size_t)(Hq + g) * HD;
  const bf16* vbase = kbase + (size_t)Hkv * HD;
  const float scale = rsqrtf((float)HD);
  const float sl2 = scale * kLog2e;

  const int qrow = qw0 + l32;
  const bool q_ok = qrow < seq;
  bf16x8 qf[8], dof[8];
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) {
    qf[kd] = global_frag(qbase, ld, qrow, q_ok, kd, half);
    dof[kd] = global_frag(dobase, ldo, qrow, q_ok, kd, half);
  }
  const float lse2 = q_ok ? lse[((size_t)b * Hq + h) * seq + qrow] * kLog2e : INFINITY;
  const float dlt = q_ok ? delta[((size_t)b * Hq + h) * seq + qrow] : 0.f;
  f32x16 dq[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;

  const int q_end = min(q0 + 128, seq);
  const int n_tiles = (q_end + 63) / 64;
  for (int t = 0; t < n_tiles; ++t) {
    const int kv0 = t * 64;
    __syncthreads();
    const long long left_k = qkv_bytes - (long long)((kbase + (size_t)kv0 * ld) - qkv) * 2;
    load_row_tile(k_tile, kbase + (size_t)kv0 * ld, ld, seq - kv0, left_k);
    load_row_tile(v_tile, vbase + (size_t)kv0 * ld, ld, seq - kv0, left_k - (long long)Hkv * HD * 2);
    TransposedStage ks;
    ks.issue(kbase + (size_t)kv0 * ld, ld, seq - kv0, left_k);
    ks.store(kt_tile);
    __syncthreads();
    if (kv0 > qw0 + 31) continue;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(k_tile, i, 0, l32, half), qf[0], kZero16, 0, 0, 0);
      dp[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(v_tile, i, 0, l32, half), dof[0], kZero16, 0, 0, 0);
    }
#pragma unroll
    for (int kd = 1; kd < 8; ++kd)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(k_tile, i, kd, l32, half), qf[kd], s[i], 0, 0, 0);
        dp[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(v_tile, i, kd, l32, half), dof[kd], dp[i], 0, 0, 0);
      }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[i][r] = fast_exp2(__builtin_fmaf(s[i][r], sl2, -lse2));
    if (kv0 + 63 > qw0) {                     // only tiles that cross the diagonal need the mask
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
          if (key > qrow) s[i][r] = 0.f;
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) dp[i][r] = s[i][r] * (dp[i][r] - dlt);
#pragma unroll
    for (int sk = 0; sk < 4; ++sk) {
      const bf16x8 dsf = acc_frag(dp[sk >> 1], sk & 1);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
        dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trans_frag(kt_tile, dt, sk, l32, half), dsf, dq[dt], 0, 0, 0);
    }
  }
  if (q_ok) {
    bf16* dqrow = dqkv + (tok0 + qrow) * ld + (size_t)h * HD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[dt][4 * gq + e] * scale);
        *reinterpret_cast<bf16x4*>(dqrow + dt * 32 + 8 * gq + 4 * half) = v;
      }
  }
}

}  // namespace

bool attention_mfma_supported(const AttnDesc& a) { return a.hd == HD; }

size_t attention_bwd_scratch_bytes(int mb, int seq, int Hq, int Hkv, int hd) {
  if (hd != HD || Hq <= Hkv) return 0;
  return (size_t)2 * mb * Hq * seq * HD * sizeof(float);
}

hipError_t launch_attention_fwd_mfma(const AttnDesc& a, hipStream_t s) {
  dim3 grid(a.Hq * a.mb, (a.seq + 127) / 128);
  const long long bytes = (long long)a.mb * a.seq * (a.Hq + 2 * a.Hkv) * HD * 2;
  attn_fwd_mfma_kernel<<<grid, kThreads, 0, s>>>((const bf16*)a.qkv, (bf16*)a.out, a.lse, a.seq, a.Hq, a.Hkv, bytes);
  return hipGetLastError();
}

hipError_t launch_attention_bwd_mfma(const AttnDesc& a, hipStream_t s) {
  const long long qkv_bytes = (long long)a.mb * a.seq * (a.Hq + 2 * a.Hkv) * HD * 2;
  const long long do_bytes = (long long)a.mb * a.seq * a.Hq * HD * 2;
  const size_t rows = (size_t)a.mb * a.seq * a.Hq;
  attn_delta_kernel<<<(unsigned)((rows + 15) / 16), kThreads, 0, s>>>((const bf16*)a.out, (const bf16*)a.dout,
                                                                      a.delta, a.mb, a.seq, a.Hq);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // Grouped-query attention: a kv head's workgroups walk all its query heads, few and long
  // workgroups that a causal launch cannot balance (Llama-70B shape: 256 workgroups of 16 to
  // 512 tiles).  With scratch the query heads are spread over workgroups and summed afterwards.
  const bool split = a.dkv_partial != nullptr && a.Hq > a.Hkv;
  const long long dv_off = (long long)a.mb * a.Hq * a.seq * HD;
  dim3 gk((split ? a.Hq : a.Hkv) * a.mb, (a.seq + 127) / 128);
  attn_bwd_dkv_mfma_kernel<<<gk, kThreads, 0, s>>>((const bf16*)a.qkv, (const bf16*)a.dout, a.lse, a.delta,
                                                   (bf16*)a.dqkv, a.seq, a.Hq, a.Hkv, qkv_bytes, do_bytes,
                                                   split ? a.dkv_partial : nullptr, dv_off);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (split) {
    const size_t items = (size_t)a.mb * a.seq * a.Hkv * (HD / 4);
    const size_t blocks = (items + kThreads - 1) / kThreads;
    attn_bwd_dkv_reduce_kernel<<<(unsigned)(blocks < 8192 ? blocks : 8192), kThreads, 0, s>>>(
        a.dkv_partial, dv_off, (bf16*)a.dqkv, a.mb, a.seq, a.Hq, a.Hkv);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  dim3 gq(a.Hq * a.mb, (a.seq + 127) / 128);
  attn_bwd_dq_mfma_kernel<<<gq, kThreads, 0, s>>>((const bf16*)a.qkv, (const bf16*)a.dout, a.lse, a.delta,
                                                  (bf16*)a.dqkv, a.seq, a.Hq, a.Hkv, qkv_bytes);
  return hipGetLastError();
}

}  // namespace jpp
