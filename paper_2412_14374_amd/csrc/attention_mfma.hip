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
// {4-7, 12-15} in lanes 32-63.
//
// Tiles.  Every operand tile (64 rows of one head: K, V, Q or dO) is staged ONCE, as it lies in
// memory ([row][128 d], 256 bytes per row), by HBM -> LDS direct loads into one of two tile
// sets: the next step's tiles arrive while the current step is multiplied, no register and no
// second pass over the tile is spent on staging, and a step has one barrier.  The two operand
// shapes an MFMA wants are both read from that one tile:
//  * rows along the MFMA's M index (S = Q K^T, dP = dO V^T): one 16-byte read per lane;
//  * the head dimension along M (O^T += V^T P^T, dV^T += dO^T P, dK^T += Q^T dS, dQ^T += K^T dS^T):
//    two transposing reads per lane (ds_read_b64_tr_b16: lane i of a 16-lane group receives
//    element (i & 3) of the 8-byte runs that lanes 4j + (i >> 2), j = 0..3, address), each
//    returning 4 consecutive tile rows for the lane's d, which is the key order above.
// The 16-byte chunk c of row r is stored at chunk c ^ swz16(r): 16 consecutive rows reading
// one logical chunk (first shape) hit 16 different bank quads, and the 4 rows x 64 bytes that
// 32 lanes read together in the second shape go to four different 64-byte bank groups.
//
// Determinism: the backward uses two kernels (one owns dK/dV rows, one owns dQ rows);
// nothing is accumulated with atomics.
#include "device_utils.h"
#include "internal.h"

namespace jpp {

namespace {

constexpr int HD = 128;
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_t;

constexpr int kTileBytes = 64 * HD * 2;   // a 64-row tile of one head: 16 KiB
constexpr f32x16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

// chunk swizzle of a tile row: bits 0-1 of the row go to bits 2-3 of the chunk index, bits 2-3
// to bits 0-1 (a bijection of 0..15 for 16 consecutive rows)
__device__ inline int swz16(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// 2^x by the hardware instruction alone (arguments here are <= 0 or masked; results below the
// normal range flush to zero, which is what the sums want).  The library exp2f wraps the same
// instruction in range scaling that triples its cost.
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- tile staging ------------------------------------------------------------------------
// Raw buffer descriptor (base, stride 0, num_records = bytes, untyped 32-bit format) in scalar
// registers, for the HBM -> LDS loads below.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ inline i32x4 make_rsrc_s(const void* p, long long bytes) {
  const uint32_t n = bytes > 0x7FFFFF00LL ? 0x7FFFFF00u : (bytes < 0 ? 0u : (uint32_t)bytes);
  const unsigned long long a = (unsigned long long)p;
  i32x4 r;
  r[0] = (int)(uint32_t)a;
  r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);
  r[2] = (int)n;
  r[3] = 0x00020000;
  return r;
}
// 16 bytes per lane, HBM -> LDS without passing through registers: the wave's 64 lanes fill the
// 1 KiB at LDS byte address `lds_addr` in lane order; lanes whose byte offset `voff` is outside
// the descriptor's range store zeros.  Inline assembly on purpose: the compiler's wait-count
// pass makes every LDS read that follows such a load wait for ALL loads in flight (it cannot
// tell the tile set being filled from the one being read), which would put the whole memory
// latency back in front of every step.  The one wait a step needs is in step_barrier().
__device__ inline void dma16(const i32x4& rsrc, uint32_t lds_addr, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rsrc)
               : "memory", "m0");
}
__device__ inline uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const char*)p;
}
// The barrier between two steps: this wave's loads into LDS have landed and its LDS writes are
// done (the counters), then every wave's (the barrier).  Also a compiler-level memory barrier.
__device__ inline void step_barrier() {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Makes the compiler wait HERE for the load that produces `v` (an empty statement that reads
// it).  Used on the fragments fetched before a step loop: a load still pending at the loop's
// entry would otherwise be waited for with vmcnt(0) at its first use inside the loop, in every
// iteration, and that wait would also cover the HBM -> LDS loads issued just before it.
__device__ inline void settle(const bf16x8& v) { asm volatile("" ::"v"(v)); }
__device__ inline void settle(float v) { asm volatile("" ::"v"(v)); }
// Keeps an accumulator tile in the accumulation half of the register file at this point.
__device__ inline void pin_agpr(f32x16& v) { asm volatile("" : "+a"(v)); }

// Fills tiles HBM -> LDS: each wave instruction fills 4 rows (1 KiB) of the tile in lane order,
// so the swizzle is applied to WHICH chunk of the row a lane fetches.  The per-lane byte
// offsets depend only on the row pitch and are computed once; a tile then costs a few scalar
// instructions (its descriptor) and four loads per thread, in flight until the next
// step_barrier().  Rows at and beyond `valid` read as zero: the descriptor ends with row
// valid - 1, and the hardware returns zero beyond a descriptor's range.
struct TileLoader {
  uint32_t voff[4];
  int ld;
  __device__ inline void init(int ld_elems) {
    ld = ld_elems;
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (wave * 4 + i) * 4 + (lane >> 4);
      const int c = (lane & 15) ^ swz16(row);
      voff[i] = (uint32_t)(row * ld + c * 8) * 2u;
    }
  }
  // `base`: (row 0, d 0) of the tile in global memory; 1 <= valid rows (more than 64 count as 64)
  __device__ inline void issue(char* tile, const bf16* base, int valid) const {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int rows = valid < 64 ? valid : 64;
    const i32x4 rs = make_rsrc_s(base, ((long long)(rows - 1) * ld + HD) * 2);
    const uint32_t t0 = lds_addr_of(tile) + wave * 4096;
#pragma unroll
    for (int i = 0; i < 4; ++i) dma16(rs, t0 + i * 1024, voff[i]);
  }
};

// A operand with tile rows along M: rows mt*32 + l32, k = d chunk (2*kd + half).
__device__ inline bf16x8 row_frag(const char* tile, int mt, int kd, int l32, int half) {
  const int row = mt * 32 + l32;
  return *reinterpret_cast<const bf16x8*>(tile + row * 256 + (((kd * 2 + half) ^ swz16(row)) << 4));
}

// A operand with the head dimension along M, read from the same tile by transposing reads.
// For lane (l32, half), M row d = 32 dt + l32 and k-step s (16 tile rows) the operand holds
// tile rows 16 s + 4 half + 0..3 and 16 s + 8 + 4 half + 0..3 (the order of an accumulator
// used as B operand).  The lane ADDRESSES, per read, the 8-byte run (tile row 16 s + 4 half
// [+ 8] + (r >> 2), d = 32 dt + (l32 & 16) + 4 (r & 3) .. + 3), r = l32 & 15.
// TransOffsets holds the byte offsets of those runs for s = 0 (a step of s adds 16 rows).
struct TransOffsets { int lo[4], hi[4]; };
__device__ inline TransOffsets trans_offsets(int l32, int half) {
  TransOffsets o;
  const int r = l32 & 15;
  const int row_lo = 4 * half + (r >> 2), row_hi = row_lo + 8;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    const int d = 32 * dt + (l32 & 16) + 4 * (r & 3);
    o.lo[dt] = row_lo * 256 + (((d >> 3) ^ swz16(row_lo)) << 4) + (d & 4) * 2;
    o.hi[dt] = row_hi * 256 + (((d >> 3) ^ swz16(row_hi)) << 4) + (d & 4) * 2;
  }
  return o;
}
__device__ inline bf16x8 trans_frag(const char* tile, const TransOffsets& o, int dt, int s) {
  const char* p = tile + s * (16 * 256);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(p + o.lo[dt]));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(p + o.hi[dt]));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
// B operand straight from global memory: row `row` (zero if not valid), d = 16*kd + 8*half ..
__device__ inline bf16x8 global_frag(const bf16* base, int ld, int row, bool valid, int kd, int half) {
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16)0.f;
  if (!valid) return z;
  return *reinterpret_cast<const bf16x8*>(base + (size_t)row * ld + kd * 16 + half * 8);
}
// Stores a wave's 32 x 128 result, held transposed in four accumulator tiles (register r of lane
// (l32, half) in tile dt is column 32 dt + 8 (r / 4) + 4 half + r % 4 of row l32), times the
// lane's `scale`, as bf16 rows: rows row0 .. row0 + 31 of `base` (row pitch ld elements), those
// below `n_rows` only.  The lanes' own 8-byte pieces would make every store instruction touch
// 32 rows; they go through `stage` (8 KiB of LDS that only this wave uses at this point, chunk
// c of row r at chunk c ^ (r & 15), its halves swapped in rows 16..31: no bank conflict either
// way) and leave as whole rows, four rows of 256 bytes per instruction.
__device__ inline void store_rows_bf16(char* stage, const f32x16 (&acc)[4], float scale, bf16* base, size_t ld,
                                       int row0, int n_rows, int lane) {
  const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (bf16)(acc[dt][4 * gq + e] * scale);
      const int c = (dt * 4 + gq) ^ (l32 & 15);
      // (rows r and r + 16 share a chunk position: they take opposite 8-byte halves of it)
      *reinterpret_cast<bf16x4*>(stage + l32 * 256 + c * 16 + ((half ^ (l32 >> 4)) << 3)) = v;
    }
  wave_lds_sync();
  const int c = lane & 15;
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int r = 4 * p + (lane >> 4);
    u32x4 v = *reinterpret_cast<const u32x4*>(stage + r * 256 + ((c ^ (r & 15)) << 4));
    if (r & 16) v = u32x4{v[2], v[3], v[0], v[1]};
    if (row0 + r < n_rows) *reinterpret_cast<u32x4*>(base + (size_t)(row0 + r) * ld + c * 8) = v;
  }
  wave_lds_sync();   // the region may be rewritten (the next tensor of this wave)
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
//   S^T = K Q^T (A = K rows from LDS, B = Q fragments in registers), online softmax along the
//   lanes, O^T += V^T P^T (A = V read transposed from LDS, B = P from the accumulator registers).
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv,
                                                                 bf16* __restrict__ out,
                                                                 float* __restrict__ lse, int seq, int Hq,
                                                                 int Hkv) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];   // two sets of (K, V)
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
  const TransOffsets to = trans_offsets(l32, half);

  bf16x8 qf[8];
  const int qrow = qw0 + l32;
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) qf[kd] = global_frag(qbase, ld, qrow, qrow < seq, kd, half);
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) settle(qf[kd]);

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int q_end = min(q0 + 128, seq);      // keys needed: 0 .. q_end-1
  const int n_tiles = (q_end + 63) / 64;
  TileLoader loader;
  loader.init(ld);
  auto issue = [&](int t) {
    const int kv0 = t * 64;
    char* set = lds + (t & 1) * (2 * kTileBytes);
    loader.issue(set, kbase + (size_t)kv0 * ld, seq - kv0);
    loader.issue(set + kTileBytes, vbase + (size_t)kv0 * ld, seq - kv0);
  };
  issue(0);
  for (int t = 0; t < n_tiles; ++t) {
    const int kv0 = t * 64;
    // tile t has landed for every wave, and every wave is done with tile t-1, whose set the
    // loads issued next overwrite while this tile is multiplied
    step_barrier();
    if (t + 1 < n_tiles) issue(t + 1);
    const char* k_tile = lds + (t & 1) * (2 * kTileBytes);
    const char* v_tile = k_tile + kTileBytes;
    if (kv0 > qw0 + 31) continue;             // every key of this tile is in this wave's future
    // Every MFMA multiplies a fragment requested from LDS kAhead MFMAs earlier (a ring of
    // kAhead + 1 fragments); scheduling barriers keep the requests in front.
    constexpr int kAhead = 4, kRing = kAhead + 1;
    bf16x8 ring[kRing];
    f32x16 s[2];
    {
      // S^T of the tile's two key halves, their k-steps interleaved: item n = (k-step n / 2, half n % 2)
      auto frag = [&](int n) { return row_frag(k_tile, n & 1, n >> 1, l32, half); };
#pragma unroll
      for (int n = 0; n < kAhead; ++n) ring[n] = frag(n);
#pragma unroll
      for (int n = 0; n < 16; ++n) {
        if (n + kAhead < 16) ring[(n + kAhead) % kRing] = frag(n + kAhead);
        __builtin_amdgcn_sched_barrier(0);
        s[n & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % kRing], qf[n >> 1], n < 2 ? kZero16 : s[n & 1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the first transposed V fragments: requested now, they arrive during the softmax
    auto tfrag = [&](int m) { return trans_frag(v_tile, to, m & 3, m >> 2); };
#pragma unroll
    for (int m = 0; m < kAhead; ++m) ring[m] = tfrag(m);
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
    bf16x8 pf[4];
#pragma unroll
    for (int sk = 0; sk < 4; ++sk) pf[sk] = acc_frag(s[sk >> 1], sk & 1);
#pragma unroll
    for (int m = 0; m < 16; ++m) {             // item m = (k-step m / 4, d block m % 4)
      if (m + kAhead < 16) ring[(m + kAhead) % kRing] = tfrag(m + kAhead);
      __builtin_amdgcn_sched_barrier(0);
      o[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[m % kRing], pf[m >> 2], o[m & 3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const float ltot = l + __shfl_xor(l, 32, 64);
  if (qrow < seq && half == 0) lse[((size_t)b * Hq + h) * seq + qrow] = (m + log2f(ltot)) * kLn2;
  __syncthreads();   // every wave is done with the tiles: LDS becomes the staging area of the stores
  store_rows_bf16(lds + wave * 8192, o, 1.f / ltot, out + tok0 * ((size_t)Hq * HD) + (size_t)h * HD, (size_t)Hq * HD,
                  qw0, seq, lane);
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

// ---- backward: one step of the dK/dV kernel ------------------------------------------------
// 64 queries against this wave's 32 keys, in two halves of 32 queries (one accumulator tile
// each) so that the VALU work of one half runs in the shadow of the other half's MFMAs:
//   A(0);  A(1) with softmax(0) between its MFMAs;  C(0) with softmax(1) between its MFMAs;  C(1)
// A(i): S_i = Q_i K^T, dP_i = dO_i V^T (16 MFMAs); softmax(i): P_i = exp2(S_i sl2 - lse),
// dS_i = P_i (dP_i - D); C(i): dV^T += dO_i^T P_i, dK^T += Q_i^T dS_i (16 MFMAs).
// A wave has its SIMD to itself (the dK / dV accumulators fill half of the register file), so
// nothing hides an LDS read that is waited for right before its MFMA: every fragment is
// requested four MFMA pairs ahead (a ring of five that runs through all four phases), and
// scheduling barriers pin the order "MFMA, one softmax element, MFMA, one softmax element".  On the tiles that cross the diagonal
// (`diag`, uniform over the wave) P and dS of a half are masked in a pass of their own before
// the half's C phase: query 32 i + 8 (r / 4) + (r % 4) + 4 half of the tile is hidden from this
// lane's key when that index, without the lane's 4 half, is below `first_q`.
__device__ __forceinline__ void dkv_step(const char* q_tile, const char* do_tile, const float* lse_j,
                                         const float* delta_j, const bf16x8 (&kf)[8], const bf16x8 (&vf)[8],
                                         f32x16 (&dk)[4], f32x16 (&dv)[4], const TransOffsets& to, int l32, int half,
                                         bool diag, int first_q, float sl2) {
  f32x16 s[2], dp[2];
  // row statistics of queries 32 i + 8 c + 4 half + 0..3, fetched from LDS one group of four
  // elements ahead of their use (all of them up front would cost 64 registers that the
  // accumulators need)
  f32x4 lse_v[2][4], delta_v[2][4];
  auto load_stat = [&](int i, int c) {
    lse_v[i][c] = *reinterpret_cast<const f32x4*>(lse_j + 32 * i + 8 * c + 4 * half);
    delta_v[i][c] = *reinterpret_cast<const f32x4*>(delta_j + 32 * i + 8 * c + 4 * half);
  };
  // element r of half i: s <- P, dp <- dS
  auto soft = [&](int i, int r) {
    float p = fast_exp2(__builtin_fmaf(s[i][r], sl2, -lse_v[i][r >> 2][r & 3]));
    s[i][r] = p;
    dp[i][r] = p * (dp[i][r] - delta_v[i][r >> 2][r & 3]);
  };
  // Fragment rings.  The 32 MFMA pairs of a step -- A(0), A(1), C(0), C(1), eight pairs each --
  // form ONE sequence: pair n multiplies the fragments requested kAhead pairs earlier, across
  // the phase boundaries (none of them depends on anything a phase computes), so only the
  // step's first pairs wait for LDS.
  constexpr int kAhead = 4, kRing = kAhead + 1;
  bf16x8 fq[kRing], fd[kRing];
  auto fetch = [&](int n) {
    const int ph = n >> 3, k = n & 7;
    if (ph < 2) {          // A(ph): rows of Q / dO, k-step k
      fq[n % kRing] = row_frag(q_tile, ph, k, l32, half);
      fd[n % kRing] = row_frag(do_tile, ph, k, l32, half);
    } else {               // C(ph - 2): transposed, d block k & 3, k-step 2 (ph - 2) + (k >> 2)
      fd[n % kRing] = trans_frag(do_tile, to, k & 3, 2 * (ph - 2) + (k >> 2));
      fq[n % kRing] = trans_frag(q_tile, to, k & 3, 2 * (ph - 2) + (k >> 2));
    }
  };
  auto mask = [&](int i) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (32 * i + 8 * (r >> 2) + (r & 3) < first_q) { s[i][r] = 0.f; dp[i][r] = 0.f; }
  };
  // A(i); `between(n)` runs after MFMA n of the phase, n = 0..15
  auto phase_a = [&](int i, auto&& between) {
#pragma unroll
    for (int kd = 0; kd < 8; ++kd) {
      const int n = 8 * i + kd;
      if (n + kAhead < 32) fetch(n + kAhead);
      __builtin_amdgcn_sched_barrier(0);
      s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % kRing], kf[kd], kd == 0 ? kZero16 : s[i], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      between(2 * kd);
      __builtin_amdgcn_sched_barrier(0);
      dp[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[n % kRing], vf[kd], kd == 0 ? kZero16 : dp[i], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      between(2 * kd + 1);
    }
  };
  // C(i): k-steps 2 i and 2 i + 1 (the 16 queries each of P_i / dS_i), four d blocks each
  auto phase_c = [&](int i, auto&& between) {
    bf16x8 pf, dsf;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int n = 16 + 8 * i + m;
      const int dt = m & 3, s2 = m >> 2;
      if (n + kAhead < 32) fetch(n + kAhead);
      if (dt == 0) { pf = acc_frag(s[i], s2); dsf = acc_frag(dp[i], s2); }
      __builtin_amdgcn_sched_barrier(0);
      dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[n % kRing], pf, dv[dt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      between(2 * m);
      __builtin_amdgcn_sched_barrier(0);
      dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % kRing], dsf, dk[dt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      between(2 * m + 1);
    }
  };
#pragma unroll
  for (int n = 0; n < kAhead; ++n) fetch(n);
  phase_a(0, [&](int) {});
  load_stat(0, 0);
  phase_a(1, [&](int n) {
    if (n % 4 == 0 && n < 12) load_stat(0, n / 4 + 1);
    soft(0, n);
  });
  load_stat(1, 0);
  if (diag) mask(0);
  phase_c(0, [&](int n) {
    if (n % 4 == 0 && n < 12) load_stat(1, n / 4 + 1);
    soft(1, n);
  });
  if (diag) mask(1);
  phase_c(1, [&](int) {});
}

// ---- backward: dK, dV ----------------------------------------------------------------------
// One workgroup: 128 keys of one (b, kv head); wave w owns keys [32w, 32w+32).  For every query
// head of the group (ascending) and every 64-query tile at or below the diagonal:
//   S = Q K^T, dP = dO V^T  (A = Q / dO rows from LDS, B = K / V fragments in registers)
//   P = exp(S/sqrt(hd) - lse), dS = P (dP - D)
//   dV^T += dO^T P,  dK^T += Q^T dS  (A = the same Q / dO tiles read transposed, B = P / dS
//   from the accumulator registers)
// The (head, tile) steps form one sequence whose tiles alternate between two LDS sets.
// With `partial` (grouped-query attention with a scratch buffer) a workgroup handles ONE query
// head (grid x = query heads x batch) and stores its unscaled fp32 dK and dV rows to
// partial[(b * Hq + h) * seq + key][0..127] and, mb * Hq * seq rows further, the dV rows; the
// group's heads are then summed in ascending order by attn_bwd_dkv_reduce_kernel.  Without
// it a workgroup walks the whole group of its kv head itself (grid x = kv heads x batch).
__global__ __launch_bounds__(kThreads) void attn_bwd_dkv_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16* __restrict__ dqkv, int seq, int Hq, int Hkv,
    float* __restrict__ partial, long long partial_dv_offset) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];   // two sets of (Q, dO)
  __shared__ float lse_s[2][64], delta_s[2][64];
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
  const TransOffsets to = trans_offsets(l32, half);

  bf16x8 kf[8], vf[8];
  const int krow = kw0 + l32;
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) {
    kf[kd] = global_frag(kbase, ld, krow, krow < seq, kd, half);
    vf[kd] = global_frag(vbase, ld, krow, krow < seq, kd, half);
  }
  // (these loads are settled below, after the first tiles' loads have been issued: the two
  // latencies of a workgroup's start then overlap)
  // The accumulators start as the result of an MFMA (0 * 0 + 0) rather than of a zero fill, and
  // are pinned once: they then live in the accumulation registers from here to the epilogue.  A
  // tile that ordinary arithmetic defines is kept in architectural registers instead and copied,
  // sixteen registers in and sixteen out, around every MFMA that adds to it.
  f32x16 dk[4], dv[4];
  {
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (bf16)0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(z, z, kZero16, 0, 0, 0);
      dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(z, z, kZero16, 0, 0, 0);
      pin_agpr(dk[dt]);
      pin_agpr(dv[dt]);
    }
  }

  const int first_tile = k0 / 64;
  const int n_tiles = (seq + 63) / 64;
  const int per_head = n_tiles - first_tile;             // >= 1: k0 < seq
  const int n_steps = (hh_end - hh_first) * per_head;
  // step j -> (query head, query tile); starts the loads of its tiles into set j & 1 and
  // fetches (first wave) the tile's row statistics into registers
  float lse_r = INFINITY, delta_r = 0.f;
  TileLoader q_loader, do_loader;
  q_loader.init(ld);
  do_loader.init(ldo);
  auto issue = [&](int j) {
    const int h = g * group + hh_first + j / per_head;
    const int qt0 = (first_tile + j % per_head) * 64;
    const bf16* qbase = qkv + tok0 * ld + (size_t)h * HD;
    const bf16* dobase = dout + tok0 * ldo + (size_t)h * HD;
    if (threadIdx.x < 64) {
      const int q = qt0 + (int)threadIdx.x;
      const size_t row = ((size_t)b * Hq + h) * seq;
      lse_r = q < seq ? lse[row + q] : INFINITY;            // +inf makes P = 0 beyond the end
      delta_r = q < seq ? delta[row + q] : 0.f;
    }
    char* set = lds + (j & 1) * (2 * kTileBytes);
    q_loader.issue(set, qbase + (size_t)qt0 * ld, seq - qt0);
    do_loader.issue(set + kTileBytes, dobase + (size_t)qt0 * ldo, seq - qt0);
  };
  auto publish = [&](int j) {
    // (the scaling waits for the load: here, a step after it was issued, not in issue())
    if (threadIdx.x < 64) { lse_s[j & 1][threadIdx.x] = lse_r * kLog2e; delta_s[j & 1][threadIdx.x] = delta_r; }
  };
  issue(0);
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) { settle(kf[kd]); settle(vf[kd]); }
  publish(0);
  for (int j = 0; j < n_steps; ++j) {
    const int qt0 = (first_tile + j % per_head) * 64;
    // the tiles and statistics of step j are in place for every wave, and every wave is done
    // with step j-1, whose set and statistics the next step's loads and publish overwrite
    step_barrier();
    if (j + 1 < n_steps) issue(j + 1);
    const char* q_tile = lds + (j & 1) * (2 * kTileBytes);
    const char* do_tile = q_tile + kTileBytes;
    const float* lse_j = lse_s[j & 1];
    const float* delta_j = delta_s[j & 1];
    if (qt0 + 63 >= kw0) {                     // else every query of this tile precedes this wave's keys
      // query qt0 + ql is masked for key krow when qt0 + ql < krow; only tiles that cross the diagonal have such pairs
      dkv_step(q_tile, do_tile, lse_j, delta_j, kf, vf, dk, dv, to, l32, half, qt0 < kw0 + 31, krow - qt0 - 4 * half, sl2);
    }
    if (j + 1 < n_steps) publish(j + 1);
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
  __syncthreads();   // every wave is done with the tiles: LDS becomes the staging area of the stores
  bf16* dkbase = dqkv + tok0 * ld + (size_t)(Hq + g) * HD;
  store_rows_bf16(lds + wave * 8192, dk, scale, dkbase, (size_t)ld, kw0, seq, lane);
  store_rows_bf16(lds + wave * 8192, dv, 1.f, dkbase + (size_t)Hkv * HD, (size_t)ld, kw0, seq, lane);
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
//   S^T = K Q^T, dP^T = V dO^T (A = K / V rows from LDS, B = Q / dO fragments in registers)
//   dS^T = P^T (dP^T - D);  dQ^T += K^T dS^T (A = the K tile read transposed)
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16* __restrict__ dqkv, int seq, int Hq, int Hkv) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];   // two sets of (K, V)
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
  const TransOffsets to = trans_offsets(l32, half);

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
#pragma unroll
  for (int kd = 0; kd < 8; ++kd) { settle(qf[kd]); settle(dof[kd]); }
  settle(lse2);
  settle(dlt);
  f32x16 dq[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;

  const int q_end = min(q0 + 128, seq);
  const int n_tiles = (q_end + 63) / 64;
  TileLoader loader;
  loader.init(ld);
  auto issue = [&](int t) {
    const int kv0 = t * 64;
    char* set = lds + (t & 1) * (2 * kTileBytes);
    loader.issue(set, kbase + (size_t)kv0 * ld, seq - kv0);
    loader.issue(set + kTileBytes, vbase + (size_t)kv0 * ld, seq - kv0);
  };
  issue(0);
  for (int t = 0; t < n_tiles; ++t) {
    const int kv0 = t * 64;
    step_barrier();                             // tile t in place, tile t-1's set free for tile t+1
    if (t + 1 < n_tiles) issue(t + 1);
    const char* k_tile = lds + (t & 1) * (2 * kTileBytes);
    const char* v_tile = k_tile + kTileBytes;
    if (kv0 > qw0 + 31) continue;
    const bool diag = kv0 + 63 > qw0;          // only tiles that cross the diagonal need the mask
    // The tile's 64 keys in two halves of 32 (one accumulator tile of S^T and of dP^T each).
    // Every MFMA multiplies a fragment requested from LDS kAhead MFMAs earlier (a ring of
    // kAhead + 1 fragments); scheduling barriers keep the requests in front.  What a wave
    // still waits for, the other workgroup's wave on its SIMD fills.
    constexpr int kAhead = 4, kRing = kAhead + 1;
    bf16x8 ring[kRing];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      f32x16 s, dp;
      // S^T_i and dP^T_i, their k-steps interleaved: item n = (k-step n / 2, S or dP)
      auto frag = [&](int n) { return row_frag((n & 1) ? v_tile : k_tile, i, n >> 1, l32, half); };
#pragma unroll
      for (int n = 0; n < kAhead; ++n) ring[n] = frag(n);
#pragma unroll
      for (int n = 0; n < 16; ++n) {
        if (n + kAhead < 16) ring[(n + kAhead) % kRing] = frag(n + kAhead);
        __builtin_amdgcn_sched_barrier(0);
        if (n & 1) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % kRing], dof[n >> 1], n == 1 ? kZero16 : dp, 0, 0, 0);
        else s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % kRing], qf[n >> 1], n == 0 ? kZero16 : s, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      // the transposed K fragments of this half's two k-steps: requested now, they arrive while
      // the exponentials are computed
      auto tfrag = [&](int m) { return trans_frag(k_tile, to, m & 3, 2 * i + (m >> 2)); };
#pragma unroll
      for (int m = 0; m < kAhead; ++m) ring[m] = tfrag(m);
      // s[r]: key kv0 + 32 i + 8 (r/4) + 4 half + r%4, query qw0 + l32
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = fast_exp2(__builtin_fmaf(s[r], sl2, -lse2));
      if (diag) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
          if (key > qrow) s[r] = 0.f;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] *= dp[r] - dlt;        // dS^T = P^T (dP^T - D)
      const bf16x8 b0 = acc_frag(s, 0), b1 = acc_frag(s, 1);
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        if (m + kAhead < 8) ring[(m + kAhead) % kRing] = tfrag(m + kAhead);
        __builtin_amdgcn_sched_barrier(0);
        dq[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[m % kRing], m < 4 ? b0 : b1, dq[m & 3], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  __syncthreads();   // every wave is done with the tiles: LDS becomes the staging area of the stores
  store_rows_bf16(lds + wave * 8192, dq, scale, dqkv + tok0 * ld + (size_t)h * HD, (size_t)ld, qw0, seq, lane);
}

}  // namespace

bool attention_mfma_supported(const AttnDesc& a) { return a.hd == HD; }

size_t attention_bwd_scratch_bytes(int mb, int seq, int Hq, int Hkv, int hd) {
  if (hd != HD || Hq <= Hkv) return 0;
  return (size_t)2 * mb * Hq * seq * HD * sizeof(float);
}

hipError_t launch_attention_fwd_mfma(const AttnDesc& a, hipStream_t s) {
  dim3 grid(a.Hq * a.mb, (a.seq + 127) / 128);
  attn_fwd_mfma_kernel<<<grid, kThreads, 0, s>>>((const bf16*)a.qkv, (bf16*)a.out, a.lse, a.seq, a.Hq, a.Hkv);
  return hipGetLastError();
}

hipError_t launch_attention_bwd_mfma(const AttnDesc& a, hipStream_t s) {
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
                                                   (bf16*)a.dqkv, a.seq, a.Hq, a.Hkv,
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
                                                  (bf16*)a.dqkv, a.seq, a.Hq, a.Hkv);
  return hipGetLastError();
}

}  // namespace jpp
