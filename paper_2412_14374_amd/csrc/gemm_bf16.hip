// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
//   C[M,N] (op)= sum_k A(m,k) * B(n,k)  (+ bias[n]) (+ residual[m,n])
//
// Either operand may be stored "k-contiguous" (element (r,k) at P[r*ld + k]) or
// "k-strided" (at P[k*ld + r]).  The three GEMMs of a linear layer y = x W^T map to
//   forward  y  = x  W^T : A = x  (k-contig), B = W  (k-contig)
//   dgrad    dx = dy W   : A = dy (k-contig), B = W  (k-strided)
//   wgrad    G += dy^T x : A = dy (k-strided), B = x (k-strided), fp32 read-modify-write of G
// so no transposed copy of a weight or an activation ever exists in HBM.  The last form is
// the `grads += mugrads` of the paper's Section 3.1 fused into the producing GEMM: the
// unrounded fp32 accumulator is added to the fp32 gradient.
//
// Design (one workgroup = one BM x BN tile of C):
//  * The default is a 256 x 256 x 64 tile, eight waves (wave tile 128 x 64), two LDS stages
//    of 64 KB.  (Four waves with 128 x 128 wave tiles, forced variant 8, read a third less
//    from LDS per MFMA and run at a 10 % higher clock under the board's power limit, but a
//    lone wave per SIMD has nobody to hide its waits behind: 73 % matrix-pipe occupancy
//    against 84 %, 1.24-1.28 against 1.31-1.33 PFLOP/s.)  A 64-wide stage makes every row of a k-contiguous tile one full 128-byte
//    cache line (32-wide stages fetch every line twice and lose more than a deeper ring
//    gains), and 256 x 256 is the largest tile whose accumulators fit the register file --
//    the L2 -> CU path is the busiest resource beside the matrix pipe, so bytes per flop matter most.
//  * Two loaders fill the stages.  The default ("register-staged", VG = true): every thread
//    fetches its 16-byte chunks of k-tile kt+2 into registers while tile kt is multiplied and
//    writes them to the free stage one iteration later, one chunk between two MFMA groups, so
//    a load has a whole iteration to arrive.  The other (VG = false, kept as forced
//    variants) fills a ring of NS stages HBM -> LDS directly (buffer_load ... lds: no VGPRs,
//    no ds_write); every wave instruction of such a load fills 1 KiB of LDS in lane order,
//    so the swizzle is applied to WHICH global chunk each lane fetches.  Its loads are inline
//    assembly and the cross-wave hand-over is an explicit "s_waitcnt vmcnt(loads still
//    allowed in flight); s_barrier": the compiler's wait-count pass cannot tell the stages
//    apart and would wait for every load in flight.  The lane's byte offset of every load is
//    computed once per kernel; a k-tile costs the scalar arithmetic of its descriptor.  It is
//    slower on every shape measured (1.03-1.19 against 1.31 PFLOP/s at the feed-forward
//    shapes), also when every tile is requested at the very start of its iteration: with
//    all operands resident in L2 the eight-wave form reaches 1.39, so what it lacks is the
//    second iteration of flight time that the registers give a load.
//  * LDS layouts, the same for both loaders, bank-conflict free by an XOR swizzle of the
//    16-byte chunk index:
//      k-contiguous tile: LDS [rows][BKT] bf16; fragment = one 16-byte read per lane.
//      k-strided tile:    LDS [BKT][rows] bf16, as in memory; fragment = two
//                         ds_read_b64_tr_b16 per lane (the CDNA4 transposing LDS read: lane i
//                         of a 16-lane group receives element (i & 3) of the 8-byte rows
//                         4j + (i >> 2), j = 0..3, that the group's lanes address).
//    Both give lane (row = lane % 32, half = lane / 32) the 8 k-values 16*kk + 8*half + 0..7,
//    so the MFMA loop is the same for all four layout combinations.
//  * Loads, LDS writes and fragment reads are issued between the single MFMAs of a group (one
//    32-row block): MFMA, the group's LDS write, MFMA, the global load that refills the
//    register just written and the group's fragment reads -- a wave's memory instructions
//    then issue while the matrix pipe works on that wave's own MFMA, which measures 4 % faster
//    than memory work in front of each group.
//    Fragments are double-buffered in registers and the last k-step of a stage is split around
//    the barrier; the next stage's first fragments are spread over the groups behind it.
//  * Rows beyond the matrix read as zero through the buffer range check, the contiguous
//    dimension is predicated, so M, N, K need only be multiples of 8.
//  * Epilogue: accumulators go through LDS so that every global access is 8 or 16 bytes per
//    lane on full rows.  A tile inside the matrix takes a pass without predicates or run-time
//    mode branches, so that all of its loads and stores are in flight together (behind a branch
//    the compiler waits for every outstanding access, stores included, before a loaded register
//    is used: 32 serial store round trips per accumulating tile, 0.2 ms of a 2 ms launch at
//    K = 2048); the fp32 gradient rows are requested one 32-row block ahead.
//  * Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs)
//    works on a contiguous band of tiles and shares operand panels in its own L2.
#include <cstdlib>
#include <type_traits>

#include "device_utils.h"
#include "internal.h"

namespace jpp {

namespace {

constexpr uint32_t kOOB = 0x7FFFFFFFu;
constexpr uint32_t kMaxRecords = 0x7FFFFF00u;
constexpr int kMaxStages = 5;

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_t;

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptor (base, stride 0, num_records = bytes, untyped 32-bit format).
__device__ inline i32x4 make_rsrc(const void* p, long long bytes) {
  const uint32_t n = bytes > (long long)kMaxRecords ? kMaxRecords : (bytes < 0 ? 0u : (uint32_t)bytes);
  const unsigned long long a = (unsigned long long)p;
  i32x4 r;
  r[0] = (int)(uint32_t)a;
  r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);
  r[2] = (int)n;
  r[3] = 0x00020000;
  return r;
}

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc_v(const void* p, long long bytes) {
  const uint32_t n = bytes > (long long)kMaxRecords ? kMaxRecords : (bytes < 0 ? 0u : (uint32_t)bytes);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)n, 0x00020000);
}

// The same from a byte count that is known to fit (what a tile can touch, see records() of the
// tile classes): no 64-bit compares, which this target only has as vector instructions.
__device__ inline i32x4 make_rsrc32(const void* p, uint32_t bytes) {
  const unsigned long long a = (unsigned long long)p;
  i32x4 r;
  r[0] = (int)(uint32_t)a;
  r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc32_v(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// 16 bytes per lane, HBM -> LDS without passing through registers: the wave's 64 lanes fill
// the 1 KiB at LDS byte address `lds_addr` in lane order; lanes whose byte offset `voff` is
// outside the descriptor's range store zeros.  Issued as inline assembly on purpose: the
// compiler's wait-count pass would otherwise make every later LDS read wait for ALL loads in
// flight, which defeats a multi-stage ring; the waits are placed by hand below.
__device__ inline void dma16(const i32x4& rsrc, uint32_t lds_addr, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rsrc)
               : "memory", "m0");
}
__device__ inline uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const char*)p;
}

constexpr int kCus = 256;   // compute units of the MI355X

struct Epilogue {
  void* C; int ldc; int out_mode;
  const bf16* bias; const bf16* residual;
  // Split tail (see launch_cfg): workgroups with id >= split_first each compute one of
  // split_s k-ranges of a tile and store the fp32 partial tile to split_ws; 0 = no splitting.
  int split_first; int split_s; float* split_ws;
  // 1: tile_of_square (outputs whose tile counts are multiples of 16 in both directions)
  int square_map;
  // fused GeLU (GemmDesc::act) and its second tensor
  int act; bf16* aux;
};

// Stores four consecutive outputs of a bf16 store-mode GEMM, applying the fused activation ACT:
// forward, h goes to C and gelu(h), evaluated on the rounded h, to aux; backward, the rounded
// value is da and C receives da * gelu'(h) with h read from aux.
template <int ACT>
__device__ inline void store_bf16x4_act(const Epilogue& ep, size_t idx, const f32x4& v, bf16x4 h = bf16x4{}) {
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
  bf16* c = reinterpret_cast<bf16*>(ep.C) + idx;
  if constexpr (ACT == ACT_NONE) {
    *reinterpret_cast<bf16x4*>(c) = o;
  } else if constexpr (ACT == ACT_FWD_ERF || ACT == ACT_FWD_TANH) {
    bf16x4 a;
#pragma unroll
    for (int e = 0; e < 4; ++e) a[e] = (bf16)(ACT == ACT_FWD_ERF ? gelu_erf_fit((float)o[e]) : gelu_tanh((float)o[e]));
    *reinterpret_cast<bf16x4*>(c) = o;
    *reinterpret_cast<bf16x4*>(ep.aux + idx) = a;
  } else {
    bf16x4 d;   // h: the four values of aux at idx, loaded by the caller
#pragma unroll
    for (int e = 0; e < 4; ++e)
      d[e] = (bf16)((float)o[e] * (ACT == ACT_BWD_ERF ? gelu_erf_grad_fit((float)h[e]) : gelu_tanh_grad((float)h[e])));
    *reinterpret_cast<bf16x4*>(c) = d;
  }
}
// The same with the activation chosen at run time (the fix-up kernel of split tiles).
__device__ inline void store_bf16x4_act_rt(const Epilogue& ep, size_t idx, const f32x4& v) {
  switch (ep.act) {
    case ACT_FWD_ERF: store_bf16x4_act<ACT_FWD_ERF>(ep, idx, v); break;
    case ACT_FWD_TANH: store_bf16x4_act<ACT_FWD_TANH>(ep, idx, v); break;
    case ACT_BWD_ERF:
      store_bf16x4_act<ACT_BWD_ERF>(ep, idx, v, *reinterpret_cast<const bf16x4*>(ep.aux + idx));
      break;
    case ACT_BWD_TANH:
      store_bf16x4_act<ACT_BWD_TANH>(ep, idx, v, *reinterpret_cast<const bf16x4*>(ep.aux + idx));
      break;
    default: store_bf16x4_act<ACT_NONE>(ep, idx, v); break;
  }
}

struct Operand {
  const bf16* p; int ld; int rows;  // rows = M (for A) or N (for B)
};

// ---- operand tiles -------------------------------------------------------------------------
// R rows (m or n) x BKT k.  `issue` starts the HBM -> LDS copy of the tile whose first row is
// r0 and first k is k0 (every thread issues kLoads loads, also for tiles past the end of K,
// which then read as zero: the wait counts below rely on a fixed number per tile).
// `frag` returns the MFMA operand of the 32-row block `blk` for k-step kk.

template <int R, int BKT, int NT>
struct KContigTile {
  static constexpr int kRowBytes = BKT * 2;
  static constexpr int CPR = BKT / 8;            // 16-byte chunks per row
  // The LDS of gfx950 has 64 banks of 4 bytes: 16 lanes x 16 bytes are served per clock when
  // they fall into 16 different bank quads.  Rows that share a 256-byte line get the same
  // swizzle, consecutive lines rotate it, so 16 consecutive rows reading the same logical chunk
  // touch every quad once.
  static constexpr int RPL = 256 / kRowBytes;    // rows per 256-byte LDS line (2 or 4)
  static constexpr int kRowsPerInstr = 64 / CPR;
  static constexpr int kLoads = R * CPR / NT;
  static constexpr int kBytes = R * kRowBytes;
  static_assert((R * CPR) % NT == 0, "tile chunks must divide evenly over the threads");
  __device__ static inline int swz(int row) { return (row / RPL) % CPR; }

  // load i (0 .. kLoads-1) of the tile at (r0, k0) into the tile at LDS address `tile`
  __device__ static inline void issue_one(const Operand& op, int r0, int k0, int K, uint32_t tile, int i) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    const bf16* base = op.p + (size_t)r0 * op.ld + k0;
    const i32x4 rs = make_rsrc(base, ((long long)(op.rows - r0) * op.ld - k0) * 2);
    const int blk = i * (NT / 64) + wave;       // 1 KiB block of the tile
    const int row = blk * kRowsPerInstr + lane / CPR;
    const int kc = (lane % CPR) ^ swz(row);
    const uint32_t off = (k0 + kc * 8 < K) ? (uint32_t)(row * op.ld + kc * 8) * 2u : kOOB;
    dma16(rs, tile + blk * 1024, off);
  }
  // The same load split into what depends on the tile (the descriptor: base and range) and what
  // does not (the lane's byte offset, computed once per kernel): lane_offset() leaves out the
  // k-range predicate, so issue_fast() serves every k-tile that lies wholly inside K.
  __device__ static inline uint32_t lane_offset(const Operand& op, int r0, int i) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    const int blk = i * (NT / 64) + wave;
    const int row = blk * kRowsPerInstr + lane / CPR;
    const int kc = (lane % CPR) ^ swz(row);
    return (uint32_t)(row * op.ld + kc * 8) * 2u;
  }
  __device__ static inline bool fast_ok(int k0, int K) { return k0 + BKT <= K; }
  // Bytes from (r0, k0) that the descriptor of a tile must cover: up to the end of the tile's
  // last row inside the matrix, and never into the row after it, whose lanes must read zero
  // (lanes at k >= K are sent out of range one by one).  The same for every k-tile of a row
  // block, and at most R * ld * 2 < 2^31 (gemm_bf16_shape_ok).
  __device__ static inline uint32_t records(const Operand& op, int r0) {
    const int valid = op.rows - r0 < R ? op.rows - r0 : R;
    if (valid <= 0) return 0u;
    const int last = (valid - 1) * op.ld + BKT, all = valid * op.ld;
    return (uint32_t)(last < all ? last : all) * 2u;
  }
  __device__ static inline i32x4 tile_rsrc(const Operand& op, int r0, int k0, int K) {
    return make_rsrc32(op.p + (size_t)r0 * op.ld + k0, records(op, r0));
  }
  __device__ static inline void issue_fast(const i32x4& rs, uint32_t tile, int i, uint32_t voff) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    dma16(rs, tile + (i * (NT / 64) + wave) * 1024, voff);
  }
  // Register-staged variant: chunk i*NT + tid of the tile; 8 consecutive lanes read one
  // 128-byte row segment, the swizzle is applied when the chunk is written to LDS.
  __device__ static inline u32x4 load_one(const Operand& op, int r0, int k0, int K, int i) {
    const int cidx = i * NT + threadIdx.x;
    const int row = cidx / CPR, c = cidx % CPR;
    const bf16* base = op.p + (size_t)r0 * op.ld + k0;
    const auto rs = make_rsrc32_v(base, records(op, r0));
    const uint32_t off = (k0 + c * 8 < K) ? (uint32_t)(row * op.ld + c * 8) * 2u : kOOB;
    return __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
  }
  __device__ static inline void store_one(char* tile, int i, const u32x4& v) {
    const int cidx = i * NT + threadIdx.x;
    const int row = cidx / CPR, c = cidx % CPR;
    *reinterpret_cast<u32x4*>(tile + row * kRowBytes + ((c ^ swz(row)) << 4)) = v;
  }
  // byte offset of the kk = 0 fragment of the 32-row block starting at `row0`
  __device__ static inline int frag_base(int row0, int l32, int half) {
    const int row = row0 + l32;
    return row * kRowBytes + ((half ^ swz(row)) << 4);
  }
  __device__ static inline bf16x8 frag(const char* tile, int base, int kk) {
    // chunk = 2*kk + half; the swizzle only touches the low bits that 2*kk leaves alone or
    // flips consistently: (2kk + half) ^ s == ((half ^ s) ^ 2kk)
    return *reinterpret_cast<const bf16x8*>(tile + (base ^ ((kk * 2) << 4)));
  }
};

template <int R, int BKT, int NT>
struct KStridedTile {
  static constexpr int kRowBytes = R * 2;        // one k-row of the tile
  static constexpr int CPR = R / 8;
  static constexpr int kRowsPerInstr = 64 / CPR;
  static constexpr int kLoads = BKT * CPR / NT;
  static constexpr int kBytes = BKT * kRowBytes;
  static_assert((BKT * CPR) % NT == 0 && CPR <= 64, "tile chunks must divide evenly over the threads");

  __device__ static inline void issue_one(const Operand& op, int r0, int k0, int K, uint32_t tile, int i) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    const bf16* base = op.p + (size_t)k0 * op.ld + r0;
    const i32x4 rs = make_rsrc(base, ((long long)(K - k0) * op.ld - r0) * 2);
    const int blk = i * (NT / 64) + wave;
    const int k = blk * kRowsPerInstr + lane / CPR;
    const int c = (lane % CPR) ^ ((k & 3) << 2);
    const uint32_t off = (r0 + c * 8 < op.rows) ? (uint32_t)(k * op.ld + c * 8) * 2u : kOOB;
    dma16(rs, tile + blk * 1024, off);
  }
  // tile-independent lane offset (the row-range predicate does not depend on k) and the
  // descriptor of one k-tile, whose range makes k-rows at and beyond K read as zero
  __device__ static inline uint32_t lane_offset(const Operand& op, int r0, int i) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    const int blk = i * (NT / 64) + wave;
    const int k = blk * kRowsPerInstr + lane / CPR;
    const int c = (lane % CPR) ^ ((k & 3) << 2);
    return (r0 + c * 8 < op.rows) ? (uint32_t)(k * op.ld + c * 8) * 2u : kOOB;
  }
  __device__ static inline bool fast_ok(int, int) { return true; }
  // Bytes from (k0, r0) that the descriptor of a tile must cover: up to the end of its last
  // k-row below K (none: a tile requested beyond the contraction reads zeros), never into the
  // k-row after it; columns beyond the matrix are sent out of range lane by lane.
  __device__ static inline uint32_t records(const Operand& op, int k0, int K) {
    const int valid = K - k0 < BKT ? K - k0 : BKT;
    if (valid <= 0) return 0u;
    const int last = (valid - 1) * op.ld + R, all = valid * op.ld;
    return (uint32_t)(last < all ? last : all) * 2u;
  }
  __device__ static inline i32x4 tile_rsrc(const Operand& op, int r0, int k0, int K) {
    return make_rsrc32(op.p + (size_t)k0 * op.ld + r0, records(op, k0, K));
  }
  __device__ static inline void issue_fast(const i32x4& rs, uint32_t tile, int i, uint32_t voff) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    dma16(rs, tile + (i * (NT / 64) + wave) * 1024, voff);
  }
  __device__ static inline u32x4 load_one(const Operand& op, int r0, int k0, int K, int i) {
    const int cidx = i * NT + threadIdx.x;
    const int k = cidx / CPR, c = cidx % CPR;
    const bf16* base = op.p + (size_t)k0 * op.ld + r0;
    const auto rs = make_rsrc32_v(base, records(op, k0, K));
    const uint32_t off = (r0 + c * 8 < op.rows) ? (uint32_t)(k * op.ld + c * 8) * 2u : kOOB;
    return __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
  }
  __device__ static inline void store_one(char* tile, int i, const u32x4& v) {
    const int cidx = i * NT + threadIdx.x;
    const int k = cidx / CPR, c = cidx % CPR;
    *reinterpret_cast<u32x4*>(tile + k * kRowBytes + ((c ^ ((k & 3) << 2)) << 4)) = v;
  }
  // Lane l of a 16-lane group addresses the 8-byte row (k = .. + (l>>2), rows 4*(l&3) .. +3)
  // and receives k = .. + 0..3 for row (l & 15) of the group's 16 rows.  The 32 lanes served
  // together read 4 k-rows x 32 rows; k-row k has its 16-byte chunks XORed with 4 * (k & 3), which
  // sends the four k-rows to four different 64-byte bank groups: 256 distinct bytes, no conflict.
  __device__ static inline int frag_base(int row0, int l32, int half) {
    const int r = l32 & 15;
    const int row = row0 + (l32 & 16) + 4 * (r & 3);
    const int k = half * 8 + (r >> 2);
    return k * kRowBytes + (((row >> 3) ^ ((k & 3) << 2)) << 4) + (row & 4) * 2;
  }
  __device__ static inline bf16x8 frag(const char* tile, int base, int kk) {
    const char* p = tile + base + kk * 16 * kRowBytes;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(p + 4 * kRowBytes));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
};

template <int R, int BKT, int NT, bool KS>
struct TileSel { typedef KContigTile<R, BKT, NT> type; };
template <int R, int BKT, int NT>
struct TileSel<R, BKT, NT, true> { typedef KStridedTile<R, BKT, NT> type; };

// Maps the linear workgroup id to a tile.  Ids are dealt round-robin to the 8 XCDs, so the
// ids {x, x+8, x+16, ...} share one L2: give each XCD a contiguous range of tile numbers, and
// number tiles in bands of kBand tile-rows, column-major inside a band.
__device__ inline void tile_of(int pid, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;
  constexpr int kXcd = 8;
  int t = pid;
  if (total >= kXcd * 4) {
    const int per = (total + kXcd - 1) / kXcd;
    const int x = pid % kXcd, r = pid / kXcd;
    const int full = total % kXcd == 0 ? kXcd : total % kXcd;  // XCDs holding `per` tiles
    const int start = x < full ? x * per : full * per + (x - full) * (per - 1);
    t = start + r;
  }
  constexpr int kBand = 8;
  const int band_tiles = kBand * tiles_n;
  const int band = t / band_tiles;
  const int first_m = band * kBand;
  const int rows_in_band = (tiles_m - first_m) < kBand ? (tiles_m - first_m) : kBand;
  const int in_band = t - band * band_tiles;
  tm = first_m + in_band % rows_in_band;
  tn = in_band / rows_in_band;
}

// The same for large outputs whose tile counts are multiples of 16 both ways: in every round
// of 256 workgroups the 8 XCDs work on a 2 x 4 arrangement of 8 x 4 blocks, i.e. together on a
// 16 x 16 square of tiles, so the chip touches 32 operand panels per round instead of 68 and
// what one XCD fetched is in the last-level cache for its neighbours; squares are visited
// along a band of 16 tile-rows, so consecutive rounds keep the band's 16 row panels.
__device__ inline void tile_of_square(int pid, int tiles_n, int& tm, int& tn) {
  const int x = pid & 7, r = pid >> 3;
  const int round = r >> 5, w = r & 31;
  const int squares_n = tiles_n >> 4;
  const int sq_m = round / squares_n, sq_n = round % squares_n;
  tm = sq_m * 16 + (x >> 2) * 8 + (w & 7);
  tn = sq_n * 16 + (x & 3) * 4 + (w >> 3);
}

// "s_waitcnt vmcnt(N); s_barrier" with a compiler-level memory barrier and no fence: the
// fence of __syncthreads() would wait for every outstanding load, which is exactly what the
// multi-stage ring must not do.
template <int N>
__device__ inline void wait_loads_and_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// MINW: waves per SIMD the register allocation must leave room for (1 = use the whole file).
// ACT: the fused GeLU of the store-mode epilogue (ACT_NONE in all but the few instantiations
// that the feed-forward block uses, so that the common kernels carry none of its code).
template <int BM, int BN, int BKT, int NS, int WM, int WN, bool AKS, bool BKS, bool VG = false, int MINW = 1,
          int ACT = ACT_NONE>
__global__ __launch_bounds__(64 * WM * WN, MINW) void gemm_bf16_kernel(int M, int N, int K, Operand A, Operand B,
                                                                        Epilogue ep) {
  constexpr int NT = 64 * WM * WN;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int KSTEPS = BKT / 16;
  typedef typename TileSel<BM, BKT, NT, AKS>::type TA;
  typedef typename TileSel<BN, BKT, NT, BKS>::type TB;
  constexpr int kABytes = TA::kBytes;
  constexpr int kStage = TA::kBytes + TB::kBytes;
  constexpr int kLoadsPerStage = TA::kLoads + TB::kLoads;
  static_assert(NS >= 2 && NS <= kMaxStages, "2..5 stages");
  static_assert(MI % NI == 0 && MI % 2 == 0, "wave tile: rows a multiple of columns, at least 64 rows");

  // One __shared__ array per stage: distinct objects, so that the compiler's alias analysis
  // can tell a stage that is being filled from the one that is being read.
  __shared__ __attribute__((aligned(1024))) char stage0[kStage];
  __shared__ __attribute__((aligned(1024))) char stage1[kStage];
  __shared__ __attribute__((aligned(1024))) char stage2[NS > 2 ? kStage : 16];
  __shared__ __attribute__((aligned(1024))) char stage3[NS > 3 ? kStage : 16];
  __shared__ __attribute__((aligned(1024))) char stage4[NS > 4 ? kStage : 16];
  auto stage = [&](int s) -> char* {
    switch (s) {
      case 0: return stage0;
      case 1: return stage1;
      case 2: return stage2;
      case 3: return stage3;
      default: return stage4;
    }
  };

  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int pid = blockIdx.x, part = -1, kbeg = 0;
  int nk = (K + BKT - 1) / BKT;
  if (ep.split_s > 0 && pid >= ep.split_first) {
    const int j = pid - ep.split_first;
    pid = ep.split_first + j / ep.split_s;
    part = j % ep.split_s;
    const int per = (nk + ep.split_s - 1) / ep.split_s;
    kbeg = part * per;
    nk = (nk < kbeg + per ? nk : kbeg + per) - kbeg;   // > 0: the host sizes split_s so
  }
  int tm, tn;
  if (ep.square_map) tile_of_square(pid, tiles_n, tm, tn);
  else tile_of(pid, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, half = lane >> 5;

  // A wave tile of more than 128 accumulator registers leaves no room for them beside the
  // operands in the 256 ordinary registers: they live in the accumulation half of the file.
  // Defined there by an MFMA of zeros and pinned, or the register allocator would carry them
  // through the loop in ordinary registers and copy every tile in and out around each MFMA.
  constexpr bool kAccInAgprs = MINW == 1 && MI * NI * 16 > 128;
  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      if constexpr (kAccInAgprs) {
        const bf16x8 z = {};
        const f32x16 zero = {};
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(z, z, zero, 0, 0, 0);
        asm volatile("" : "+a"(acc[i][j]));
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
      }
    }

  int a_base[MI], b_base[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) a_base[i] = TA::frag_base(wm * TM + i * 32, l32, half);
#pragma unroll
  for (int j = 0; j < NI; ++j) b_base[j] = kABytes + TB::frag_base(wn * TN + j * 32, l32, half);

  bf16x8 af[2][MI], bfr[2][NI];
  // one load of k-tile kt (A loads first, then B loads) into the stage at LDS address dst
  // (the lane offsets are computed once; a k-tile that reaches beyond K takes the general form)
  uint32_t a_voff[VG ? 1 : TA::kLoads], b_voff[VG ? 1 : TB::kLoads];
  if constexpr (!VG) {
#pragma unroll
    for (int l = 0; l < TA::kLoads; ++l) a_voff[l] = TA::lane_offset(A, m0, l);
#pragma unroll
    for (int l = 0; l < TB::kLoads; ++l) b_voff[l] = TB::lane_offset(B, n0, l);
  }
  auto issue_load = [&](int kt, uint32_t dst, int idx) {
    const int k0 = (kbeg + kt) * BKT;
    if (idx < TA::kLoads) {
      if (TA::fast_ok(k0, K)) TA::issue_fast(TA::tile_rsrc(A, m0, k0, K), dst, idx, a_voff[VG ? 0 : idx]);
      else TA::issue_one(A, m0, k0, K, dst, idx);
    } else {
      const int j = idx - TA::kLoads;
      if (TB::fast_ok(k0, K)) TB::issue_fast(TB::tile_rsrc(B, n0, k0, K), dst + kABytes, j, b_voff[VG ? 0 : j]);
      else TB::issue_one(B, n0, k0, K, dst + kABytes, j);
    }
  };
  auto mfma_row = [&](int set, int i) {
#pragma unroll
    for (int j = 0; j < NI; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bfr[set][j], acc[i][j], 0, 0, 0);
  };
  // the part of k-step kk's fragments that is fetched while MFMA row i runs
  auto read_frag_part = [&](const char* tile, int kk, int set, int i) {
    if constexpr (MI == NI && MI % 2 == 0) {
      // square wave tile, one wave per SIMD: nothing hides a late fragment, so the column
      // fragments (all needed by the next k-step's first group) are read first, two per group,
      // then the row fragments in the order the groups use them: every fragment is requested
      // at least two groups (8 MFMAs) before its first use
      const int first = 2 * i;
#pragma unroll
      for (int q = first; q < first + 2; ++q) {
        if (q < NI) bfr[set][q] = TB::frag(tile, b_base[q], kk);
        else af[set][q - NI] = TA::frag(tile, a_base[q - NI], kk);
      }
      return;
    }
    af[set][i] = TA::frag(tile, a_base[i], kk);
#pragma unroll
    for (int j = 0; j < NI; ++j)
      if (j * MI / NI == i && (j * MI) % NI == 0) bfr[set][j] = TB::frag(tile, b_base[j], kk);
  };

  // Ring: stage kt % NS holds k-tile kt.  One "group" = one 32-row block of MFMAs (NI of
  // them); memory instructions are issued between groups so that they hide in the shadow of
  // the matrix pipe: the loads of tile kt+NS-1 are spread over the first kSpread groups of
  // iteration kt, and the fragment reads of k-step kk+1 over the groups of k-step kk.
  constexpr int kGroups = KSTEPS * MI;
  constexpr int kSpread = NS == 2 ? 4 : kGroups;   // with 2 stages the tile is needed at the end: request it at once
  constexpr int LPG = (kLoadsPerStage + kSpread - 1) / kSpread;
  // loads of the refill tile issued before the barrier of an iteration
  constexpr int kGroupsBeforeBarrier = (KSTEPS - 1) * MI + MI / 2;
  constexpr int kIssuedBeforeBarrier =
      (kGroupsBeforeBarrier * LPG < kLoadsPerStage ? kGroupsBeforeBarrier * LPG : kLoadsPerStage);
  constexpr int kWaitSteady = NS == 2 ? 0 : (NS - 3) * kLoadsPerStage + kIssuedBeforeBarrier;
  static_assert(kWaitSteady < 64, "too many loads in flight for the 6-bit vmcnt");

  if constexpr (VG) {
    // Register-staged loads (two LDS stages): tile kt+2 travels in registers while tile kt is
    // multiplied; at the start of iteration kt the registers (tile kt+1, loaded one iteration
    // ago) are written to the free stage and immediately reloaded, one chunk per MFMA group.
    static_assert(NS == 2, "register staging uses two LDS stages");
    constexpr int L = kLoadsPerStage;
    constexpr int kGroupsV = KSTEPS * MI;
    constexpr int kBefore = (KSTEPS - 1) * MI + MI / 2;      // groups before the barrier
    u32x4 regs[L];
    auto vload = [&](int kt, int idx) {
      regs[idx] = idx < TA::kLoads ? TA::load_one(A, m0, (kbeg + kt) * BKT, K, idx)
                                   : TB::load_one(B, n0, (kbeg + kt) * BKT, K, idx - TA::kLoads);
    };
    auto vstore = [&](char* dst, int idx) {
      if (idx < TA::kLoads) TA::store_one(dst, idx, regs[idx]);
      else TB::store_one(dst + kABytes, idx - TA::kLoads, regs[idx]);
    };
#pragma unroll
    for (int l = 0; l < L; ++l) vload(0, l);
#pragma unroll
    for (int l = 0; l < L; ++l) vstore(stage(0), l);
    __syncthreads();
#pragma unroll
    for (int l = 0; l < L; ++l) vload(1, l);
#pragma unroll
    for (int i = 0; i < MI; ++i) read_frag_part(stage(0), 0, 0, i);
    for (int kt0 = 0; kt0 < nk; kt0 += 2) {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const int kt = kt0 + s;
        if (kt < nk) {
          const char* cur = stage(s);
          char* nxt = stage(s ^ 1);
          if constexpr (MI == 4 && NI == 4 && KSTEPS == 4 && L == 16) {
            // One wave per SIMD (128 x 128 wave tile): nobody covers for a wave whose MFMA is held
            // up behind several memory instructions that wait to be issued, so the iteration's 64
            // memory instructions (16 LDS writes, 16 global loads, 32 fragment reads) go one into
            // each of the 64 gaps between its MFMAs.  MFMA n = (k-step n / 16, row block, column
            // block); in k-steps 0..2 the odd gaps read the next k-step's eight fragments (columns
            // first: the next k-step's first MFMAs need all four) and the even gaps alternate "write
            // chunk t to LDS" and "reload its register"; the first half of k-step 3 does the last
            // four chunks, the barrier follows, and the second half reads the next tile's first
            // fragments.  (Reading the fragments in the exact order of their use, or the barrier
            // four MFMAs earlier, lengthens register lifetimes enough to spill in the k-strided
            // layouts, and gains nothing in the k-contiguous one.)
#pragma unroll
            for (int n = 0; n < 64; ++n) {
              const int kk = n / 16, i = (n / 4) % 4, j = n % 4, e = n % 16;
              if (n == 56) __syncthreads();   // tile kt+1 is complete in `nxt`; nobody reads `cur` any more
              __builtin_amdgcn_sched_barrier(0);
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
              __builtin_amdgcn_sched_barrier(0);
              if (n >= 56) {
                const int q = n - 56;
                if (q < 4) bfr[0][q] = TB::frag(nxt, b_base[q], 0);
                else af[0][q - 4] = TA::frag(nxt, a_base[q - 4], 0);
              } else if (kk < 3 && (e & 1)) {
                const int q = e / 2, set = (kk + 1) & 1;
                if (q < 4) bfr[set][q] = TB::frag(cur, b_base[q], kk + 1);
                else af[set][q - 4] = TA::frag(cur, a_base[q - 4], kk + 1);
              } else {
                const int t = kk < 3 ? kk * 8 + e / 2 : 24 + (n - 48);
                if (t % 2 == 0) vstore(nxt, t / 2);
                else vload(kt + 2, t / 2);
              }
            }
          } else {
#pragma unroll
          for (int kk = 0; kk < KSTEPS; ++kk) {
#pragma unroll
            for (int i = 0; i < MI; ++i) {
              const int grp = kk * MI + i;
              if (kk == KSTEPS - 1 && i == MI / 2) {
                __syncthreads();  // tile kt+1 is complete in `nxt`; nobody reads `cur` any more
              }
              // A group's memory work sits between its MFMAs, not in front of them: the wave
              // issues an MFMA, then its LDS write while the matrix pipe works on it, then the
              // next MFMA, then the global load and the fragment reads.  The LDS write and the
              // load that refills its register are in different gaps, so the load is not held
              // up behind the write's wait for the register.  After the barrier the fragments of
              // the next tile's first k-step are fetched the same way, spread over the two
              // groups that remain (set 0; the last k-step multiplies from set 1).
              static_assert((KSTEPS - 1) % 2 == 1, "the last k-step must use fragment set 1");
              const bool after_barrier = kk == KSTEPS - 1 && i >= MI / 2;
              __builtin_amdgcn_sched_barrier(0);
              acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][0], acc[i][0], 0, 0, 0);
              __builtin_amdgcn_sched_barrier(0);
#pragma unroll
              for (int idx = 0; idx < L; ++idx)
                if (idx * kBefore / L == grp) vstore(nxt, idx);   // chunks spread evenly over the groups before the barrier
              if (after_barrier && i == MI / 2) {
#pragma unroll
                for (int j = 0; j < NI; ++j) bfr[0][j] = TB::frag(nxt, b_base[j], 0);
              }
              __builtin_amdgcn_sched_barrier(0);
#pragma unroll
              for (int j = 1; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
              __builtin_amdgcn_sched_barrier(0);
#pragma unroll
              for (int idx = 0; idx < L; ++idx)
                if (idx * kBefore / L == grp) vload(kt + 2, idx);  // the slot just written is reloaded
              if (kk + 1 < KSTEPS) read_frag_part(cur, kk + 1, (kk + 1) & 1, i);
              if (after_barrier) {
                const int first = (i - MI / 2) * 2;      // two A fragments per group after the barrier
#pragma unroll
                for (int ii = first; ii < first + 2 && ii < MI; ++ii) af[0][ii] = TA::frag(nxt, a_base[ii], 0);
              }
            }
          }
          }
        }
      }
    }
    (void)kGroupsV;
  } else {
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
#pragma unroll
    for (int l = 0; l < kLoadsPerStage; ++l) issue_load(s, lds_addr_of(stage(s)), l);
  wait_loads_and_barrier<(NS - 2) * kLoadsPerStage>();  // tile 0 has landed for every wave
#pragma unroll
  for (int i = 0; i < MI; ++i) read_frag_part(stage(0), 0, 0, i);

  for (int kt0 = 0; kt0 < nk; kt0 += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int kt = kt0 + s;
      if (kt < nk) {
        const char* cur = stage(s);
        const char* nxt = stage((s + 1) % NS);
        const uint32_t refill = lds_addr_of(stage((s + NS - 1) % NS));  // held tile kt-1: free since the last barrier
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
#pragma unroll
          for (int i = 0; i < MI; ++i) {
            const int grp = kk * MI + i;
            if (kk == KSTEPS - 1 && i == MI / 2) {
              // tile kt+1 must have landed in every wave's share, and every wave must be done
              // reading `cur` before the next iteration refills it
              wait_loads_and_barrier<kWaitSteady>();
#pragma unroll
              for (int ii = 0; ii < MI; ++ii) read_frag_part(nxt, 0, 0, ii);
            }
#pragma unroll
            for (int l = 0; l < LPG; ++l)
              if (grp < kSpread && grp * LPG + l < kLoadsPerStage) issue_load(kt + NS - 1, refill, grp * LPG + l);
            if (kk + 1 < KSTEPS) read_frag_part(cur, kk + 1, (kk + 1) & 1, i);
            __builtin_amdgcn_sched_barrier(0);
            mfma_row(kk & 1, i);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  }
  }
  wait_loads_and_barrier<0>();  // nothing in flight, all operands consumed: LDS is free

  // ---- epilogue -------------------------------------------------------------------------
  // Accumulator register r of lane (l32, half) is C[8*(r/4) + 4*half + r%4][l32] of its 32x32
  // block.  Each wave stages one 32 x TN row block at a time in its private LDS region and
  // reads it back row-major, 4 consecutive columns per lane.
  constexpr int LDW = TN + 8;                 // padded row length in floats: lanes 32..63 (4 rows down) land 32 banks away
  constexpr int LPR = TN / 4;                 // lanes per row
  constexpr int RPI = 64 / LPR;               // rows per wave instruction
  constexpr int kSteps = 32 / RPI;
  constexpr int kRegion = 32 * LDW * 4;       // bytes per wave
  constexpr int kWavesPerStage = kStage / kRegion;
  static_assert(kWavesPerStage >= 1 && kWavesPerStage * NS >= NT / 64, "epilogue staging must fit in LDS");
  float* stg = reinterpret_cast<float*>(stage(wave / kWavesPerStage) + (wave % kWavesPerStage) * kRegion);
  const int erow = lane / LPR, ecol = (lane % LPR) * 4;
  if (part >= 0) {
    // k-range of a split tile: the whole fp32 tile goes to its slot of the workspace, row
    // major with BN columns; bias, residual and the conversion happen in the fix-up kernel
    float* dst = ep.split_ws + ((size_t)(pid - ep.split_first) * ep.split_s + part) * (size_t)(BM * BN);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      wave_lds_sync();
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          stg[(8 * (r >> 2) + 4 * half + (r & 3)) * LDW + j * 32 + l32] = acc[i][j][r];
      wave_lds_sync();
#pragma unroll
      for (int st = 0; st < kSteps; ++st) {
        const int row = wm * TM + i * 32 + st * RPI + erow;
        *reinterpret_cast<f32x4*>(dst + (size_t)row * BN + wn * TN + ecol) =
            *reinterpret_cast<const f32x4*>(stg + (st * RPI + erow) * LDW + ecol);
      }
    }
    return;
  }
  const int n = n0 + wn * TN + ecol;
  const bool n_ok = n < N;
  f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
  if (ep.bias && n_ok) {
    const bf16x4 b = *reinterpret_cast<const bf16x4*>(ep.bias + n);
#pragma unroll
    for (int e = 0; e < 4; ++e) bias4[e] = (float)b[e];
  }
  constexpr bool kActBwd = ACT == ACT_BWD_ERF || ACT == ACT_BWD_TANH;
  // A tile that lies wholly inside the matrix: no access is predicated and the output mode is
  // a compile-time constant of the pass, so the pass is straight-line code whose loads and
  // stores are all in flight together.  (Behind a branch the compiler waits for everything
  // outstanding, the previous row step's store included, before it uses a loaded register: an
  // accumulating tile then pays 32 store round trips one after the other.)  Everything a row
  // block reads from memory -- the gradient rows of an accumulating output, for which the NEXT
  // block's rows are requested too, the residual, the pre-activations -- is requested before
  // the block is staged.
  auto full_tile_pass = [&](auto mode_c, auto res_c) {
    constexpr int MODE = decltype(mode_c)::value;
    constexpr bool RES = decltype(res_c)::value;
    constexpr bool ACC = MODE == OUT_ACC_F32;
    f32x4 prev[ACC ? 2 : 1][kSteps];
    bf16x4 resv[RES ? kSteps : 1];
    bf16x4 hpre[kActBwd ? kSteps : 1];
    auto index = [&](int i, int s) { return (size_t)(m0 + wm * TM + i * 32 + s * RPI + erow) * ep.ldc + n; };
    auto load_prev = [&](int i) {
#pragma unroll
      for (int s = 0; s < kSteps; ++s)
        prev[ACC ? i & 1 : 0][s] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(ep.C) + index(i, s));
    };
    if constexpr (ACC) load_prev(0);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      if constexpr (ACC) {
        if (i + 1 < MI) load_prev(i + 1);
      }
      if constexpr (RES) {
#pragma unroll
        for (int s = 0; s < kSteps; ++s) resv[s] = *reinterpret_cast<const bf16x4*>(ep.residual + index(i, s));
      }
      if constexpr (kActBwd) {
#pragma unroll
        for (int s = 0; s < kSteps; ++s) hpre[s] = *reinterpret_cast<const bf16x4*>(ep.aux + index(i, s));
      }
      wave_lds_sync();  // the previous pass's reads are done before its region is rewritten
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          stg[(8 * (r >> 2) + 4 * half + (r & 3)) * LDW + j * 32 + l32] = acc[i][j][r];
      wave_lds_sync();
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        f32x4 v = *reinterpret_cast<const f32x4*>(stg + (s * RPI + erow) * LDW + ecol);
        const size_t idx = index(i, s);
        v += bias4;
        if constexpr (RES) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += (float)resv[s][e];
        }
        if constexpr (ACT != ACT_NONE) {
          store_bf16x4_act<ACT>(ep, idx, v, hpre[kActBwd ? s : 0]);
        } else if constexpr (MODE == OUT_STORE) {
          store_bf16x4_act<ACT_NONE>(ep, idx, v);
        } else if constexpr (MODE == OUT_STORE_F32) {
          *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.C) + idx) = v;
        } else {
          *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.C) + idx) = prev[i & 1][s] + v;
        }
      }
    }
  };
  if (m0 + BM <= M && n0 + BN <= N) {
    using std::integral_constant;
    if constexpr (ACT != ACT_NONE) {
      full_tile_pass(integral_constant<int, OUT_STORE>{}, std::false_type{});
    } else if (ep.out_mode == OUT_ACC_F32) {
      full_tile_pass(integral_constant<int, OUT_ACC_F32>{}, std::false_type{});
    } else if (ep.out_mode == OUT_STORE_F32) {
      full_tile_pass(integral_constant<int, OUT_STORE_F32>{}, std::false_type{});
    } else if (ep.residual) {
      full_tile_pass(integral_constant<int, OUT_STORE>{}, std::true_type{});
    } else {
      full_tile_pass(integral_constant<int, OUT_STORE>{}, std::false_type{});
    }
    return;
  }
  // a tile that crosses the matrix's edge: every access predicated, the mode chosen per store
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int mbase = m0 + wm * TM + i * 32;
    f32x4 prev[kSteps];
    if (ep.out_mode == OUT_ACC_F32) {
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const int m = mbase + s * RPI + erow;
        if (n_ok && m < M)
          prev[s] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(ep.C) + (size_t)m * ep.ldc + n);
      }
    }
    // backward GeLU: the block's pre-activations are requested before the staging pass, so
    // that their latency is spent there and not once per row step
    bf16x4 hpre[kActBwd ? kSteps : 1];
    if constexpr (kActBwd) {
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const int m = mbase + s * RPI + erow;
        hpre[s] = bf16x4{};
        if (n_ok && m < M) hpre[s] = *reinterpret_cast<const bf16x4*>(ep.aux + (size_t)m * ep.ldc + n);
      }
    }
    wave_lds_sync();  // the previous pass's reads are done before its region is rewritten
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stg[(8 * (r >> 2) + 4 * half + (r & 3)) * LDW + j * 32 + l32] = acc[i][j][r];
    wave_lds_sync();
    if constexpr (ACT != ACT_NONE) {
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const int m = mbase + s * RPI + erow;
        if (!(n_ok && m < M)) continue;
        f32x4 v = *reinterpret_cast<const f32x4*>(stg + (s * RPI + erow) * LDW + ecol);
        v += bias4;
        store_bf16x4_act<ACT>(ep, (size_t)m * ep.ldc + n, v, hpre[kActBwd ? s : 0]);
      }
      continue;
    }
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      const int m = mbase + s * RPI + erow;
      if (!(n_ok && m < M)) continue;
      f32x4 v = *reinterpret_cast<const f32x4*>(stg + (s * RPI + erow) * LDW + ecol);
      const size_t idx = (size_t)m * ep.ldc + n;
      v += bias4;
      if (ep.residual) {
        const bf16x4 rv = *reinterpret_cast<const bf16x4*>(ep.residual + idx);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += (float)rv[e];
      }
      if (ep.out_mode == OUT_STORE) {
        store_bf16x4_act<ACT_NONE>(ep, idx, v);
      } else if (ep.out_mode == OUT_STORE_F32) {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.C) + idx) = v;
      } else {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.C) + idx) = prev[s] + v;
      }
    }
  }
}

// Sums the split_s partial tiles of every split tile in ascending k order, adds bias and
// residual and stores in the output mode (for an accumulating output: adds the sum to the fp32
// gradient, which this kernel alone touches).  One thread per 4 consecutive columns.
template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_split_fixup_kernel(int M, int N, Epilogue ep, int n_split) {
  constexpr int kQuads = BM * BN / 4;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  for (long long q = blockIdx.x * 256LL + threadIdx.x; q < (long long)n_split * kQuads; q += 256LL * gridDim.x) {
    const int t = (int)(q / kQuads), e = (int)(q % kQuads);
    const int row = e / (BN / 4), col = (e % (BN / 4)) * 4;
    int tm, tn;
    tile_of(ep.split_first + t, tiles_m, tiles_n, tm, tn);
    const int m = tm * BM + row, n = tn * BN + col;
    if (m >= M || n >= N) continue;
    const float* src = ep.split_ws + (size_t)t * ep.split_s * (size_t)(BM * BN) + (size_t)row * BN + col;
    f32x4 v = *reinterpret_cast<const f32x4*>(src);
    for (int p = 1; p < ep.split_s; ++p) v += *reinterpret_cast<const f32x4*>(src + (size_t)p * (BM * BN));
    const size_t idx = (size_t)m * ep.ldc + n;
    if (ep.bias) {
      const bf16x4 b = *reinterpret_cast<const bf16x4*>(ep.bias + n);
#pragma unroll
      for (int c = 0; c < 4; ++c) v[c] += (float)b[c];
    }
    if (ep.residual) {
      const bf16x4 rv = *reinterpret_cast<const bf16x4*>(ep.residual + idx);
#pragma unroll
      for (int c = 0; c < 4; ++c) v[c] += (float)rv[c];
    }
    if (ep.out_mode == OUT_STORE) {
      store_bf16x4_act_rt(ep, idx, v);
    } else if (ep.out_mode == OUT_STORE_F32) {
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.C) + idx) = v;
    } else {
      float* g = reinterpret_cast<float*>(ep.C) + idx;
      *reinterpret_cast<f32x4*>(g) = *reinterpret_cast<const f32x4*>(g) + v;
    }
  }
}

// How the tail of a launch is split.  A launch of `tiles` workgroups runs in rounds of `slots`
// (CUs x workgroups per CU); when the last round is at most half full its tiles are cut into
// s k-ranges each, so that the round is as short as 1/s of a full one.
struct SplitPlan { int first; int s; size_t bytes; };
template <int BM, int BN, int BKT, int WGS_PER_CU>
SplitPlan plan_split(int M, int N, int K, int out_mode) {
  SplitPlan p{0, 0, 0};
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const int slots = kCus * WGS_PER_CU;
  const int rem = tiles % slots;
  const int nk = (K + BKT - 1) / BKT;
  if (out_mode == OUT_ACC_F32) {
    // A weight gradient: a long contraction into an output that may be smaller than the chip
    // (6144 x 2048 is 192 tiles, 2048 x 2048 is 64).  With at most two rounds of tiles, ALL of
    // them are cut into the s <= 8 ranges of k (16 k-steps or more each) that fill the rounds
    // best; the fix-up kernel then adds the partial sums, in ascending k order, to the gradient
    // exactly once.  Larger outputs keep the one-pass read-modify-write for their full rounds
    // and have a last round that is at most half full cut like a store-mode output's (below:
    // 50304 x 4096, a vocabulary's gradient, is 12.3 rounds).
    if (tiles < 2 * slots) {
    int best = 1;
    double best_eff = (double)tiles / ((double)((tiles + slots - 1) / slots) * slots);
    for (int s = 2; s <= 8 && nk / s >= 16; ++s) {
      const long long wgs = (long long)tiles * s;
      const double eff = (double)wgs / ((double)((wgs + slots - 1) / slots) * slots);
      if (eff > best_eff + 0.05) { best_eff = eff; best = s; }
    }
    if (best < 2) return p;
    const int per = (nk + best - 1) / best;
    best = (nk + per - 1) / per;             // no empty part
    if (best < 2) return p;
    p.first = 0;
    p.s = best;
    p.bytes = (size_t)tiles * best * BM * BN * 4;
    return p;
    }
  }
  if (rem == 0 || rem * 2 > slots) return p;
  int s = slots / rem;
  if (s > 8) s = 8;
  if (s > nk / 4) s = nk / 4;              // at least 4 k-steps per part
  if (s < 2) return p;
  const int per = (nk + s - 1) / s;
  s = (nk + per - 1) / per;                // no empty part
  if (s < 2) return p;
  p.first = tiles - rem;
  p.s = s;
  p.bytes = (size_t)rem * s * BM * BN * 4;
  return p;
}

template <int BM, int BN, int BKT, int NS, int WM, int WN, bool AKS, bool BKS, bool VG = false, int MINW = 1,
          int ACT = ACT_NONE>
hipError_t launch_cfg(const GemmDesc& g, hipStream_t s) {
  constexpr int NT = 64 * WM * WN;
  constexpr int kWgsPerCu = BM * BN >= 256 * 256 ? 1 : 2;
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  Operand A{(const bf16*)g.A, g.lda, g.M};
  Operand B{(const bf16*)g.B, g.ldb, g.N};
  Epilogue ep{g.C, g.ldc, g.out_mode, (const bf16*)g.bias, (const bf16*)g.residual, 0, 0, nullptr, 0, ACT, (bf16*)g.aux};
  {
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    ep.square_map = BM == 256 && BN == 256 && g.out_mode == OUT_ACC_F32 && tiles_m % 16 == 0 && tiles_n % 16 == 0;
  }
  int grid = tiles;
  const SplitPlan sp = plan_split<BM, BN, BKT, kWgsPerCu>(g.M, g.N, g.K, g.out_mode);
  const bool split = g.workspace && sp.s >= 2 && sp.bytes <= g.workspace_bytes;
  if (split) {
    ep.split_first = sp.first; ep.split_s = sp.s; ep.split_ws = (float*)g.workspace;
    ep.square_map = 0;                 // the fix-up kernel numbers tiles with tile_of
    grid = sp.first + (tiles - sp.first) * sp.s;
  }
  gemm_bf16_kernel<BM, BN, BKT, NS, WM, WN, AKS, BKS, VG, MINW, ACT><<<grid, NT, 0, s>>>(g.M, g.N, g.K, A, B, ep);
  if (split) {
    const long long quads = (long long)(tiles - sp.first) * (BM * BN / 4);
    const int blocks = (int)((quads + 255) / 256 < 4096 ? (quads + 255) / 256 : 4096);
    gemm_split_fixup_kernel<BM, BN><<<blocks, 256, 0, s>>>(g.M, g.N, ep, tiles - sp.first);
  }
  return hipGetLastError();
}

template <int BM, int BN, int BKT, int NS, int WM, int WN, bool VG = false, int MINW = 1>
hipError_t launch_layout(const GemmDesc& g, hipStream_t s) {
  if (!g.a_kstrided && !g.b_kstrided) return launch_cfg<BM, BN, BKT, NS, WM, WN, false, false, VG, MINW>(g, s);
  if (!g.a_kstrided && g.b_kstrided) return launch_cfg<BM, BN, BKT, NS, WM, WN, false, true, VG, MINW>(g, s);
  if (g.a_kstrided && g.b_kstrided) return launch_cfg<BM, BN, BKT, NS, WM, WN, true, true, VG, MINW>(g, s);
  return launch_cfg<BM, BN, BKT, NS, WM, WN, true, false, VG, MINW>(g, s);
}

int g_variant = 0;

}  // namespace

bool gemm_bf16_shape_ok(const GemmDesc& g, std::string& why) {
  auto mult8 = [](long long v) { return v > 0 && v % 8 == 0; };
  if (!mult8(g.M) || !mult8(g.N) || !mult8(g.K) || !mult8(g.lda) || !mult8(g.ldb) || !mult8(g.ldc)) {
    why = "bf16 GEMM needs M, N, K and leading dimensions to be positive multiples of 8";
    return false;
  }
  // tile-local offsets are 32-bit byte offsets: 256 rows (k-contig) or 64 k-rows (k-strided) of ld
  const long long a_span = (g.a_kstrided ? 64LL : 256LL) * g.lda * 2;
  const long long b_span = (g.b_kstrided ? 64LL : 256LL) * g.ldb * 2;
  if (a_span >= (long long)kMaxRecords || b_span >= (long long)kMaxRecords) {
    why = "leading dimension too large for 32-bit tile offsets";
    return false;
  }
  if ((g.a_kstrided ? g.lda < g.M : g.lda < g.K) || (g.b_kstrided ? g.ldb < g.N : g.ldb < g.K) || g.ldc < g.N) {
    why = "leading dimension smaller than the row length";
    return false;
  }
  if (g.bias && ((uintptr_t)g.bias % 8) != 0) { why = "bias must be 8-byte aligned"; return false; }
  if (g.act != ACT_NONE && (g.act < ACT_FWD_ERF || g.act > ACT_BWD_TANH || !g.aux || g.out_mode != OUT_STORE ||
                            ((uintptr_t)g.aux % 8) != 0 || g.aux == g.C)) {
    why = "a fused activation needs a storage-type output, and a second tensor of its shape that is not the output";
    return false;
  }
  return true;
}

void set_gemm_variant(int v) { g_variant = v; }

namespace {
// The automatic tile choice: large tiles when they still give every CU work, smaller ones
// otherwise.  An accumulating output (a weight gradient) with a long contraction also takes the
// large tiles when cutting them along k fills the chip (plan_split) and the caller's scratch
// holds the partial tiles; `scratch_bytes` = what the caller offers (SIZE_MAX: assume enough).
bool use_large_tiles(int M, int N, int K, int out_mode, size_t scratch_bytes) {
  const long long big_tiles = (long long)((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 192) return true;
  if (out_mode != OUT_ACC_F32) return false;
  const SplitPlan sp = plan_split<256, 256, 64, 1>(M, N, K, out_mode);
  return sp.s >= 2 && big_tiles * sp.s >= 192 && sp.bytes <= scratch_bytes;
}
}  // namespace

size_t gemm_bf16_workspace_bytes(int M, int N, int K, int out_mode) {
  // mirrors the automatic choice of launch_gemm_bf16
  if (use_large_tiles(M, N, K, out_mode, (size_t)-1)) return plan_split<256, 256, 64, 1>(M, N, K, out_mode).bytes;
  return plan_split<128, 128, 64, 2>(M, N, K, out_mode).bytes;
}

namespace {
// The fused-GeLU instantiations: the two automatically chosen tile configurations, forward in
// the forward layout (both operands k-contiguous), backward in the input-gradient layout.
template <int BM, int BN, int WN, int MINW>
hipError_t launch_act(const GemmDesc& g, hipStream_t s) {
  switch (g.act) {
    case ACT_FWD_ERF: return launch_cfg<BM, BN, 64, 2, 2, WN, false, false, true, MINW, ACT_FWD_ERF>(g, s);
    case ACT_FWD_TANH: return launch_cfg<BM, BN, 64, 2, 2, WN, false, false, true, MINW, ACT_FWD_TANH>(g, s);
    case ACT_BWD_ERF: return launch_cfg<BM, BN, 64, 2, 2, WN, false, true, true, MINW, ACT_BWD_ERF>(g, s);
    default: return launch_cfg<BM, BN, 64, 2, 2, WN, false, true, true, MINW, ACT_BWD_TANH>(g, s);
  }
}
}  // namespace

hipError_t launch_gemm_bf16(const GemmDesc& g, hipStream_t s) {
  if (g.act != ACT_NONE) {
    const bool fwd = g.act == ACT_FWD_ERF || g.act == ACT_FWD_TANH;
    const bool layout_ok = !g.a_kstrided && g.b_kstrided == !fwd;
    const bool tiles_ok = g_variant == 0 || g_variant == 6 || g_variant == 7;
    if (g.out_mode == OUT_STORE && layout_ok && tiles_ok) {
      const bool large = g_variant == 6 || (g_variant == 0 && use_large_tiles(g.M, g.N, g.K, g.out_mode, 0));
      return large ? launch_act<256, 256, 4, 2>(g, s) : launch_act<128, 128, 2, 2>(g, s);
    }
    // another layout or a forced tile configuration: the plain GEMM, then the element-wise
    // kernel (in place for the backward: C holds da, then dh) -- the same bits
    GemmDesc plain = g;
    plain.act = ACT_NONE;
    plain.aux = nullptr;
    hipError_t e = launch_gemm_bf16(plain, s);
    if (e != hipSuccess) return e;
    const int act = (g.act == ACT_FWD_ERF || g.act == ACT_BWD_ERF) ? JPP_GELU : JPP_GELU_TANH;
    if (g.ldc != g.N) return hipErrorInvalidValue;   // the element-wise kernels take dense rows
    return fwd ? launch_act_fwd(JPP_BF16, act, g.M, g.N, g.C, g.aux, s)
               : launch_act_bwd(JPP_BF16, act, g.M, g.N, g.aux, g.C, g.C, s);
  }
  switch (g_variant) {
    case 1: return launch_layout<256, 256, 32, 4, 2, 2>(g, s);
    case 2: return launch_layout<256, 256, 32, 5, 2, 2>(g, s);
    case 3: return launch_layout<128, 128, 32, 4, 2, 2, false, 2>(g, s);
    case 4: return launch_layout<256, 256, 64, 2, 2, 2>(g, s);
    case 5: return launch_layout<256, 256, 64, 2, 2, 4, false, 2>(g, s);
    case 6: return launch_layout<256, 256, 64, 2, 2, 4, true, 2>(g, s);
    case 7: return launch_layout<128, 128, 64, 2, 2, 2, true, 2>(g, s);
    case 8: return launch_layout<256, 256, 64, 2, 2, 2, true, 1>(g, s);
    default: break;
  }
  if (use_large_tiles(g.M, g.N, g.K, g.out_mode, g.workspace ? g.workspace_bytes : 0))
    return launch_layout<256, 256, 64, 2, 2, 4, true, 2>(g, s);
  return launch_layout<128, 128, 64, 2, 2, 2, true, 2>(g, s);
}

}  // namespace jpp
