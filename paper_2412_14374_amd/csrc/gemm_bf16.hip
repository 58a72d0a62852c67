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
// Design (one workgroup = one BM x BN tile of C, BK = 64, two LDS stages):
//  * LDS holds each operand tile as [rows][64 k] bf16, 128 bytes per row, with the 16-byte
//    chunk index XOR-swizzled by ((row ^ row>>3) & 7): the 16-byte MFMA fragment reads
//    (lanes = consecutive rows, same k chunk) and the transposing staging writes (lanes =
//    rows 8 apart) both spread over all banks.
//  * A k-contiguous operand goes HBM -> LDS directly (buffer_load ... lds): each wave
//    instruction fills 1 KiB of LDS in lane order, and the swizzle is applied by choosing
//    which global chunk each lane fetches.  No VGPRs and no ds_write are spent on it.
//  * A k-strided operand is transposed on the way in: a thread loads an 8(k) x 8(row) block
//    as eight 16-byte row segments, transposes it in registers with byte permutes and writes
//    eight 16-byte k-runs.  The MFMA loop is identical for all four layout combinations.
//  * Rows beyond the matrix read as zero through the buffer range check, the contiguous
//    dimension is predicated, so M, N, K need only be multiples of 8.
//  * MFMA fragments are double-buffered in registers: the LDS reads of k-step kk+1 are issued
//    before the MFMAs of k-step kk.
//  * Epilogue: accumulators go through LDS (free after the main loop) so that every global
//    access is 8 or 16 bytes per lane on full rows; the fp32 gradient tile is read with
//    16-byte loads issued before the staging.
//  * Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs)
//    works on a contiguous band of tiles and shares operand panels in its own L2.
#include "device_utils.h"
#include "internal.h"

namespace jpp {

namespace {

constexpr int BK = 64;
constexpr int kRowBytes = BK * 2;  // 128
constexpr uint32_t kOOB = 0x7FFFFFFFu;
constexpr uint32_t kMaxRecords = 0x7FFFFF00u;

typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ inline int swz(int row) { return (row ^ (row >> 3)) & 7; }

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, long long bytes) {
  const uint32_t n = bytes > (long long)kMaxRecords ? kMaxRecords : (bytes < 0 ? 0u : (uint32_t)bytes);
  // 0x00020000: untyped raw buffer, 32-bit data format (gfx9 resource word 3)
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)n, 0x00020000);
}

struct Epilogue {
  void* C; int ldc; int out_mode;
  const bf16* bias; const bf16* residual;
};

struct Operand {
  const bf16* p; int ld; int rows;  // rows = M (for A) or N (for B)
};

// Transposes an 8x8 block of bf16: in[j] holds 8 consecutive rows' elements at k = j; out[r]
// holds 8 consecutive k at row r.
__device__ inline void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int w = r >> 1;
    const uint32_t sel = (r & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
    for (int p = 0; p < 4; ++p) out[r][p] = __builtin_amdgcn_perm(in[2 * p + 1][w], in[2 * p][w], sel);
  }
}

// k-contiguous operand, HBM -> LDS without registers.  Wave w, step i fills LDS rows
// [(i*NW + w)*8, +8): lane l lands on row (l>>3), physical chunk (l&7), and therefore
// fetches the logical chunk (l&7) ^ swz(row).
template <int R, int NT>
struct DirectLoader {
  static constexpr int NW = NT / 64;
  static constexpr int kSteps = R * 8 / NT;
  static_assert((R * 8) % NT == 0, "tile rows x 8 must be a multiple of the thread count");
  int wave, lane;
  __device__ inline void init(const Operand&, int) {
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    lane = threadIdx.x % 64;
  }
  __device__ inline void issue(const Operand& op, int r0, int k0, int K, char* tile) {
    const bf16* base = op.p + (size_t)r0 * op.ld + k0;
    const auto rs = make_rsrc(base, ((long long)(op.rows - r0) * op.ld - k0) * 2);
#pragma unroll
    for (int i = 0; i < kSteps; ++i) {
      const int rowblk = i * NW + wave;
      const int row = rowblk * 8 + (lane >> 3);
      const int kc = (lane & 7) ^ swz(row);
      const uint32_t off = (k0 + kc * 8 < K) ? (uint32_t)(row * op.ld + kc * 8) * 2u : kOOB;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(tile + rowblk * 1024), 16, (int)off, 0, 0, 0);
    }
  }
  __device__ inline void store(char*) {}
};

// k-strided operand: R units of 8(k) x 8(rows); unit u is handled by thread (u + PHASE) % NT.
template <int R, int NT, int PHASE>
struct TransposeLoader {
  static_assert(R <= NT, "expects at most one unit per thread");
  u32x4 regs[8];
  uint32_t goff[8];
  bool active;
  int unit;
  __device__ inline void init(const Operand& op, int r0) {
    unit = (threadIdx.x + NT - PHASE) % NT;
    active = unit < R;
    const int rb = unit % (R / 8), kb = unit / (R / 8);
    const bool col_ok = (r0 + rb * 8) < op.rows;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      goff[j] = (active && col_ok) ? (uint32_t)((kb * 8 + j) * op.ld + rb * 8) * 2u : kOOB;
  }
  __device__ inline void issue(const Operand& op, int r0, int k0, int K, char*) {
    const bf16* base = op.p + (size_t)k0 * op.ld + r0;
    const auto rs = make_rsrc(base, ((long long)(K - k0) * op.ld - r0) * 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) regs[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)goff[j], 0, 0);
  }
  __device__ inline void store(char* tile) {
    if (active) {
      u32x4 t[8];
      transpose8x8(regs, t);
      const int rb = unit % (R / 8), kb = unit / (R / 8);
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int row = rb * 8 + r;
        *reinterpret_cast<u32x4*>(tile + row * kRowBytes + ((kb ^ swz(row)) << 4)) = t[r];
      }
    }
  }
};

template <int R, int NT, bool KS, int PHASE>
struct LoaderSel { typedef DirectLoader<R, NT> type; };
template <int R, int NT, int PHASE>
struct LoaderSel<R, NT, true, PHASE> { typedef TransposeLoader<R, NT, PHASE> type; };

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

template <int BM, int BN, int WM, int WN, bool AKS, bool BKS>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_kernel(int M, int N, int K, Operand A, Operand B,
                                                                  Epilogue ep) {
  constexpr int NT = 64 * WM * WN;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int kABytes = BM * kRowBytes, kBBytes = BN * kRowBytes;
  constexpr int kStage = kABytes + kBBytes;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int tm, tn;
  tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, half = lane >> 5;

  typename LoaderSel<BM, NT, AKS, 0>::type la;
  typename LoaderSel<BN, NT, BKS, NT / 2>::type lb;
  la.init(A, m0);
  lb.init(B, n0);

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment addresses: byte offset of (row, chunk = half) inside a tile; the k-step kk adds
  // 2*kk to the chunk, i.e. XORs (2*kk) << 4 into the offset (swizzle and k-step commute).
  int a_off[MI], b_off[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int row = wm * TM + i * 32 + l32;
    a_off[i] = row * kRowBytes + ((half ^ swz(row)) << 4);
  }
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int row = wn * TN + j * 32 + l32;
    b_off[j] = kABytes + row * kRowBytes + ((half ^ swz(row)) << 4);
  }

  const int nk = (K + BK - 1) / BK;
  la.issue(A, m0, 0, K, lds);
  lb.issue(B, n0, 0, K, lds + kABytes);
  la.store(lds);
  lb.store(lds + kABytes);
  __syncthreads();

  bf16x8 af[2][MI], bfr[2][NI];
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = lds + (kt & 1) * kStage;
    char* nxt = lds + ((kt + 1) & 1) * kStage;
    const bool more = kt + 1 < nk;
    if (more) {
      la.issue(A, m0, (kt + 1) * BK, K, nxt);
      lb.issue(B, n0, (kt + 1) * BK, K, nxt + kABytes);
    }
#pragma unroll
    for (int i = 0; i < MI; ++i) af[0][i] = *reinterpret_cast<const bf16x8*>(cur + a_off[i]);
#pragma unroll
    for (int j = 0; j < NI; ++j) bfr[0][j] = *reinterpret_cast<const bf16x8*>(cur + b_off[j]);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) {
        const int x = ((kk + 1) * 2) << 4;
#pragma unroll
        for (int i = 0; i < MI; ++i)
          af[(kk + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(cur + (a_off[i] ^ x));
#pragma unroll
        for (int j = 0; j < NI; ++j)
          bfr[(kk + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(cur + (b_off[j] ^ x));
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      la.store(nxt);
      lb.store(nxt + kABytes);
    }
    __syncthreads();
  }

  // ---- epilogue -------------------------------------------------------------------------
  // Accumulator register r of lane (l32, half) is C[8*(r/4) + 4*half + r%4][l32] of its 32x32
  // block.  Each wave stages one 32 x TN row block at a time in its private LDS region and
  // reads it back row-major, 4 consecutive columns per lane.
  constexpr int LDW = TN + 4;                 // padded row length in floats
  constexpr int LPR = TN / 4;                 // lanes per row
  constexpr int RPI = 64 / LPR;               // rows per wave instruction
  constexpr int kSteps = 32 / RPI;
  static_assert((size_t)NT / 64 * 32 * LDW * 4 <= 2 * (size_t)kStage, "epilogue staging must fit in LDS");
  float* stage = reinterpret_cast<float*>(lds) + (size_t)wave * 32 * LDW;
  const int erow = lane / LPR, ecol = (lane % LPR) * 4;
  const int n = n0 + wn * TN + ecol;
  const bool n_ok = n < N;
  f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
  if (ep.bias && n_ok) {
    const bf16x4 b = *reinterpret_cast<const bf16x4*>(ep.bias + n);
#pragma unroll
    for (int e = 0; e < 4; ++e) bias4[e] = (float)b[e];
  }
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
    wave_lds_sync();  // the previous pass's reads are done before its region is rewritten
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stage[(8 * (r >> 2) + 4 * half + (r & 3)) * LDW + j * 32 + l32] = acc[i][j][r];
    wave_lds_sync();
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      const int m = mbase + s * RPI + erow;
      if (!(n_ok && m < M)) continue;
      f32x4 v = *reinterpret_cast<const f32x4*>(stage + (s * RPI + erow) * LDW + ecol);
      const size_t idx = (size_t)m * ep.ldc + n;
      v += bias4;
      if (ep.residual) {
        const bf16x4 rv = *reinterpret_cast<const bf16x4*>(ep.residual + idx);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += (float)rv[e];
      }
      if (ep.out_mode == OUT_STORE) {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
        *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16*>(ep.C) + idx) = o;
      } else if (ep.out_mode == OUT_STORE_F32) {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.C) + idx) = v;
      } else {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.C) + idx) = prev[s] + v;
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, bool AKS, bool BKS>
hipError_t launch_cfg(const GemmDesc& g, hipStream_t s) {
  constexpr int NT = 64 * WM * WN;
  constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * kRowBytes;
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, AKS, BKS>;
  static bool attr_set = false;  // per instantiation; the attribute is per function, set once
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  Operand A{(const bf16*)g.A, g.lda, g.M};
  Operand B{(const bf16*)g.B, g.ldb, g.N};
  Epilogue ep{g.C, g.ldc, g.out_mode, (const bf16*)g.bias, (const bf16*)g.residual};
  kern<<<tiles, NT, lds_bytes, s>>>(g.M, g.N, g.K, A, B, ep);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_layout(const GemmDesc& g, hipStream_t s) {
  if (!g.a_kstrided && !g.b_kstrided) return launch_cfg<BM, BN, WM, WN, false, false>(g, s);
  if (!g.a_kstrided && g.b_kstrided) return launch_cfg<BM, BN, WM, WN, false, true>(g, s);
  if (g.a_kstrided && g.b_kstrided) return launch_cfg<BM, BN, WM, WN, true, true>(g, s);
  return launch_cfg<BM, BN, WM, WN, true, false>(g, s);
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
  return true;
}

void set_gemm_variant(int v) { g_variant = v; }

hipError_t launch_gemm_bf16(const GemmDesc& g, hipStream_t s) {
  switch (g_variant) {
    case 1: return launch_layout<256, 256, 2, 2>(g, s);
    case 2: return launch_layout<256, 256, 2, 4>(g, s);
    case 3: return launch_layout<128, 128, 2, 2>(g, s);
    default: break;
  }
  // Large tiles when they still give every CU work; smaller ones otherwise.
  const long long big_tiles = (long long)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (big_tiles >= 192) return launch_layout<256, 256, 2, 2>(g, s);
  return launch_layout<128, 128, 2, 2>(g, s);
}

}  // namespace jpp
