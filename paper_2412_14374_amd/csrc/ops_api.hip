// C entry points for single operations (see include/jpp.h): argument checks, then the same
// launchers the stage executor uses.
#include <mutex>

#include "internal.h"

using namespace jpp;

// Scratch of jpp_op_attention_bwd_static, the entry point for callers that cannot allocate:
// JPP_STATIC_SCRATCH_BYTES of device memory that exist in every GPU the library is loaded on
// from load time to the end of the process.  In host code this name is only a handle for
// hipGetSymbolAddress; the address kernels are given is the one looked up per device below.
static __device__ __align__(256) float scratch[JPP_STATIC_SCRATCH_BYTES / sizeof(float)];

namespace {
bool dtype_ok(int dtype) { return dtype == JPP_F32 || dtype == JPP_BF16; }
int chunk_of(int dtype) { return dtype == JPP_BF16 ? 8 : 4; }

// Device address of `scratch` on the current device, looked up once per device (every GPU
// holds its own copy of the array at its own address).  No allocation.
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

jpp_status static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(JPP_EDEVICE, "device index beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(scratch)");
    if (!p) return fail(JPP_EDEVICE, "hipGetSymbolAddress returned a null address for the static scratch");
    g_scratch_ptr[dev] = (float*)p;
  }
  *out = g_scratch_ptr[dev];
  return JPP_OK;
}
}  // namespace

extern "C" {

void jpp_set_gemm_variant(int variant) { set_gemm_variant(variant); }

jpp_status jpp_op_gemm(int dtype, int M, int N, int K, const void* A, int lda, int a_kstrided, const void* B,
                       int ldb, int b_kstrided, void* C, int ldc, int out_mode, const void* bias,
                       const void* residual, void* stream) {
  return jpp_op_gemm_ws(dtype, M, N, K, A, lda, a_kstrided, B, ldb, b_kstrided, C, ldc, out_mode, bias, residual,
                        nullptr, 0, stream);
}

size_t jpp_op_gemm_workspace_bytes(int dtype, int M, int N, int K, int out_mode) {
  if (dtype != JPP_BF16 || M < 1 || N < 1 || K < 1) return 0;
  return gemm_bf16_workspace_bytes(M, N, K, out_mode);
}

jpp_status jpp_op_gemm_ws(int dtype, int M, int N, int K, const void* A, int lda, int a_kstrided, const void* B,
                          int ldb, int b_kstrided, void* C, int ldc, int out_mode, const void* bias,
                          const void* residual, void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dtype)) return fail(JPP_EINVAL, "bad dtype");
  if (workspace && ((uintptr_t)workspace % 16) != 0) return fail(JPP_EINVAL, "workspace must be 16-byte aligned");
  if (!A || !B || !C) return fail(JPP_EINVAL, "null operand");
  if (M < 1 || N < 1 || K < 1) return fail(JPP_EINVAL, "sizes must be positive");
  if (out_mode < OUT_STORE || out_mode > OUT_ACC_F32) return fail(JPP_EINVAL, "bad out_mode");
  GemmDesc g{M, N, K, A, lda, a_kstrided != 0, B, ldb, b_kstrided != 0, C, ldc, out_mode, bias, residual};
  g.workspace = workspace;
  g.workspace_bytes = workspace ? workspace_bytes : 0;
  hipError_t e;
  if (dtype == JPP_BF16) {
    std::string why;
    if (!gemm_bf16_shape_ok(g, why)) return fail(JPP_EINVAL, why);
    e = launch_gemm_bf16(g, (hipStream_t)stream);
  } else {
    if ((a_kstrided ? lda < M : lda < K) || (b_kstrided ? ldb < N : ldb < K) || ldc < N)
      return fail(JPP_EINVAL, "leading dimension smaller than the row length");
    e = launch_gemm_f32(g, (hipStream_t)stream);
  }
  return e == hipSuccess ? JPP_OK : fail_hip(e, "gemm launch");
}

jpp_status jpp_op_gemm_gelu(int M, int N, int K, const void* A, int lda, int a_kstrided, const void* B, int ldb,
                            int b_kstrided, void* C, int ldc, const void* bias, int act, int backward, void* aux,
                            void* workspace, size_t workspace_bytes, void* stream) {
  if (!A || !B || !C || !aux) return fail(JPP_EINVAL, "null operand");
  if (M < 1 || N < 1 || K < 1) return fail(JPP_EINVAL, "sizes must be positive");
  if (act != JPP_GELU && act != JPP_GELU_TANH) return fail(JPP_EINVAL, "act must be JPP_GELU or JPP_GELU_TANH");
  if (workspace && ((uintptr_t)workspace % 16) != 0) return fail(JPP_EINVAL, "workspace must be 16-byte aligned");
  GemmDesc g{M, N, K, A, lda, a_kstrided != 0, B, ldb, b_kstrided != 0, C, ldc, OUT_STORE, bias, nullptr};
  g.workspace = workspace;
  g.workspace_bytes = workspace ? workspace_bytes : 0;
  g.act = backward ? (act == JPP_GELU ? ACT_BWD_ERF : ACT_BWD_TANH) : (act == JPP_GELU ? ACT_FWD_ERF : ACT_FWD_TANH);
  g.aux = aux;
  std::string why;
  if (!gemm_bf16_shape_ok(g, why)) return fail(JPP_EINVAL, why);
  hipError_t e = launch_gemm_bf16(g, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "gemm launch");
}

static jpp_status attn_check(int dtype, int mb, int seq, int Hq, int Hkv, int hd) {
  if (!dtype_ok(dtype)) return fail(JPP_EINVAL, "bad dtype");
  if (mb < 1 || seq < 1 || Hq < 1 || Hkv < 1 || hd < 1) return fail(JPP_EINVAL, "sizes must be positive");
  if (Hq % Hkv != 0) return fail(JPP_EINVAL, "Hq must be a multiple of Hkv");
  if (hd % chunk_of(dtype) != 0 || hd > 256) return fail(JPP_EINVAL, "unsupported head_dim");
  return JPP_OK;
}

jpp_status jpp_op_attention_fwd(int dtype, int mb, int seq, int Hq, int Hkv, int hd, const void* qkv, void* out,
                                float* lse, void* stream) {
  jpp_status rc = attn_check(dtype, mb, seq, Hq, Hkv, hd);
  if (rc != JPP_OK) return rc;
  if (!qkv || !out || !lse) return fail(JPP_EINVAL, "null operand");
  AttnDesc a{mb, seq, Hq, Hkv, hd, qkv, out, lse, nullptr, nullptr, nullptr};
  hipError_t e = (dtype == JPP_BF16 && attention_mfma_supported(a))
                     ? launch_attention_fwd_mfma(a, (hipStream_t)stream)
                     : launch_attention_fwd_generic(dtype, a, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "attention forward launch");
}

size_t jpp_op_attention_bwd_scratch_bytes(int dtype, int mb, int seq, int Hq, int Hkv, int hd) {
  if (dtype != JPP_BF16 || mb < 1 || seq < 1 || Hq < 1 || Hkv < 1) return 0;
  return attention_bwd_scratch_bytes(mb, seq, Hq, Hkv, hd);
}

jpp_status jpp_op_attention_bwd(int dtype, int mb, int seq, int Hq, int Hkv, int hd, const void* qkv,
                                const void* out, const float* lse, const void* dout, void* dqkv, float* delta,
                                void* stream) {
  return jpp_op_attention_bwd_ws(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, delta, nullptr, 0, stream);
}

jpp_status jpp_op_attention_bwd_ws(int dtype, int mb, int seq, int Hq, int Hkv, int hd, const void* qkv,
                                   const void* out, const float* lse, const void* dout, void* dqkv, float* delta,
                                   void* scratch, size_t scratch_bytes, void* stream) {
  jpp_status rc = attn_check(dtype, mb, seq, Hq, Hkv, hd);
  if (rc != JPP_OK) return rc;
  if (!qkv || !out || !lse || !dout || !dqkv || !delta) return fail(JPP_EINVAL, "null operand");
  if (scratch && ((uintptr_t)scratch % 16) != 0) return fail(JPP_EINVAL, "scratch must be 16-byte aligned");
  AttnDesc a{mb, seq, Hq, Hkv, hd, qkv, const_cast<void*>(out), const_cast<float*>(lse), dout, dqkv, delta};
  const size_t need = jpp_op_attention_bwd_scratch_bytes(dtype, mb, seq, Hq, Hkv, hd);
  if (scratch && need > 0 && scratch_bytes >= need) a.dkv_partial = (float*)scratch;
  hipError_t e = (dtype == JPP_BF16 && attention_mfma_supported(a))
                     ? launch_attention_bwd_mfma(a, (hipStream_t)stream)
                     : launch_attention_bwd_generic(dtype, a, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "attention backward launch");
}

jpp_status jpp_op_attention_bwd_static(int dtype, int mb, int seq, int Hq, int Hkv, int hd, const void* qkv,
                                       const void* out, const float* lse, const void* dout, void* dqkv,
                                       void* stream) {
  jpp_status rc = attn_check(dtype, mb, seq, Hq, Hkv, hd);
  if (rc != JPP_OK) return rc;
  // delta holds one float per (batch, query head, position)
  const unsigned long long need = 4ull * (unsigned long long)mb * (unsigned long long)Hq * (unsigned long long)seq;
  if (need > JPP_STATIC_SCRATCH_BYTES)
    return fail(JPP_EINVAL, "jpp_op_attention_bwd_static: mb * Hq * seq = " +
                                std::to_string((unsigned long long)mb * Hq * seq) + " exceeds the static scratch of " +
                                std::to_string(JPP_STATIC_SCRATCH_BYTES / 4) + " floats; use jpp_op_attention_bwd");
  float* delta = nullptr;
  rc = static_scratch(&delta);
  if (rc != JPP_OK) return rc;
  // every element of delta that the kernels read is written first by the same call: nothing to clear
  return jpp_op_attention_bwd_ws(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, delta, nullptr, 0, stream);
}

jpp_status jpp_op_norm_fwd(int dtype, int norm, int rows, int d, float eps, const void* x, const void* gamma,
                           const void* beta, void* y, float* stats, void* stream) {
  if (!dtype_ok(dtype) || (norm != JPP_LAYERNORM && norm != JPP_RMSNORM)) return fail(JPP_EINVAL, "bad dtype/norm");
  if (rows < 1 || !norm_shape_ok(dtype, d)) return fail(JPP_EINVAL, "unsupported norm shape");
  if (!x || !gamma || !y || !stats) return fail(JPP_EINVAL, "null operand");
  hipError_t e = launch_norm_fwd(dtype, norm, rows, d, eps, x, gamma, beta, y, stats, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "norm forward launch");
}

size_t jpp_op_colreduce_scratch(int rows, int d) {
  if (rows < 1 || d < 1) return 0;
  return 2 * (size_t)colreduce_blocks(rows) * d;
}

jpp_status jpp_op_norm_bwd(int dtype, int norm, int rows, int d, const void* x, const void* gamma,
                           const float* stats, const void* dy, const void* dx_add, void* dx, float* g_gamma,
                           float* g_beta, float* partial, void* stream) {
  if (!dtype_ok(dtype) || (norm != JPP_LAYERNORM && norm != JPP_RMSNORM)) return fail(JPP_EINVAL, "bad dtype/norm");
  if (rows < 1 || !norm_shape_ok(dtype, d)) return fail(JPP_EINVAL, "unsupported norm shape");
  if (!x || !gamma || !stats || !dy || !dx || !g_gamma || !partial) return fail(JPP_EINVAL, "null operand");
  if (dx == dx_add) return fail(JPP_EINVAL, "dx must not alias dx_add");
  hipError_t e = launch_norm_bwd(dtype, norm, rows, d, x, gamma, stats, dy, dx_add, dx, g_gamma, g_beta, partial,
                                 (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "norm backward launch");
}

jpp_status jpp_op_act_fwd(int dtype, int act, int rows, int f, const void* h, void* a, void* stream) {
  if (!dtype_ok(dtype) || act < JPP_GELU || act > JPP_SWIGLU) return fail(JPP_EINVAL, "bad dtype/act");
  if (rows < 1 || f < 1 || f % chunk_of(dtype) != 0) return fail(JPP_EINVAL, "f must be a multiple of the 16-byte chunk");
  if (!h || !a) return fail(JPP_EINVAL, "null operand");
  hipError_t e = launch_act_fwd(dtype, act, rows, f, h, a, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "activation forward launch");
}

jpp_status jpp_op_act_bwd(int dtype, int act, int rows, int f, const void* h, const void* da, void* dh,
                          void* stream) {
  if (!dtype_ok(dtype) || act < JPP_GELU || act > JPP_SWIGLU) return fail(JPP_EINVAL, "bad dtype/act");
  if (rows < 1 || f < 1 || f % chunk_of(dtype) != 0) return fail(JPP_EINVAL, "f must be a multiple of the 16-byte chunk");
  if (!h || !da || !dh) return fail(JPP_EINVAL, "null operand");
  hipError_t e = launch_act_bwd(dtype, act, rows, f, h, da, dh, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "activation backward launch");
}

jpp_status jpp_op_cross_entropy(int dtype, int rows, int vocab, const float* z, const int32_t* targets, void* dz,
                                float* row_loss, float* loss, void* stream) {
  if (!dtype_ok(dtype)) return fail(JPP_EINVAL, "bad dtype");
  if (rows < 1 || vocab < 1) return fail(JPP_EINVAL, "sizes must be positive");
  if (!z || !targets || !dz || !row_loss || !loss) return fail(JPP_EINVAL, "null operand");
  hipError_t e = launch_cross_entropy(dtype, rows, vocab, z, targets, dz, row_loss, loss, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "cross-entropy launch");
}

jpp_status jpp_op_embed_fwd(int dtype, int rows, int d, int vocab, const int32_t* ids, const void* table, void* x,
                            void* stream) {
  if (!dtype_ok(dtype)) return fail(JPP_EINVAL, "bad dtype");
  if (rows < 1 || vocab < 1 || d < 1 || d % chunk_of(dtype) != 0)
    return fail(JPP_EINVAL, "d must be a multiple of the 16-byte chunk");
  if (!ids || !table || !x) return fail(JPP_EINVAL, "null operand");
  hipError_t e = launch_embed_fwd(dtype, rows, d, vocab, ids, table, x, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "embedding forward launch");
}

jpp_status jpp_op_embed_bwd(int dtype, int rows, int d, int vocab, const int32_t* ids, const void* dx, float* g_table,
                            void* stream) {
  if (!dtype_ok(dtype)) return fail(JPP_EINVAL, "bad dtype");
  if (rows < 1 || rows > 393216 || vocab < 1 || d < 1) return fail(JPP_EINVAL, "rows must be in [1, 393216]");
  if (!ids || !dx || !g_table) return fail(JPP_EINVAL, "null operand");
  hipError_t e = launch_embed_bwd(dtype, rows, d, vocab, ids, dx, g_table, (hipStream_t)stream);
  return e == hipSuccess ? JPP_OK : fail_hip(e, "embedding backward launch");
}

}  // extern "C"
