// Internal declarations shared by the host-side executor and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "../../include/jpp.h"

namespace jpp {

// Records `msg` as the calling thread's last error and returns `code`.
jpp_status fail(jpp_status code, const std::string& msg);
jpp_status fail_hip(hipError_t e, const char* what);

int validate_tasks(const jpp_layer_config* cfg, int M, const jpp_task* tasks, int n, int* peak,
                   std::string& why);

// ---- kernel launchers (all asynchronous on `s`; return the launch status) -------------

// C[M,N] (op)= sum_k A(m,k) B(n,k) (+bias[n]) (+residual[m,n]).
// *_kstrided = false: element (r,k) at P[r*ld + k]; true: at P[k*ld + r].
enum { OUT_STORE = 0, OUT_STORE_F32 = 1, OUT_ACC_F32 = 2 };
struct GemmDesc {
  int M, N, K;
  const void* A; int lda; bool a_kstrided;
  const void* B; int ldb; bool b_kstrided;
  void* C; int ldc; int out_mode;
  const void* bias;      // storage dtype [N] or null
  const void* residual;  // storage dtype, leading dimension ldc, or null
  // Optional fp32 scratch (bf16 GEMM, store modes): when given and large enough
  // (gemm_bf16_workspace_bytes), the tiles of a mostly empty last round of workgroups are
  // split along k and summed by a second kernel.  Must not be shared by concurrent launches.
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
  // Optional fused activation (bf16 GEMM, out_mode OUT_STORE; `aux` has the shape, type and
  // leading dimension of C).  ACT_FWD_*: C receives h = the product (+ bias), aux receives
  // a = gelu(h) evaluated on the stored (rounded) h.  ACT_BWD_*: the product, rounded to the
  // storage type, is the cotangent da of a; C receives dh = da * gelu'(h) with h read from aux.
  // Either way the values are the bits that the separate activation kernels produce.
  int act = 0;
  void* aux = nullptr;
};
enum { ACT_NONE = 0, ACT_FWD_ERF = 1, ACT_FWD_TANH = 2, ACT_BWD_ERF = 3, ACT_BWD_TANH = 4 };
hipError_t launch_gemm_f32(const GemmDesc& g, hipStream_t s);
hipError_t launch_gemm_bf16(const GemmDesc& g, hipStream_t s);
bool gemm_bf16_shape_ok(const GemmDesc& g, std::string& why);
size_t gemm_bf16_workspace_bytes(int M, int N, int K, int out_mode);  // 0: this shape is never split
void set_gemm_variant(int v);  // 0 = automatic tile selection; 1..7 force a configuration (benchmarking)

struct AttnDesc {
  int mb, seq, Hq, Hkv, hd;
  const void* qkv;   // [mb*seq, (Hq+2Hkv)*hd]
  void* out;         // [mb*seq, Hq*hd]
  float* lse;        // [mb, Hq, seq]
  const void* dout;  // backward only
  void* dqkv;        // backward only
  float* delta;      // backward only, [mb, Hq, seq]
  // backward only, optional: fp32 scratch of attention_bwd_scratch_bytes() for grouped-query
  // attention on the MFMA path (per-query-head partial dK / dV, summed in head order)
  float* dkv_partial = nullptr;
};
size_t attention_bwd_scratch_bytes(int mb, int seq, int Hq, int Hkv, int hd);   // 0: no use for scratch
hipError_t launch_attention_fwd_generic(int dtype, const AttnDesc& a, hipStream_t s);
hipError_t launch_attention_bwd_generic(int dtype, const AttnDesc& a, hipStream_t s);
bool attention_mfma_supported(const AttnDesc& a);
hipError_t launch_attention_fwd_mfma(const AttnDesc& a, hipStream_t s);
hipError_t launch_attention_bwd_mfma(const AttnDesc& a, hipStream_t s);

// Row-wise and element-wise kernels.  dtype selects float or bf16 storage.
constexpr int kNormMaxChunksPerThread = 8;  // 256 threads x 16-byte chunks: d <= 8192 (fp32), 16384 (bf16)
bool norm_shape_ok(int dtype, int d);
hipError_t launch_norm_fwd(int dtype, int norm, int rows, int d, float eps, const void* x,
                           const void* gamma, const void* beta, void* y, float* stats, hipStream_t s);
int colreduce_blocks(int rows);  // number of row groups (= rows of the partial buffer)
hipError_t launch_norm_bwd(int dtype, int norm, int rows, int d, const void* x, const void* gamma,
                           const float* stats, const void* dy, const void* dx_add, void* dx,
                           float* g_gamma, float* g_beta, float* partial, hipStream_t s);
// g[n] += sum_rows dy[r, n]; partial: fp32 [colreduce_blocks(rows), n].
hipError_t launch_bias_grad(int dtype, int rows, int n, const void* dy, int ld, float* g,
                            float* partial, hipStream_t s);
hipError_t launch_act_fwd(int dtype, int act, int rows, int f, const void* h, void* a, hipStream_t s);
hipError_t launch_act_bwd(int dtype, int act, int rows, int f, const void* h, const void* da, void* dh,
                          hipStream_t s);
// cos/sin table fp32 [seq, hd/2, 2], computed in double precision on the device.
hipError_t launch_rope_table(float* table, int seq, int hd, float theta, hipStream_t s);
// Rotates the q and k heads of qkv [mb*seq, (Hq+2Hkv)*hd] in place; inverse = backward.
hipError_t launch_rope(int dtype, int mb, int seq, int Hq, int Hkv, int hd, void* qkv,
                       const float* table, bool inverse, hipStream_t s);
// Mean-token cross-entropy from fp32 logits z [rows, vocab]: writes dz = (softmax - onehot)/rows
// in the storage dtype and *loss = -(1/rows) sum_r log softmax(z_r)[tgt_r] (deterministic).
hipError_t launch_cross_entropy(int dtype, int rows, int vocab, const float* z, const int32_t* targets,
                                void* dz, float* row_loss, float* loss, hipStream_t s);
// Token embedding: x[t] = E[tok[t]] (storage dtype, d a multiple of the 16-byte chunk), and its
// gradient G[id] += sum_{t: tok[t] == id, ascending} dx[t] in fp32 (deterministic, no atomics).
hipError_t launch_embed_fwd(int dtype, int rows, int d, int vocab, const int32_t* tok, const void* E, void* x,
                            hipStream_t s);
hipError_t launch_embed_bwd(int dtype, int rows, int d, int vocab, const int32_t* tok, const void* dx, float* G,
                            hipStream_t s);
// a <- a + b; b <- a + b over n fp32 elements (n a multiple of 4).
hipError_t launch_tied_sum(float* a, float* b, size_t n, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
// Parameter updates over n elements (n a multiple of 4): w in the storage dtype, g fp32.
hipError_t launch_sgd(int dtype, void* w, const float* g, size_t n, float lr, float wd, hipStream_t s);
hipError_t launch_adamw(int dtype, void* w, float* master, float* m, float* v, const float* g, size_t n, float lr,
                        float b1, float b2, float eps, float wd, int step, hipStream_t s);
hipError_t launch_widen(int dtype, const void* w, float* master, size_t n, hipStream_t s);  // master <- (float) w

}  // namespace jpp
