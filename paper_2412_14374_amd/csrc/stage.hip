// The stage executor: one actor of an MPMD pipeline on one GPU.
//
// What the paper fixes (and this file implements):
//  * Section 4.2: the actor receives a list of Task(i, ty, stage) and runs it in order;
//    sends are issued asynchronously right after the producing task, receives are
//    asynchronous and act as a prefetch overlapped with compute.  Here a "send"/"receive" is
//    a device-local copy between the caller's boundary buffers and the stage's own buffers,
//    issued on a side stream and ordered with events.
//  * Section 4.3: buffers are deleted after their last use; a buffer that was sent is
//    released if its send has completed, otherwise it is parked in a pending-deletion queue
//    that every later deletion sweeps.  Here: the send staging buffers.
//  * Section 4.4: all task dispatches of a step are fused into one call; there is no host
//    round trip (no stream/event synchronisation) between tasks.
//  * Section 3.1: gradients start at zero and every backward adds its microbatch's
//    gradients (no 1/M); losses are collected per microbatch.
//  * Section 2.2.1: the activations of a forward are kept until its backward on the same
//    actor (the "stash"); the number alive at once depends on the schedule.
// The layer mathematics is not defined by the paper; see include/jpp.h.
//
// Streams.  Forward tasks are enqueued on the caller's compute stream; backward tasks on an
// internal "backward" stream and their weight-gradient GEMMs on an internal "wgrad" stream.
// Section 2.2.1 only requires that data dependencies are honoured, and a forward of one
// microbatch is independent of the backward of another, as is a layer's weight gradient of
// its input gradient: letting them overlap fills the CUs that a single GEMM leaves idle in
// its last round of tiles.  Every kernel still sees exactly the same inputs, per-parameter
// accumulation order is the task order, so results do not depend on the overlap.  Both
// internal streams are joined back into the compute stream before jpp_stage_run returns.
#include <algorithm>

#include "stage_impl.h"

namespace jpp {

static thread_local std::string g_last_error;
static int g_stream_mode = -1;
static int g_fused_act = 3;   // jpp_set_fused_activation

jpp_status fail(jpp_status code, const std::string& msg) {
  g_last_error = msg;
  return code;
}
jpp_status fail_hip(hipError_t e, const char* what) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
  return JPP_EDEVICE;
}

}  // namespace jpp

using namespace jpp;

namespace jpp {
namespace {

bool config_ok(const jpp_layer_config* c, int M, int max_in_flight, std::string& why) {
  if (!c) { why = "null config"; return false; }
  if (c->dtype != JPP_F32 && c->dtype != JPP_BF16) { why = "dtype must be JPP_F32 or JPP_BF16"; return false; }
  if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1 ||
      c->d_ffn < 1 || c->seq_len < 1 || c->microbatch < 1) { why = "sizes must be positive"; return false; }
  if (c->n_q_heads % c->n_kv_heads != 0) { why = "n_q_heads must be a multiple of n_kv_heads"; return false; }
  if (c->norm != JPP_LAYERNORM && c->norm != JPP_RMSNORM) { why = "bad norm"; return false; }
  if (c->act < JPP_GELU || c->act > JPP_SWIGLU) { why = "bad act"; return false; }
  if (c->n_virtual < 1 || c->n_virtual > JPP_MAX_VIRTUAL) { why = "n_virtual out of range"; return false; }
  for (int a = 0; a < c->n_virtual; ++a)
    for (int b = a + 1; b < c->n_virtual; ++b)
      if (c->stage_ids[a] == c->stage_ids[b]) { why = "duplicate stage id"; return false; }
  if (M < 1 || max_in_flight < 1) { why = "n_microbatches and max_in_flight must be positive"; return false; }
  if (c->loss_head && c->vocab < 1) { why = "loss_head needs vocab"; return false; }
  if (c->embed != 0 && c->embed != 1) { why = "embed must be 0 or 1"; return false; }
  if (c->embed && c->vocab < 1) { why = "embed needs vocab"; return false; }
  if (c->remat != 0 && c->remat != 1) { why = "remat must be 0 or 1"; return false; }
  if (c->wgrad_group < 0 || c->wgrad_group > M) { why = "wgrad_group must be in [0, n_microbatches]"; return false; }
  if (c->wgrad_group > 1) {
    if (c->remat) { why = "wgrad_group > 1 keeps the activations a rematerialising stage drops: not with remat"; return false; }
    if (max_in_flight < c->wgrad_group) { why = "max_in_flight must hold at least one group (wgrad_group stashes)"; return false; }
    if (c->dtype == JPP_F32 && c->loss_head && c->vocab % 4 != 0) { why = "wgrad_group > 1 in fp32 needs vocab to be a multiple of 4"; return false; }
  }
  const int chunk = c->dtype == JPP_BF16 ? 8 : 4;
  if (c->head_dim % chunk != 0 || c->head_dim > 256) { why = "head_dim must be a multiple of the 16-byte chunk and <= 256"; return false; }
  if (c->rope && (c->head_dim / 2) % chunk != 0) { why = "rope needs head_dim/2 to be a multiple of the 16-byte chunk"; return false; }
  if (!norm_shape_ok(c->dtype, c->d_model)) { why = "d_model unsupported by the norm kernels"; return false; }
  if (c->d_ffn % chunk != 0) { why = "d_ffn must be a multiple of the 16-byte chunk"; return false; }
  if (c->dtype == JPP_BF16) {
    const long T = (long)c->seq_len * c->microbatch;
    if (T % 8 != 0 || c->d_model % 8 != 0 || ((c->loss_head || c->embed) && c->vocab % 8 != 0)) {
      why = "bf16 mode needs tokens, d_model and vocab to be multiples of 8";
      return false;
    }
  }
  if (c->rope_theta <= 0.f && c->rope) { why = "rope_theta must be positive"; return false; }
  return true;
}

Dims dims_of(const jpp_layer_config& c) {
  Dims m;
  m.seq = c.seq_len; m.mb = c.microbatch; m.T = c.seq_len * c.microbatch;
  m.d = c.d_model; m.hd = c.head_dim; m.Hq = c.n_q_heads; m.Hkv = c.n_kv_heads;
  m.nq = c.n_q_heads * c.head_dim; m.nkv = c.n_kv_heads * c.head_dim; m.nqkv = m.nq + 2 * m.nkv;
  m.f = c.d_ffn; m.f1 = c.act == JPP_SWIGLU ? 2 * c.d_ffn : c.d_ffn;
  m.vocab = c.vocab; m.L = c.n_layers;
  m.esz = c.dtype == JPP_BF16 ? 2 : 4;
  return m;
}

void build_param_table(jpp_stage& st) {
  const jpp_layer_config& c = st.cfg;
  const Dims& m = st.dm;
  size_t off = 0;
  auto add = [&](const std::string& name, int64_t r, int64_t cdim) -> long {
    // every tensor starts on a 16-byte boundary of the storage type and of fp32
    off = (off + 7) / 8 * 8;
    ParamInfo p{name, {r, cdim}, off};
    st.pinfo.push_back(p);
    const long o = (long)off;
    off += (size_t)r * (cdim ? cdim : 1);
    return o;
  };
  const bool ln = c.norm == JPP_LAYERNORM;
  st.loff.resize(m.L);
  for (int l = 0; l < m.L; ++l) {
    auto& o = st.loff[l];
    const std::string pre = "layer" + std::to_string(l) + ".";
    o.ln1_g = add(pre + "ln1_g", m.d, 0);
    o.ln1_b = ln ? add(pre + "ln1_b", m.d, 0) : -1;
    o.wqkv = add(pre + "wqkv", m.nqkv, m.d);
    o.bqkv = c.use_bias ? add(pre + "bqkv", m.nqkv, 0) : -1;
    o.wo = add(pre + "wo", m.d, m.nq);
    o.bo = c.use_bias ? add(pre + "bo", m.d, 0) : -1;
    o.ln2_g = add(pre + "ln2_g", m.d, 0);
    o.ln2_b = ln ? add(pre + "ln2_b", m.d, 0) : -1;
    o.w1 = add(pre + "w1", m.f1, m.d);
    o.b1 = c.use_bias ? add(pre + "b1", m.f1, 0) : -1;
    o.w2 = add(pre + "w2", m.d, m.f);
    o.b2 = c.use_bias ? add(pre + "b2", m.d, 0) : -1;
  }
  if (c.loss_head) {
    st.lnf_g = add("head.lnf_g", m.d, 0);
    st.lnf_b = ln ? add("head.lnf_b", m.d, 0) : -1;
    st.w_head = add("head.w_head", m.vocab, m.d);
  }
  if (c.embed) st.w_embed = add("embed.w", m.vocab, m.d);
  st.pcount = (off + 7) / 8 * 8;
}

// Lays the arena out; with base == nullptr only the size is computed.
size_t carve(jpp_stage& st, char* base) {
  const jpp_layer_config& c = st.cfg;
  const Dims& m = st.dm;
  const int V = c.n_virtual;
  size_t off = 0;
  auto take = [&](size_t bytes) -> char* {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes);
    return p;
  };
  const size_t T = m.T, e = m.esz;
  st.params.resize(V); st.grads.resize(V);
  for (int v = 0; v < V; ++v) st.params[v] = take(st.pcount * e);
  for (int v = 0; v < V; ++v) st.grads[v] = (float*)take(st.pcount * 4);
  st.rope_table = c.rope ? (float*)take((size_t)m.seq * (m.hd / 2) * 2 * 4) : nullptr;
  st.losses = (float*)take((size_t)V * st.M * 4);

  // stash layout inside a (group) slot
  const size_t G = st.G = std::max(1, c.wgrad_group);
  {
    size_t o = 0;
    // a tensor of the G members: packed (GEMM operands of the weight gradients: the members
    // form one matrix) or each member aligned for itself
    auto packed = [&](size_t bytes) { Fld f{o, bytes}; o += align_up(bytes * G); return f; };
    auto apart = [&](size_t bytes) { Fld f{o, align_up(bytes)}; o += align_up(bytes) * G; return f; };
    LayerStash& ls = st.ls;
    ls.x = apart(T * m.d * e); ls.n1 = packed(T * m.d * e); ls.qkv = apart(T * m.nqkv * e);
    ls.O = packed(T * m.nq * e); ls.x1 = apart(T * m.d * e); ls.n2 = packed(T * m.d * e);
    ls.h = apart(T * m.f1 * e); ls.a = packed(T * m.f * e);
    ls.stats1 = apart(2 * T * 4); ls.stats2 = apart(2 * T * 4);
    ls.lse = apart((size_t)m.mb * m.Hq * m.seq * 4);
    if (G > 1) {
      ls.cdy = packed(T * m.d * e); ls.cdh = packed(T * m.f1 * e); ls.cdx1 = packed(T * m.d * e);
      ls.cdqkv = packed(T * m.nqkv * e);
    }
    ls.bytes = o;
    o = 0;
    if (c.loss_head) {
      st.hs.yL = apart(T * m.d * e); st.hs.nf = packed(T * m.d * e); st.hs.statsf = apart(2 * T * 4);
      st.hs.dz = packed(T * m.vocab * e);
    }
    st.hs.bytes = o;
    st.xbytes = align_up(T * m.d * e);
    st.slot_bytes = (c.remat ? st.xbytes : st.ls.bytes) * m.L + st.hs.bytes;
  }
  // max_in_flight stashes = max_in_flight / G group slots of G members each
  const size_t n_gslots = st.max_in_flight / G;
  st.slots.resize(n_gslots * G);
  for (size_t gs = 0; gs < n_gslots; ++gs) {
    char* b = take(st.slot_bytes);
    for (size_t j = 0; j < G; ++j) { st.slots[gs * G + j].base = b; st.slots[gs * G + j].j = (int)j; }
  }
  st.remat_f = c.remat ? take(st.ls.bytes) : nullptr;
  st.remat_b = c.remat ? take(st.ls.bytes) : nullptr;
  st.tx.resize(kTxBuffers);
  for (auto& t : st.tx) t.p = take(T * m.d * e);
  st.cot.resize(kCotBuffers);
  for (auto& t : st.cot) t.p = take(T * m.d * e);
  st.dbuf[0] = take(T * m.d * e); st.dbuf[1] = take(T * m.d * e);
  st.da = take(T * m.f * e); st.dh = take(T * m.f1 * e); st.dn = take(T * m.d * e); st.dx1 = take(T * m.d * e);
  st.dO = take(T * m.nq * e); st.dqkv = take(T * m.nqkv * e);
  st.delta = (float*)take((size_t)m.mb * m.Hq * m.seq * 4);
  {
    const size_t need = c.dtype == JPP_BF16 ? attention_bwd_scratch_bytes(m.mb, m.seq, m.Hq, m.Hkv, m.hd) : 0;
    st.dkv_partial = need ? (float*)take(need) : nullptr;
  }
  const size_t widest = std::max<size_t>({(size_t)m.d, (size_t)m.f1, (size_t)m.nqkv});
  // column sums run over one microbatch's rows (norm gradients) or a whole group's (bias gradients)
  st.partial = (float*)take(2 * (size_t)colreduce_blocks(m.T * (int)G) * widest * 4);
  st.dx_embed = c.embed ? take(T * m.d * e) : nullptr;
  if (c.loss_head) {
    st.z = (float*)take(T * m.vocab * 4);
    st.row_loss = (float*)take(T * 4);
  }
  // scratch for GEMMs whose last round of tiles is split along k: the largest need over the
  // store-mode GEMM shapes of this stage (forward, and input gradient = same M with N, K swapped)
  st.split_bytes = 0;
  if (c.dtype == JPP_BF16) {
    const int shapes[][2] = {{m.nqkv, m.d}, {m.d, m.nq}, {m.f1, m.d}, {m.d, m.f}, {c.loss_head ? m.vocab : 8, m.d}};
    for (const auto& nk : shapes) {
      st.split_bytes = std::max(st.split_bytes, gemm_bf16_workspace_bytes(m.T, nk[0], nk[1], OUT_STORE));
      st.split_bytes = std::max(st.split_bytes, gemm_bf16_workspace_bytes(m.T, nk[1], nk[0], OUT_STORE));
    }
  }
  st.split_f = st.split_bytes ? take(st.split_bytes) : nullptr;
  st.split_b = st.split_bytes ? take(st.split_bytes) : nullptr;
  // ... and for the weight-gradient GEMMs whose output is smaller than the chip: they contract
  // over the tokens of a whole group and are cut along k
  st.split_w_bytes = 0;
  if (c.dtype == JPP_BF16) {
    const int Kw = m.T * (int)G;
    const int shapes[][2] = {{m.nqkv, m.d}, {m.d, m.nq}, {m.f1, m.d}, {m.d, m.f}, {c.loss_head ? m.vocab : 8, m.d}};
    for (const auto& mn : shapes)
      st.split_w_bytes = std::max(st.split_w_bytes, gemm_bf16_workspace_bytes(mn[0], mn[1], Kw, OUT_ACC_F32));
  }
  st.split_w = st.split_w_bytes ? take(st.split_w_bytes) : nullptr;
  return off;
}

hipError_t ev_create(Event& e) { return hipEventCreateWithFlags(&e.ev, hipEventDisableTiming); }
void ev_destroy(Event& e) { if (e.ev) (void)hipEventDestroy(e.ev); e.ev = nullptr; }

#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t _e = (expr);                             \
    if (_e != hipSuccess) return fail_hip(_e, #expr);   \
  } while (0)

hipError_t gemm(const jpp_stage& st, hipStream_t s, int M, int N, int K, const void* A, int lda, bool aks,
                const void* B, int ldb, bool bks, void* C, int ldc, int mode, const void* bias,
                const void* residual, int act = ACT_NONE, void* aux = nullptr) {
  GemmDesc g{M, N, K, A, lda, aks, B, ldb, bks, C, ldc, mode, bias, residual};
  g.act = act;
  g.aux = aux;
  // one scratch per stream: launches on one stream are serial, the streams are not.  The
  // accumulating (weight-gradient) GEMMs, which one stream at a time launches, have their own.
  if (mode == OUT_ACC_F32) {
    g.workspace = st.split_w;
    g.workspace_bytes = st.split_w ? st.split_w_bytes : 0;
  } else {
    g.workspace = s == st.cs ? st.split_f : (s == st.bs ? st.split_b : nullptr);
    g.workspace_bytes = g.workspace ? st.split_bytes : 0;
  }
  return st.cfg.dtype == JPP_BF16 ? launch_gemm_bf16(g, s) : launch_gemm_f32(g, s);
}

// GeLU (either form) in bf16 storage can be applied by the epilogue of the GEMM that produces
// its argument (forward: h and a = gelu(h) from the FFN-up product) or its cotangent (backward:
// dh = da * gelu'(h) from the FFN-down input gradient, da never stored); which of the two is
// in use is jpp_set_fused_activation's.  SwiGLU pairs columns f apart and fp32 storage has no
// fused epilogue: both keep the element-wise kernels.
bool act_fused(const jpp_stage& st, bool backward) {
  return st.cfg.dtype == JPP_BF16 && st.cfg.act != JPP_SWIGLU && (g_fused_act & (backward ? 2 : 1));
}

hipError_t attention_fwd(const jpp_stage& st, hipStream_t s, const AttnDesc& a) {
  if (st.cfg.dtype == JPP_BF16 && attention_mfma_supported(a)) return launch_attention_fwd_mfma(a, s);
  return launch_attention_fwd_generic(st.cfg.dtype, a, s);
}
hipError_t attention_bwd(const jpp_stage& st, hipStream_t s, const AttnDesc& a) {
  if (st.cfg.dtype == JPP_BF16 && attention_mfma_supported(a)) return launch_attention_bwd_mfma(a, s);
  return launch_attention_bwd_generic(st.cfg.dtype, a, s);
}

#define K_TRY(expr)                       \
  do {                                    \
    hipError_t _e = (expr);               \
    if (_e != hipSuccess) return _e;      \
  } while (0)

const void* pptr(const jpp_stage& st, int v, long off) {
  return off < 0 ? nullptr : (const void*)(st.params[v] + (size_t)off * st.dm.esz);
}
float* gptr(const jpp_stage& st, int v, long off) { return off < 0 ? nullptr : st.grads[v] + off; }

// Forward of layer l of local stage v on stream s: input w.x, every intermediate to its place
// in w, output to y (y == nullptr: the last GEMM is skipped, which is all the backward needs
// when it recomputes a layer).
hipError_t layer_forward(jpp_stage& st, hipStream_t s, int v, int l, const LayerView& w, char* y) {
  char* x = w.x;
  const Dims& m = st.dm;
  const jpp_layer_config& c = st.cfg;
  const int dt = c.dtype;
  const auto& o = st.loff[l];
  K_TRY(launch_norm_fwd(dt, c.norm, m.T, m.d, c.norm_eps, x, pptr(st, v, o.ln1_g), pptr(st, v, o.ln1_b),
                        w.n1, (float*)(w.stats1), s));
  K_TRY(gemm(st, s, m.T, m.nqkv, m.d, w.n1, m.d, false, pptr(st, v, o.wqkv), m.d, false, w.qkv,
             m.nqkv, OUT_STORE, pptr(st, v, o.bqkv), nullptr));
  if (c.rope) K_TRY(launch_rope(dt, m.mb, m.seq, m.Hq, m.Hkv, m.hd, w.qkv, st.rope_table, false, s));
  AttnDesc a{m.mb, m.seq, m.Hq, m.Hkv, m.hd, w.qkv, w.O, (float*)(w.lse),
             nullptr, nullptr, nullptr};
  K_TRY(attention_fwd(st, s, a));
  K_TRY(gemm(st, s, m.T, m.d, m.nq, w.O, m.nq, false, pptr(st, v, o.wo), m.nq, false, w.x1, m.d,
             OUT_STORE, pptr(st, v, o.bo), x));
  K_TRY(launch_norm_fwd(dt, c.norm, m.T, m.d, c.norm_eps, w.x1, pptr(st, v, o.ln2_g),
                        pptr(st, v, o.ln2_b), w.n2, (float*)(w.stats2), s));
  if (act_fused(st, false)) {
    K_TRY(gemm(st, s, m.T, m.f1, m.d, w.n2, m.d, false, pptr(st, v, o.w1), m.d, false, w.h, m.f1,
               OUT_STORE, pptr(st, v, o.b1), nullptr, c.act == JPP_GELU ? ACT_FWD_ERF : ACT_FWD_TANH, w.a));
  } else {
    K_TRY(gemm(st, s, m.T, m.f1, m.d, w.n2, m.d, false, pptr(st, v, o.w1), m.d, false, w.h, m.f1,
               OUT_STORE, pptr(st, v, o.b1), nullptr));
    K_TRY(launch_act_fwd(dt, c.act, m.T, m.f, w.h, w.a, s));
  }
  if (y)
    K_TRY(gemm(st, s, m.T, m.d, m.f, w.a, m.f, false, pptr(st, v, o.w2), m.f, false, y, m.d, OUT_STORE,
               pptr(st, v, o.b2), w.x1));
  return hipSuccess;
}

// Forward of all layers (and the loss head) of local stage v for microbatch i, reading the
// input from the slot and writing the output to `y_out` (ignored for a loss-head stage).
hipError_t enqueue_forward(jpp_stage& st, int v, int i, Slot& slot, char* y_out) {
  const Dims& m = st.dm;
  const jpp_layer_config& c = st.cfg;
  hipStream_t s = st.cs;
  const int dt = c.dtype;
  const HeadView hv = st.head_view(slot, slot.j);
  if (st.is_embed(v))
    K_TRY(launch_embed_fwd(dt, m.T, m.d, m.vocab, (const int32_t*)st.inbox_x[(size_t)v * st.M + i],
                           pptr(st, v, st.w_embed), st.layer_view(slot, 0, false).x, s));
  for (int l = 0; l < m.L; ++l) {
    char* y = (l + 1 < m.L) ? st.layer_view(slot, l + 1, false).x : (st.is_head(v) ? hv.yL : y_out);
    K_TRY(layer_forward(st, s, v, l, st.layer_view(slot, l, false), y));
  }
  if (st.is_head(v)) {
    K_TRY(launch_norm_fwd(dt, c.norm, m.T, m.d, c.norm_eps, hv.yL, pptr(st, v, st.lnf_g),
                          pptr(st, v, st.lnf_b), hv.nf, (float*)hv.statsf, s));
    K_TRY(gemm(st, s, m.T, m.vocab, m.d, hv.nf, m.d, false, pptr(st, v, st.w_head), m.d, false, st.z,
               m.vocab, OUT_STORE_F32, nullptr, nullptr));
    K_TRY(launch_cross_entropy(dt, m.T, m.vocab, st.z, st.targets[(size_t)v * st.M + i], hv.dz,
                               st.row_loss, st.losses + (size_t)v * st.M + i, s));
  }
  return hipSuccess;
}

// Weight-gradient GEMM on the wgrad stream, after everything enqueued so far on the backward
// stream (its operands were produced there).
hipError_t wgrad(jpp_stage& st, int M, int N, int K, const void* dy, int ldy, const void* x, int ldx, float* G) {
  K_TRY(hipEventRecord(st.b2w.ev, st.bs));
  K_TRY(hipStreamWaitEvent(st.ws, st.b2w.ev, 0));
  return gemm(st, st.ws, M, N, K, dy, ldy, true, x, ldx, true, G, N, OUT_ACC_F32, nullptr, nullptr);
}

// Backward of local stage v for the microbatch in `slot`: reads the output cotangent from
// `dy_in` (ignored for a loss-head stage; with grouping it already lies in the stash, at the
// top layer's cdy), adds this microbatch's parameter gradients to the fp32 buffers and writes
// the input cotangent to `dx_out`.  The input-gradient chain runs on the backward stream, the
// weight-gradient GEMMs on the wgrad stream.  `wg_members`: how many members' worth of rows
// the weight-gradient GEMMs (and the bias gradients, column sums of the same cotangents, on
// the backward stream) cover, starting at the group's first member; 0 = none now (a later
// member of the group runs them).  Without grouping it is always 1.
hipError_t enqueue_backward(jpp_stage& st, int v, int i, Slot& slot, const char* dy_in, char* dx_out,
                            int wg_members) {
  const Dims& m = st.dm;
  const jpp_layer_config& c = st.cfg;
  hipStream_t s = st.bs;
  const int dt = c.dtype;
  const bool grouped = st.G > 1;
  const int K = wg_members * m.T;
  int cur = 0;
  const char* dy = dy_in;
  // Without grouping the cotangents live in workspace buffers that are about to be
  // overwritten: the previous backward's weight gradients, which read them, must be done.
  // With grouping every cotangent a weight gradient reads has its own place in the stash.
  if (!grouped && st.w_task.recorded) K_TRY(hipStreamWaitEvent(s, st.w_task.ev, 0));
  if (st.is_head(v)) {
    const HeadView hv = st.head_view(slot, slot.j), hg = st.head_view(slot, 0);
    if (wg_members) K_TRY(wgrad(st, m.vocab, m.d, K, hg.dz, m.vocab, hg.nf, m.d, gptr(st, v, st.w_head)));
    K_TRY(gemm(st, s, m.T, m.d, m.vocab, hv.dz, m.vocab, false, pptr(st, v, st.w_head), m.d, true, st.dn,
               m.d, OUT_STORE, nullptr, nullptr));
    char* top = grouped ? st.layer_view(slot, m.L - 1, true).cdy : st.dbuf[cur];
    K_TRY(launch_norm_bwd(dt, c.norm, m.T, m.d, hv.yL, pptr(st, v, st.lnf_g), (float*)hv.statsf,
                          st.dn, nullptr, top, gptr(st, v, st.lnf_g), gptr(st, v, st.lnf_b), st.partial, s));
    dy = top;
    cur ^= 1;
  }
  for (int l = m.L - 1; l >= 0; --l) {
    const LayerView w = st.layer_view(slot, l, true);      // this member
    const LayerView g = st.layer_view(slot, l, 0, true);   // the group's packed matrices
    const auto& o = st.loff[l];
    char* dx = (l == 0) ? dx_out : (grouped ? st.layer_view(slot, l - 1, true).cdy : st.dbuf[cur]);
    char* dh = grouped ? w.cdh : st.dh;
    char* dx1 = grouped ? w.cdx1 : st.dx1;
    char* dqkv = grouped ? w.cdqkv : st.dqkv;
    // operands of the weight gradients: the whole group's rows, or this microbatch's
    const char* wdy = grouped ? g.cdy : dy;
    const char* wdh = grouped ? g.cdh : dh;
    const char* wdx1 = grouped ? g.cdx1 : dx1;
    const char* wdqkv = grouped ? g.cdqkv : dqkv;
    if (!grouped && l != m.L - 1) {
      // the layer above's weight gradients read dh, dx1, dqkv (and, with rematerialisation,
      // the recomputed activations), which this layer rewrites
      K_TRY(hipEventRecord(st.w_layer.ev, st.ws));
      K_TRY(hipStreamWaitEvent(s, st.w_layer.ev, 0));
    }
    // Section 2.2.1, rematerialisation: only the layer's input was kept; run its forward again
    if (c.remat) K_TRY(layer_forward(st, s, v, l, w, nullptr));
    // FFN down projection
    if (wg_members) K_TRY(wgrad(st, m.d, m.f, K, wdy, m.d, g.a, m.f, gptr(st, v, o.w2)));
    if (o.b2 >= 0 && wg_members) K_TRY(launch_bias_grad(dt, K, m.d, wdy, m.d, gptr(st, v, o.b2), st.partial, s));
    if (act_fused(st, true)) {
      K_TRY(gemm(st, s, m.T, m.f, m.d, dy, m.d, false, pptr(st, v, o.w2), m.f, true, dh, m.f, OUT_STORE, nullptr,
                 nullptr, c.act == JPP_GELU ? ACT_BWD_ERF : ACT_BWD_TANH, w.h));
    } else {
      K_TRY(gemm(st, s, m.T, m.f, m.d, dy, m.d, false, pptr(st, v, o.w2), m.f, true, st.da, m.f, OUT_STORE, nullptr,
                 nullptr));
      K_TRY(launch_act_bwd(dt, c.act, m.T, m.f, w.h, st.da, dh, s));
    }
    // FFN up projection
    if (wg_members) K_TRY(wgrad(st, m.f1, m.d, K, wdh, m.f1, g.n2, m.d, gptr(st, v, o.w1)));
    if (o.b1 >= 0 && wg_members) K_TRY(launch_bias_grad(dt, K, m.f1, wdh, m.f1, gptr(st, v, o.b1), st.partial, s));
    K_TRY(gemm(st, s, m.T, m.d, m.f1, dh, m.f1, false, pptr(st, v, o.w1), m.d, true, st.dn, m.d, OUT_STORE,
               nullptr, nullptr));
    K_TRY(launch_norm_bwd(dt, c.norm, m.T, m.d, w.x1, pptr(st, v, o.ln2_g), (float*)w.stats2,
                          st.dn, dy, dx1, gptr(st, v, o.ln2_g), gptr(st, v, o.ln2_b), st.partial, s));
    // attention output projection
    if (wg_members) K_TRY(wgrad(st, m.d, m.nq, K, wdx1, m.d, g.O, m.nq, gptr(st, v, o.wo)));
    if (o.bo >= 0 && wg_members) K_TRY(launch_bias_grad(dt, K, m.d, wdx1, m.d, gptr(st, v, o.bo), st.partial, s));
    K_TRY(gemm(st, s, m.T, m.nq, m.d, dx1, m.d, false, pptr(st, v, o.wo), m.nq, true, st.dO, m.nq, OUT_STORE,
               nullptr, nullptr));
    AttnDesc a{m.mb, m.seq, m.Hq, m.Hkv, m.hd, w.qkv, w.O, (float*)w.lse, st.dO, dqkv, st.delta};
    a.dkv_partial = st.dkv_partial;
    K_TRY(attention_bwd(st, s, a));
    if (c.rope) K_TRY(launch_rope(dt, m.mb, m.seq, m.Hq, m.Hkv, m.hd, dqkv, st.rope_table, true, s));
    // QKV projection
    if (wg_members) K_TRY(wgrad(st, m.nqkv, m.d, K, wdqkv, m.nqkv, g.n1, m.d, gptr(st, v, o.wqkv)));
    if (o.bqkv >= 0 && wg_members)
      K_TRY(launch_bias_grad(dt, K, m.nqkv, wdqkv, m.nqkv, gptr(st, v, o.bqkv), st.partial, s));
    K_TRY(gemm(st, s, m.T, m.d, m.nqkv, dqkv, m.nqkv, false, pptr(st, v, o.wqkv), m.d, true, st.dn, m.d,
               OUT_STORE, nullptr, nullptr));
    K_TRY(launch_norm_bwd(dt, c.norm, m.T, m.d, w.x, pptr(st, v, o.ln1_g), (float*)w.stats1,
                          st.dn, dx1, dx, gptr(st, v, o.ln1_g), gptr(st, v, o.ln1_b), st.partial, s));
    dy = dx;
    cur ^= 1;
  }
  // an embedding stage: the cotangent of x goes into the rows of the table's gradient
  if (st.is_embed(v))
    K_TRY(launch_embed_bwd(dt, m.T, m.d, m.vocab, (const int32_t*)st.inbox_x[(size_t)v * st.M + i], dx_out,
                           gptr(st, v, st.w_embed), s));
  // The wgrad stream now also follows the whole backward chain: an event recorded on it marks
  // "nothing of this task reads the stash, the cotangent or the workspace any more".
  K_TRY(hipEventRecord(st.b2w.ev, st.bs));
  K_TRY(hipStreamWaitEvent(st.ws, st.b2w.ev, 0));
  K_TRY(hipEventRecord(st.w_task.ev, st.ws));
  st.w_task.recorded = true;
  return hipSuccess;
}

// Section 4.3: sweep the pending-deletion queue; buffers whose send has completed go back to
// the free list.  hipEventQuery does not block.
void sweep_pending(jpp_stage& st) {
  for (size_t k = 0; k < st.tx_pending.size();) {
    const int b = st.tx_pending[k];
    if (hipEventQuery(st.tx[b].sent.ev) == hipSuccess) {
      st.tx_free.push_back(b);
      st.tx_pending.erase(st.tx_pending.begin() + k);
    } else {
      ++k;
    }
  }
  (void)hipGetLastError();  // hipErrorNotReady from the query is not an error
}

// A staging buffer for the next send.  If none is free the oldest pending one is reused and
// the producing stream is made to wait (on the device) for its send.
hipError_t acquire_tx(jpp_stage& st, hipStream_t producer, int& out) {
  sweep_pending(st);
  if (!st.tx_free.empty()) {
    out = st.tx_free.back();
    st.tx_free.pop_back();
    return hipSuccess;
  }
  out = st.tx_pending.front();
  st.tx_pending.pop_front();
  return hipStreamWaitEvent(producer, st.tx[out].sent.ev, 0);
}

// Send: copy on the side stream once the producing stream has written the buffer, then the
// "deletion" of the staging buffer (Section 4.3).
hipError_t send_and_delete(jpp_stage& st, hipStream_t producer, int b, void* outbox, size_t bytes,
                           hipEvent_t signal) {
  TxBuf& t = st.tx[b];
  K_TRY(hipEventRecord(t.produced.ev, producer));
  K_TRY(hipStreamWaitEvent(st.ss, t.produced.ev, 0));
  K_TRY(hipMemcpyAsync(outbox, t.p, bytes, hipMemcpyDeviceToDevice, st.ss));
  K_TRY(hipEventRecord(t.sent.ev, st.ss));
  if (signal) K_TRY(hipEventRecord(signal, st.ss));  // the receiving actor waits for this one
  t.sent.recorded = true;
  sweep_pending(st);
  if (hipEventQuery(t.sent.ev) == hipSuccess) {
    st.tx_free.push_back(b);
  } else {
    (void)hipGetLastError();
    st.tx_pending.push_back(b);
    st.pending_peak = std::max(st.pending_peak, (int)st.tx_pending.size());
  }
  return hipSuccess;
}

// Receive of a forward input into a stash slot (side stream).
hipError_t issue_recv_x(jpp_stage& st, Slot& slot, const void* src, size_t bytes, hipEvent_t produced) {
  if (produced) K_TRY(hipStreamWaitEvent(st.ss, produced, 0));  // the sending actor's copy
  if (slot.freed.recorded) K_TRY(hipStreamWaitEvent(st.ss, slot.freed.ev, 0));
  // src == nullptr: an embedding stage, whose forward reads the token ids where they are;
  // the event still orders the forward after the slot's release
  if (src) K_TRY(hipMemcpyAsync(st.layer_view(slot, 0, false).x, src, bytes, hipMemcpyDeviceToDevice, st.ss));
  K_TRY(hipEventRecord(slot.rx.ev, st.ss));
  return hipSuccess;
}

hipError_t issue_recv_cot(jpp_stage& st, CotBuf& cb, const void* src, size_t bytes, hipEvent_t produced) {
  if (produced) K_TRY(hipStreamWaitEvent(st.ss, produced, 0));
  if (cb.freed.recorded) K_TRY(hipStreamWaitEvent(st.ss, cb.freed.ev, 0));
  K_TRY(hipMemcpyAsync(cb.p, src, bytes, hipMemcpyDeviceToDevice, st.ss));
  K_TRY(hipEventRecord(cb.rx.ev, st.ss));
  return hipSuccess;
}

}  // namespace
}  // namespace jpp

extern "C" {

const char* jpp_last_error(void) { return jpp::g_last_error.c_str(); }

size_t jpp_stage_arena_bytes(const jpp_layer_config* cfg, int n_microbatches, int max_in_flight) {
  std::string why;
  if (!config_ok(cfg, n_microbatches, max_in_flight, why)) { fail(JPP_EINVAL, why); return 0; }
  jpp_stage tmp;
  tmp.cfg = *cfg; tmp.M = n_microbatches; tmp.max_in_flight = max_in_flight;
  tmp.dm = dims_of(*cfg);
  build_param_table(tmp);
  return carve(tmp, nullptr);
}

jpp_status jpp_stage_create(const jpp_layer_config* cfg, int n_microbatches, int max_in_flight, void* arena_dev,
                            size_t arena_bytes, jpp_stage** out) {
  if (!out) return fail(JPP_EINVAL, "null output pointer");
  *out = nullptr;
  std::string why;
  if (!config_ok(cfg, n_microbatches, max_in_flight, why)) return fail(JPP_EINVAL, why);
  if (!arena_dev || ((uintptr_t)arena_dev % kAlign) != 0) return fail(JPP_EINVAL, "arena must be 256-byte aligned");
  jpp_stage* st = new jpp_stage;
  st->cfg = *cfg; st->M = n_microbatches; st->max_in_flight = max_in_flight;
  st->dm = dims_of(*cfg);
  build_param_table(*st);
  const size_t need = carve(*st, (char*)arena_dev);
  if (need > arena_bytes) { delete st; return fail(JPP_EINVAL, "arena too small"); }
  st->arena = (char*)arena_dev; st->arena_bytes = arena_bytes;
  st->params_set.assign(cfg->n_virtual, false);
  // the GEMM shapes this stage will launch must be supported
  if (cfg->dtype == JPP_BF16) {
    const Dims& m = st->dm;
    const int dimsv[] = {m.T, m.d, m.nq, m.nqkv, m.f, m.f1};
    for (int v : dimsv)
      if (v % 8 != 0) { delete st; return fail(JPP_EINVAL, "bf16 mode needs every GEMM dimension to be a multiple of 8"); }
  }
  hipError_t e = hipSuccess;
  auto mk = [&](Event& ev) { if (e == hipSuccess) e = ev_create(ev); };
  for (auto& s : st->slots) { mk(s.freed); mk(s.rx); mk(s.fwd_done); }
  for (auto& t : st->tx) { mk(t.produced); mk(t.sent); }
  for (auto& t : st->cot) { mk(t.freed); mk(t.rx); }
  mk(st->end_compute); mk(st->end_side); mk(st->run_start); mk(st->b2w); mk(st->w_layer); mk(st->w_task);
  mk(st->b_end); mk(st->w_end);
  // the two library-owned streams are created by the first run that uses them (stream modes
  // 0 and 1): a stage that computes on the caller's stream alone takes no hardware queue
  if (e == hipSuccess && cfg->rope) {
    e = launch_rope_table(st->rope_table, cfg->seq_len, cfg->head_dim, cfg->rope_theta, nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  }
  if (e != hipSuccess) { jpp_stage_destroy(st); return fail_hip(e, "stage setup"); }
  *out = st;
  return JPP_OK;
}

void jpp_stage_destroy(jpp_stage* st) {
  if (!st) return;
  if (st->cs) (void)hipStreamSynchronize(st->cs);
  if (st->ss) (void)hipStreamSynchronize(st->ss);
  if (st->bs_own) { (void)hipStreamSynchronize(st->bs_own); (void)hipStreamDestroy(st->bs_own); }
  if (st->ws_own) { (void)hipStreamSynchronize(st->ws_own); (void)hipStreamDestroy(st->ws_own); }
  for (auto& s : st->slots) { ev_destroy(s.freed); ev_destroy(s.rx); ev_destroy(s.fwd_done); }
  for (auto& t : st->tx) { ev_destroy(t.produced); ev_destroy(t.sent); }
  for (auto& t : st->cot) { ev_destroy(t.freed); ev_destroy(t.rx); }
  ev_destroy(st->end_compute); ev_destroy(st->end_side); ev_destroy(st->run_start); ev_destroy(st->b2w);
  ev_destroy(st->w_layer); ev_destroy(st->w_task); ev_destroy(st->b_end); ev_destroy(st->w_end);
  delete st;
}

int jpp_stage_param_info(const jpp_stage* st, int idx, const char** name, int64_t shape[2], size_t* elem_offset) {
  if (!st) { fail(JPP_EINVAL, "null stage"); return -JPP_EINVAL; }
  if (idx < 0) return (int)st->pinfo.size();
  if (idx >= (int)st->pinfo.size()) { fail(JPP_EINVAL, "parameter index out of range"); return -JPP_EINVAL; }
  const ParamInfo& p = st->pinfo[idx];
  if (name) *name = p.name.c_str();
  if (shape) { shape[0] = p.shape[0]; shape[1] = p.shape[1]; }
  if (elem_offset) *elem_offset = p.offset;
  return JPP_OK;
}

size_t jpp_stage_param_count(const jpp_stage* st) { return st ? st->pcount : 0; }

jpp_status jpp_stage_set_params(jpp_stage* st, int vstage, const void* src, int src_on_device) {
  if (!st || !src) return fail(JPP_EINVAL, "null argument");
  if (vstage < 0 || vstage >= st->cfg.n_virtual) return fail(JPP_EINVAL, "vstage out of range");
  HIP_TRY(hipMemcpy(st->params[vstage], src, st->pcount * st->dm.esz,
                    src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice));
  HIP_TRY(hipDeviceSynchronize());
  st->params_set[vstage] = true;
  return JPP_OK;
}

jpp_status jpp_stage_bind_boundary(jpp_stage* st, const void* const* inbox_x, const void* const* inbox_cot,
                                   void* const* outbox_y, void* const* outbox_dx,
                                   const int32_t* const* targets) {
  if (!st || !inbox_x || !outbox_dx) return fail(JPP_EINVAL, "inbox_x and outbox_dx are required");
  const int V = st->cfg.n_virtual;
  const bool any_head = st->cfg.loss_head != 0;
  const bool any_body = !any_head || V > 1;   // the head sits on the last virtual stage only
  if (any_body && (!inbox_cot || !outbox_y)) return fail(JPP_EINVAL, "inbox_cot and outbox_y are required");
  if (any_head && !targets) return fail(JPP_EINVAL, "targets are required for a loss_head stage");
  const size_t n = (size_t)V * st->M;
  for (size_t k = 0; k < n; ++k) {
    const bool head = st->is_head((int)(k / st->M));
    const bool embed = st->is_embed((int)(k / st->M));
    if (!inbox_x[k] || (!embed && !outbox_dx[k])) return fail(JPP_EINVAL, "null boundary buffer");
    if (!head && (!inbox_cot[k] || !outbox_y[k])) return fail(JPP_EINVAL, "null boundary buffer");
    if (head && !targets[k]) return fail(JPP_EINVAL, "null targets buffer");
  }
  st->inbox_x.assign(inbox_x, inbox_x + n);
  st->outbox_dx.assign(outbox_dx, outbox_dx + n);
  st->inbox_cot.assign(n, nullptr);
  st->outbox_y.assign(n, nullptr);
  st->targets.assign(n, nullptr);
  for (size_t k = 0; k < n; ++k) {
    if (st->is_head((int)(k / st->M))) {
      st->targets[k] = targets[k];
    } else {
      st->inbox_cot[k] = inbox_cot[k];
      st->outbox_y[k] = outbox_y[k];
    }
  }
  st->bound = true;
  return JPP_OK;
}

jpp_status jpp_stage_zero_grads(jpp_stage* st, void* stream) {
  if (!st) return fail(JPP_EINVAL, "null stage");
  hipStream_t s = (hipStream_t)stream;
  for (int v = 0; v < st->cfg.n_virtual; ++v)
    HIP_TRY(launch_fill_zero(st->grads[v], align_up(st->pcount * 4), s));
  HIP_TRY(launch_fill_zero(st->losses, align_up((size_t)st->cfg.n_virtual * st->M * 4), s));
  return JPP_OK;
}

}  // extern "C"

namespace jpp {

int local_stage(const jpp_layer_config& c, int global) {
  for (int v = 0; v < c.n_virtual; ++v)
    if (c.stage_ids[v] == global) return v;
  return -1;
}

jpp_status run_begin(jpp_stage* st, const jpp_task* tasks, int n_tasks, void* compute_stream, void* side_stream) {
  if (!st) return fail(JPP_EINVAL, "null stage");
  if (st->running) return fail(JPP_ESTATE, "a run is already being enqueued on this stage");
  if (!st->bound) return fail(JPP_ESTATE, "boundary buffers not bound");
  for (bool b : st->params_set)
    if (!b) return fail(JPP_ESTATE, "parameters not set for every virtual stage");
  if (compute_stream == side_stream) return fail(JPP_EINVAL, "compute and side streams must differ");
  std::string why;
  int peak = 0;
  int rc = validate_tasks(&st->cfg, st->M, tasks, n_tasks, &peak, why);
  if (rc != JPP_OK) return fail((jpp_status)rc, why);
  if (peak > st->max_in_flight)
    return fail(JPP_ECAPACITY, "task list keeps " + std::to_string(peak) + " stashes alive, arena holds " +
                                   std::to_string(st->max_in_flight));

  hipStream_t cs = (hipStream_t)compute_stream, ss = (hipStream_t)side_stream;
  // A run queries event completion (pending-deletion queue) and refers to events of earlier
  // runs, neither of which a stream capture allows; a capture-safe variant of this function
  // was tried and ending its capture crashed inside the HIP runtime, so it is refused.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  HIP_TRY(hipStreamIsCapturing(cs, &cap));
  if (cap != hipStreamCaptureStatusNone)
    return fail(JPP_ESTATE, "jpp_stage_run cannot be recorded into a HIP graph");
  // order this run after the previous one on both streams (device-side waits only)
  if (st->end_compute.recorded) {
    HIP_TRY(hipStreamWaitEvent(cs, st->end_side.ev, 0));
    HIP_TRY(hipStreamWaitEvent(ss, st->end_compute.ev, 0));
    HIP_TRY(hipStreamWaitEvent(cs, st->end_compute.ev, 0));
    HIP_TRY(hipStreamWaitEvent(ss, st->end_side.ev, 0));
  }
  st->cs = cs; st->ss = ss;
  // which streams carry the backward (benchmarking knob; the default is three-way overlap)
  const int mode = jpp_stage_stream_mode(st);
  if (mode != 2 && !st->bs_own) HIP_TRY(hipStreamCreateWithFlags(&st->bs_own, hipStreamNonBlocking));
  if (mode == 0 && !st->ws_own) HIP_TRY(hipStreamCreateWithFlags(&st->ws_own, hipStreamNonBlocking));
  st->bs = mode == 2 ? cs : st->bs_own;
  st->ws = mode == 2 ? cs : (mode == 1 ? st->bs_own : st->ws_own);
  // the internal streams start after everything already queued on the compute stream
  // (e.g. jpp_stage_zero_grads)
  HIP_TRY(hipEventRecord(st->run_start.ev, cs));
  HIP_TRY(hipStreamWaitEvent(st->bs, st->run_start.ev, 0));
  HIP_TRY(hipStreamWaitEvent(st->ws, st->run_start.ev, 0));
  HIP_TRY(hipStreamWaitEvent(ss, st->run_start.ev, 0));
  st->w_task.recorded = false;
  st->peak_in_flight = 0; st->pending_peak = 0; st->prefetched = 0;
  st->free_slots.clear();
  for (int k = (int)st->slots.size() / st->G - 1; k >= 0; --k) st->free_slots.push_back(k);
  st->grp_slot.assign((size_t)st->cfg.n_virtual * st->n_groups(), -1);
  st->grp_bwd.assign((size_t)st->cfg.n_virtual * st->n_groups(), 0);
  st->grp_fwd.assign((size_t)st->cfg.n_virtual * st->n_groups(), 0);
  // staging buffers still pending from the previous run are ordered by the waits above
  st->tx_free.clear(); st->tx_pending.clear();
  for (int k = 0; k < kTxBuffers; ++k) st->tx_free.push_back(k);

  const size_t keys = (size_t)st->cfg.n_virtual * st->M;
  st->run_tasks.assign(tasks, tasks + n_tasks);
  st->run_next = 0;
  st->slot_of.assign(keys, -1);   // stash slot of (v, i), assigned at receive time
  st->cot_of.assign(keys, -1);    // cotangent ring entry of (v, i)
  st->cot_next = 0;
  st->live = 0;
  st->running = true;
  return JPP_OK;
}

namespace {

// Issues the receive of task k (Section 4.2: asynchronous, ahead of the consumer).  `ahead`
// = issued before the task itself starts (a prefetch): skipped, without error, when no stash
// slot is free or when the producing actor has not enqueued its send yet.
hipError_t issue_recv(jpp_stage* st, int k, bool ahead) {
  const jpp_task& t = st->run_tasks[k];
  const int v = local_stage(st->cfg, t.stage);
  const size_t key = (size_t)v * st->M + t.i;
  const size_t bbytes = (size_t)st->dm.T * st->dm.d * st->dm.esz;
  if (t.ty == JPP_FWD) {
    if (st->slot_of[key] >= 0) return hipSuccess;  // already prefetched
    if (!st->avail_x.empty() && !st->avail_x[key]) return hipErrorNotReady;
    // the first forward of a weight-gradient group opens a group slot, the others join it
    int& gs = st->grp_slot[(size_t)v * st->n_groups() + t.i / st->G];
    if (gs < 0) {
      if (st->free_slots.empty()) return hipErrorNotReady;  // retried when the task itself starts
      gs = st->free_slots.back();
      st->free_slots.pop_back();
    }
    const int sl = gs * st->G + t.i % st->G;
    st->slot_of[key] = sl;
    if (ahead) ++st->prefetched;
    return issue_recv_x(*st, st->slots[sl], st->is_embed(v) ? nullptr : st->inbox_x[key], bbytes,
                        st->wait_x.empty() ? nullptr : st->wait_x[key]);
  }
  if (st->is_head(v)) return hipSuccess;  // a loss-head backward receives nothing
  if (st->cot_of[key] >= 0) return hipSuccess;
  if (!st->avail_cot.empty() && !st->avail_cot[key]) return hipErrorNotReady;
  const int cb = st->cot_next;
  st->cot_next = (st->cot_next + 1) % kCotBuffers;
  st->cot_of[key] = cb;
  if (ahead) ++st->prefetched;
  return issue_recv_cot(*st, st->cot[cb], st->inbox_cot[key], bbytes,
                        st->wait_cot.empty() ? nullptr : st->wait_cot[key]);
}

}  // namespace

jpp_status run_step(jpp_stage* st) {
  if (!st || !st->running) return fail(JPP_ESTATE, "run_step outside a run");
  const int n_tasks = (int)st->run_tasks.size();
  const int k = st->run_next;
  if (k >= n_tasks) return fail(JPP_ESTATE, "no task left");
  const Dims& m = st->dm;
  const size_t bbytes = (size_t)m.T * m.d * m.esz;
  hipStream_t cs = st->cs;
  const jpp_task& t = st->run_tasks[k];
  const int v = local_stage(st->cfg, t.stage);
  const size_t key = (size_t)v * st->M + t.i;
  const bool head = st->is_head(v);
  // this task's own receive, if it was not prefetched
  hipError_t e = issue_recv(st, k, false);
  if (e != hipSuccess) return fail_hip(e, "receive");
  // prefetch the next task's input while this task computes
  if (k + 1 < n_tasks) {
    // a cotangent ring entry may only be reused once its consumer is enqueued: with two
    // entries the next backward's receive can always go ahead of the current task
    e = issue_recv(st, k + 1, true);
    if (e != hipSuccess && e != hipErrorNotReady) return fail_hip(e, "prefetch");
  }
  if (t.ty == JPP_FWD) {
    Slot& slot = st->slots[st->slot_of[key]];
    // stashes in use: a group holds all its G places from its first forward on
    if (st->grp_fwd[(size_t)v * st->n_groups() + t.i / st->G]++ == 0) st->live += st->G;
    st->peak_in_flight = std::max(st->peak_in_flight, st->live);
    HIP_TRY(hipStreamWaitEvent(cs, slot.rx.ev, 0));
    int txb = -1;
    if (!head) HIP_TRY(acquire_tx(*st, cs, txb));
    e = enqueue_forward(*st, v, t.i, slot, head ? nullptr : st->tx[txb].p);
    if (e != hipSuccess) return fail_hip(e, "forward kernels");
    HIP_TRY(hipEventRecord(slot.fwd_done.ev, cs));
    if (!head)
      HIP_TRY(send_and_delete(*st, cs, txb, st->outbox_y[key], bbytes,
                              st->signal_y.empty() ? nullptr : st->signal_y[key]));
  } else {
    Slot& slot = st->slots[st->slot_of[key]];
    const char* dy = nullptr;
    HIP_TRY(hipStreamWaitEvent(st->bs, slot.fwd_done.ev, 0));  // the forward that filled the stash
    const bool grouped = st->G > 1;
    if (!head) {
      CotBuf& cb = st->cot[st->cot_of[key]];
      HIP_TRY(hipStreamWaitEvent(st->bs, cb.rx.ev, 0));
      dy = cb.p;
      if (grouped) {
        // the group's weight gradients read this cotangent later: move it into the stash and
        // give the ring entry back at once
        char* kept = st->layer_view(slot, m.L - 1, true).cdy;
        HIP_TRY(hipMemcpyAsync(kept, cb.p, bbytes, hipMemcpyDeviceToDevice, st->bs));
        HIP_TRY(hipEventRecord(cb.freed.ev, st->bs));
        cb.freed.recorded = true;
        dy = kept;
      }
    }
    // the task that completes its group runs the group's weight gradients
    const int grp = t.i / st->G;
    const size_t gkey = (size_t)v * st->n_groups() + grp;
    const bool completes = ++st->grp_bwd[gkey] == st->group_size(grp);
    // an embedding stage sends no input cotangent: it stays in a buffer of the backward stream
    const bool embed = st->is_embed(v);
    int txb = -1;
    if (!embed) HIP_TRY(acquire_tx(*st, st->bs, txb));
    e = enqueue_backward(*st, v, t.i, slot, dy, embed ? st->dx_embed : st->tx[txb].p,
                         completes ? st->group_size(grp) : 0);
    if (e != hipSuccess) return fail_hip(e, "backward kernels");
    // enqueue_backward left the wgrad stream behind both the input-gradient chain and the
    // weight gradients of this task: events recorded there cover every reader
    if (!head && !grouped) {
      CotBuf& cb = st->cot[st->cot_of[key]];
      HIP_TRY(hipEventRecord(cb.freed.ev, st->ws));
      cb.freed.recorded = true;
    }
    if (!embed)
      HIP_TRY(send_and_delete(*st, st->bs, txb, st->outbox_dx[key], bbytes,
                              st->signal_dx.empty() ? nullptr : st->signal_dx[key]));
    st->slot_of[key] = -1;
    if (completes) {
      // the group's stash is dead: release its slot; the events protect every member against
      // an early receive on the side stream (and, through the receive, against the next forward)
      const int gs = st->grp_slot[gkey];
      for (int j = 0; j < st->G; ++j) {
        Slot& member = st->slots[(size_t)gs * st->G + j];
        HIP_TRY(hipEventRecord(member.freed.ev, st->ws));
        member.freed.recorded = true;
      }
      st->free_slots.push_back(gs);
      st->grp_slot[gkey] = -1;
      st->live -= st->G;
    }
  }
  st->run_next = k + 1;
  return JPP_OK;
}

jpp_status run_end(jpp_stage* st) {
  if (!st || !st->running) return fail(JPP_ESTATE, "run_end outside a run");
  st->running = false;
  // join the internal streams back into the caller's compute stream
  HIP_TRY(hipEventRecord(st->b_end.ev, st->bs));
  HIP_TRY(hipEventRecord(st->w_end.ev, st->ws));
  HIP_TRY(hipStreamWaitEvent(st->cs, st->b_end.ev, 0));
  HIP_TRY(hipStreamWaitEvent(st->cs, st->w_end.ev, 0));
  // ... and the side stream: when the compute stream reaches this point the run is over
  HIP_TRY(hipEventRecord(st->end_side.ev, st->ss));
  HIP_TRY(hipStreamWaitEvent(st->cs, st->end_side.ev, 0));
  HIP_TRY(hipEventRecord(st->end_compute.ev, st->cs));
  st->end_compute.recorded = true;
  return JPP_OK;
}

}  // namespace jpp

extern "C" {

jpp_status jpp_stage_run(jpp_stage* st, const jpp_task* tasks, int n_tasks, void* compute_stream,
                         void* side_stream) {
  jpp_status rc = run_begin(st, tasks, n_tasks, compute_stream, side_stream);
  if (rc != JPP_OK) return rc;
  for (int k = 0; k < n_tasks; ++k) {
    rc = run_step(st);
    if (rc != JPP_OK) { st->running = false; return rc; }
  }
  return run_end(st);
}

jpp_status jpp_stage_grads(jpp_stage* st, int vstage, const float** grads_dev, size_t* n_elems) {
  if (!st || !grads_dev) return fail(JPP_EINVAL, "null argument");
  if (vstage < 0 || vstage >= st->cfg.n_virtual) return fail(JPP_EINVAL, "vstage out of range");
  if (st->cs) HIP_TRY(hipStreamSynchronize(st->cs));
  if (st->ss) HIP_TRY(hipStreamSynchronize(st->ss));
  *grads_dev = st->grads[vstage];
  if (n_elems) *n_elems = st->pcount;
  return JPP_OK;
}

jpp_status jpp_stage_losses(jpp_stage* st, const float** loss_dev) {
  if (!st || !loss_dev) return fail(JPP_EINVAL, "null argument");
  if (!st->cfg.loss_head) return fail(JPP_ESTATE, "stage has no loss head");
  if (st->cs) HIP_TRY(hipStreamSynchronize(st->cs));
  if (st->ss) HIP_TRY(hipStreamSynchronize(st->ss));
  *loss_dev = st->losses;
  return JPP_OK;
}

jpp_status jpp_stage_params(jpp_stage* st, int vstage, const void** params_dev, size_t* n_elems) {
  if (!st || !params_dev) return fail(JPP_EINVAL, "null argument");
  if (vstage < 0 || vstage >= st->cfg.n_virtual) return fail(JPP_EINVAL, "vstage out of range");
  if (st->cs) HIP_TRY(hipStreamSynchronize(st->cs));
  *params_dev = st->params[vstage];
  if (n_elems) *n_elems = st->pcount;
  return JPP_OK;
}

size_t jpp_stage_optimizer_bytes(const jpp_stage* st, int kind) {
  if (!st || kind != JPP_OPT_ADAMW) return 0;
  return (size_t)st->cfg.n_virtual * 3 * st->pcount * sizeof(float);
}

jpp_status jpp_stage_optimizer_bind(jpp_stage* st, int kind, void* state_dev, size_t state_bytes, void* stream) {
  if (!st) return fail(JPP_EINVAL, "null stage");
  if (kind == JPP_OPT_SGD) { st->opt_state = nullptr; return JPP_OK; }
  if (kind != JPP_OPT_ADAMW) return fail(JPP_EINVAL, "unknown optimizer kind");
  for (bool b : st->params_set)
    if (!b) return fail(JPP_ESTATE, "set the parameters first: the master weights are copied from them");
  if (!state_dev || ((uintptr_t)state_dev % 16) != 0) return fail(JPP_EINVAL, "state must be 16-byte aligned");
  if (state_bytes < jpp_stage_optimizer_bytes(st, kind)) return fail(JPP_EINVAL, "optimizer state too small");
  hipStream_t s = (hipStream_t)stream;
  float* base = (float*)state_dev;
  for (int v = 0; v < st->cfg.n_virtual; ++v) {
    float* master = base + (size_t)v * 3 * st->pcount;
    HIP_TRY(launch_widen(st->cfg.dtype, st->params[v], master, st->pcount, s));
    HIP_TRY(launch_fill_zero(master + st->pcount, 2 * st->pcount * sizeof(float), s));
  }
  st->opt_state = base;
  return JPP_OK;
}

jpp_status jpp_stage_apply_gradients(jpp_stage* st, const jpp_optimizer_step* o, void* stream) {
  if (!st || !o) return fail(JPP_EINVAL, "null argument");
  if (st->running) return fail(JPP_ESTATE, "a run is being enqueued on this stage");
  hipStream_t s = (hipStream_t)stream;
  if (o->kind == JPP_OPT_SGD) {
    for (int v = 0; v < st->cfg.n_virtual; ++v)
      HIP_TRY(launch_sgd(st->cfg.dtype, st->params[v], st->grads[v], st->pcount, o->lr, o->weight_decay, s));
    return JPP_OK;
  }
  if (o->kind != JPP_OPT_ADAMW) return fail(JPP_EINVAL, "unknown optimizer kind");
  if (!st->opt_state) return fail(JPP_ESTATE, "AdamW needs jpp_stage_optimizer_bind first");
  if (o->step < 1) return fail(JPP_EINVAL, "step counts from 1");
  if (!(o->beta1 >= 0.f && o->beta1 < 1.f && o->beta2 >= 0.f && o->beta2 < 1.f))
    return fail(JPP_EINVAL, "beta1 and beta2 must be in [0, 1)");
  for (int v = 0; v < st->cfg.n_virtual; ++v) {
    float* master = st->opt_state + (size_t)v * 3 * st->pcount;
    HIP_TRY(launch_adamw(st->cfg.dtype, st->params[v], master, master + st->pcount, master + 2 * st->pcount,
                         st->grads[v], st->pcount, o->lr, o->beta1, o->beta2, o->eps, o->weight_decay, o->step, s));
  }
  return JPP_OK;
}

void jpp_set_fused_activation(int mask) { jpp::g_fused_act = mask < 0 ? 3 : (mask & 3); }
void jpp_set_stream_mode(int mode) { jpp::g_stream_mode = mode < 0 || mode > 2 ? -1 : mode; }

int jpp_stage_stream_mode(const jpp_stage* st) {
  if (jpp::g_stream_mode >= 0 || !st) return std::max(0, jpp::g_stream_mode);
  const jpp::Dims& m = st->dm;
  return 2.0 * m.T * m.d * m.nq >= 5e10 ? 2 : 0;
}

int jpp_stage_peak_in_flight(const jpp_stage* st) { return st ? st->peak_in_flight : -1; }
int jpp_stage_pending_peak(const jpp_stage* st) { return st ? st->pending_peak : -1; }
int jpp_stage_prefetched(const jpp_stage* st) { return st ? st->prefetched : -1; }

}  // extern "C"
