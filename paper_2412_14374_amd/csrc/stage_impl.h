// State of one stage executor (one actor), shared by the executor and the multi-actor
// pipeline driver.  Not part of the C interface.
#pragma once

#include <algorithm>
#include <deque>
#include <string>
#include <vector>

#include "internal.h"

namespace jpp {

constexpr size_t kAlign = 256;
constexpr int kTxBuffers = 3;   // send staging ring
constexpr int kCotBuffers = 2;  // cotangent receive ring

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct ParamInfo { std::string name; int64_t shape[2]; size_t offset; };

struct Dims {
  int T, d, nq, nkv, nqkv, f, f1, hd, Hq, Hkv, seq, mb, vocab, L;
  size_t esz;
};

// One tensor of the stash: a slot holds it for the g microbatches of a weight-gradient group
// (g = 1 without grouping), member j at off + j * stride bytes.  The operands of the
// weight-gradient GEMMs are packed (stride = the tensor's own size), so that a group's
// members form one matrix with g * T rows.
struct Fld { size_t off = 0, stride = 0; };
// One layer's stash.  cdy, cdh, cdx1, cdqkv exist with grouping only: the cotangents that
// the weight gradients of w2, w1, wo, wqkv contract with, kept until the group is complete.
struct LayerStash {
  Fld x, n1, qkv, O, x1, n2, h, a, stats1, stats2, lse, cdy, cdh, cdx1, cdqkv;
  size_t bytes = 0;
};
struct HeadStash { Fld yL, nf, statsf, dz; size_t bytes = 0; };
// The same, as addresses for one member of one slot.
struct LayerView { char *x, *n1, *qkv, *O, *x1, *n2, *h, *a, *stats1, *stats2, *lse, *cdy, *cdh, *cdx1, *cdqkv; };
struct HeadView { char *yL, *nf, *statsf, *dz; };

struct Event {
  hipEvent_t ev = nullptr;
  bool recorded = false;
};

struct Slot {
  char* base = nullptr;  // of the group slot this member belongs to
  int j = 0;             // member index in the group
  Event freed;  // recorded on the wgrad stream when the last reader of the (group) slot is done
  Event rx;     // recorded on the side stream when the received input is in place
  Event fwd_done;  // recorded on the compute stream when the forward that filled the slot is enqueued
};

struct TxBuf {
  char* p = nullptr;
  Event produced;  // compute stream: contents written
  Event sent;      // side stream: copied to the outbox
};

struct CotBuf {
  char* p = nullptr;
  Event freed;  // compute stream: consumer done
  Event rx;     // side stream: cotangent in place
};

}  // namespace jpp

struct jpp_stage {
  typedef jpp::Dims Dims; typedef jpp::ParamInfo ParamInfo; typedef jpp::LayerStash LayerStash;
  typedef jpp::HeadStash HeadStash; typedef jpp::Event Event; typedef jpp::Slot Slot;
  typedef jpp::TxBuf TxBuf; typedef jpp::CotBuf CotBuf; typedef jpp::Fld Fld;
  typedef jpp::LayerView LayerView; typedef jpp::HeadView HeadView;
  jpp_layer_config cfg;
  int M = 0, max_in_flight = 0;
  Dims dm{};
  std::vector<ParamInfo> pinfo;
  size_t pcount = 0;
  // per-layer parameter offsets (elements) by role; -1 if absent
  struct LayerOff { long ln1_g, ln1_b, wqkv, bqkv, wo, bo, ln2_g, ln2_b, w1, b1, w2, b2; };
  std::vector<LayerOff> loff;
  long lnf_g = -1, lnf_b = -1, w_head = -1, w_embed = -1;

  char* arena = nullptr;
  size_t arena_bytes = 0;
  std::vector<char*> params;   // per vstage
  std::vector<float*> grads;   // per vstage
  float* rope_table = nullptr;
  float* losses = nullptr;     // [V*M]
  LayerStash ls{};
  HeadStash hs{};
  size_t slot_bytes = 0;
  // Rematerialisation: a slot then holds only the layers' inputs (xbytes each, then the head
  // stash); everything else of a layer lives in one of two workspaces laid out like a layer
  // stash, remat_f for the forward stream and remat_b for the backward's recomputation.
  size_t xbytes = 0;
  char *remat_f = nullptr, *remat_b = nullptr;
  int G = 1;   // weight-gradient group size (cfg.wgrad_group, at least 1)
  int group_size(int grp) const { return std::min(G, M - grp * G); }
  int n_groups() const { return (M + G - 1) / G; }
  // Addresses of layer l's stash for member j of the slot's group (j = 0: the start of the
  // group's packed matrices).  `backward` picks the rematerialisation workspace.
  LayerView layer_view(const Slot& slot, int l, int j, bool backward) const {
    char* b = cfg.remat ? (backward ? remat_b : remat_f) : slot.base + (size_t)l * ls.bytes;
    auto at = [&](const Fld& f) { return b + f.off + (size_t)j * f.stride; };
    LayerView w{at(ls.x), at(ls.n1), at(ls.qkv), at(ls.O), at(ls.x1), at(ls.n2), at(ls.h), at(ls.a),
                at(ls.stats1), at(ls.stats2), at(ls.lse), at(ls.cdy), at(ls.cdh), at(ls.cdx1), at(ls.cdqkv)};
    if (cfg.remat) w.x = slot.base + (size_t)l * xbytes;
    return w;
  }
  LayerView layer_view(const Slot& slot, int l, bool backward) const { return layer_view(slot, l, slot.j, backward); }
  HeadView head_view(const Slot& slot, int j) const {
    char* b = slot.base + (size_t)cfg.n_layers * (cfg.remat ? xbytes : ls.bytes);
    auto at = [&](const Fld& f) { return b + f.off + (size_t)j * f.stride; };
    return HeadView{at(hs.yL), at(hs.nf), at(hs.statsf), at(hs.dz)};
  }
  std::vector<Slot> slots;   // G members per group slot: slots[gs * G + j]
  std::vector<TxBuf> tx;
  std::vector<CotBuf> cot;
  // workspace
  char *dbuf[2] = {nullptr, nullptr}, *da = nullptr, *dh = nullptr, *dn = nullptr, *dx1 = nullptr, *dO = nullptr,
       *dqkv = nullptr;
  float *delta = nullptr, *partial = nullptr, *z = nullptr, *row_loss = nullptr;
  float* dkv_partial = nullptr;   // scratch of the grouped-query attention backward (null: not needed)
  char* dx_embed = nullptr;   // cotangent of the embedded input (embed stage), consumed by the table's gradient
  // GEMM split scratch, one per stream that launches store-mode GEMMs (forward, backward chain)
  char *split_f = nullptr, *split_b = nullptr;
  size_t split_bytes = 0;
  // ... and for the accumulating weight-gradient GEMMs (one stream at a time launches those)
  char* split_w = nullptr;
  size_t split_w_bytes = 0;

  // boundary
  std::vector<const void*> inbox_x, inbox_cot;
  std::vector<void*> outbox_y, outbox_dx;
  std::vector<const int32_t*> targets;
  bool bound = false;
  std::vector<bool> params_set;

  // run state
  hipStream_t cs = nullptr, ss = nullptr;   // caller's streams of the current / last run
  hipStream_t bs = nullptr, ws = nullptr;   // backward chain, weight-gradient GEMMs: chosen per run, see jpp_set_stream_mode
  hipStream_t bs_own = nullptr, ws_own = nullptr;   // the two library-owned streams
  Event end_compute, end_side, run_start, b2w, w_layer, w_task, b_end, w_end;
  int peak_in_flight = 0, pending_peak = 0, prefetched = 0;
  std::vector<int> free_slots;      // free group slots
  std::vector<int> grp_slot, grp_fwd, grp_bwd;  // per (v, group): its group slot (-1: none), forwards / backwards enqueued
  std::vector<int> tx_free;
  std::deque<int> tx_pending;
  // the task list being enqueued (between run_begin and run_end)
  std::vector<jpp_task> run_tasks;
  int run_next = 0;                 // index of the next task to enqueue
  std::vector<int> slot_of, cot_of; // stash slot / cotangent ring entry of (v, i); -1 = none
  int cot_next = 0, live = 0;
  bool running = false;

  // Hand-offs to other actors on the same device, set by a pipeline (empty otherwise); all
  // indexed v * M + i.  A receive waits (on the side stream) for wait_*[key] before it copies;
  // a send records signal_*[key] after its copy.  avail_*[key] says that the producer of the
  // input has been enqueued, i.e. that wait_*[key] has been recorded: only then may the
  // receive be issued (a wait on an event that is not yet recorded does not wait).
  std::vector<hipEvent_t> wait_x, wait_cot, signal_y, signal_dx;
  std::vector<char> avail_x, avail_cot;

  // AdamW state, caller-owned (jpp_stage_optimizer_bind): per virtual stage [master | m | v],
  // pcount floats each
  float* opt_state = nullptr;

  // The loss head, if configured, belongs to the actor's last virtual stage.
  bool is_head(int v) const { return cfg.loss_head != 0 && v == cfg.n_virtual - 1; }
  // The token embedding, if configured, belongs to the actor's first virtual stage.
  bool is_embed(int v) const { return cfg.embed != 0 && v == 0; }
};

namespace jpp {

int local_stage(const jpp_layer_config& c, int global);
// jpp_stage_run in three parts, so that a pipeline can interleave the task lists of several
// actors: run_begin validates and prepares (no kernel is launched on failure), run_step
// enqueues the next task (its receive, kernels and send) and run_end joins the streams.
jpp_status run_begin(jpp_stage* st, const jpp_task* tasks, int n_tasks, void* compute_stream, void* side_stream);
jpp_status run_step(jpp_stage* st);
jpp_status run_end(jpp_stage* st);

}  // namespace jpp

