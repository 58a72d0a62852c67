// Host-side schedule generators and task-list validator (no GPU code).
//
// A per-actor schedule is an array of Task(i, ty, stage) records (paper, Section 4.2).
// Section 2.2.1 describes GPipe (all forwards, then all backwards), 1F1B (backwards are
// scheduled eagerly so live activations are bounded by the number of stages) and
// interleaved 1F1B (several stages per actor, "circular repeat").  The paper's figures
// are not reproduced in its source, so the block order of the latter two follows the
// published schedules it cites; the interleaved order reproduces the two-actor example
// printed in Section 4.2.
#include "internal.h"

#include <algorithm>
#include <vector>

namespace jpp {

static bool sched_args_ok(int kind, int P, int rank, int V, int M) {
  if (P < 1 || rank < 0 || rank >= P || M < 1 || V < 1 || V > JPP_MAX_VIRTUAL) return false;
  if (kind == JPP_GPIPE || kind == JPP_1F1B) return V == 1;
  if (kind == JPP_INTERLEAVED_1F1B) return M % P == 0;
  return false;
}

namespace {

// Interleaved order: the actor's forward work items are numbered 0..M*V-1.  Item k belongs
// to round k / (P*V); within a round the actor pushes P consecutive microbatches through
// its first local stage, then the same P through its second, ... (backward work items walk
// the local stages from last to first).
struct InterleavedCursor {
  int P, V, rank;
  jpp_task at(int k, bool fwd) const {
    const int round = k / (P * V);
    const int pos = k % (P * V);
    int local = pos / P;
    if (!fwd) local = V - 1 - local;
    jpp_task t;
    t.i = round * P + pos % P;
    t.ty = fwd ? JPP_FWD : JPP_BWD;
    t.stage = local * P + rank;
    return t;
  }
};

}  // namespace

static void make_schedule(int kind, int P, int rank, int V, int M, std::vector<jpp_task>& out) {
  out.clear();
  auto push = [&](int i, int ty, int stage) { out.push_back(jpp_task{i, ty, stage}); };
  if (kind == JPP_GPIPE) {
    for (int i = 0; i < M; ++i) push(i, JPP_FWD, rank);
    for (int i = 0; i < M; ++i) push(i, JPP_BWD, rank);
    return;
  }
  if (kind == JPP_1F1B) {
    // Forwards needed to fill the pipeline below this actor, then one forward per backward.
    int ahead = P - 1 - rank;
    if (ahead > M) ahead = M;
    int nf = 0, nb = 0;
    while (nf < ahead) push(nf++, JPP_FWD, rank);
    while (nf < M) {  // steady state: the forward that keeps the pipe full, then the oldest backward
      push(nf++, JPP_FWD, rank);
      push(nb++, JPP_BWD, rank);
    }
    while (nb < M) push(nb++, JPP_BWD, rank);
    return;
  }
  // interleaved 1F1B
  InterleavedCursor cur{P, V, rank};
  const int total = M * V;
  int warm = (P - 1 - rank) * 2 + (V - 1) * P;
  if (warm > total) warm = total;
  for (int k = 0; k < warm; ++k) out.push_back(cur.at(k, true));
  for (int k = warm; k < total; ++k) {
    out.push_back(cur.at(k, true));
    out.push_back(cur.at(k - warm, false));
  }
  for (int k = total - warm; k < total; ++k) out.push_back(cur.at(k, false));
}

int validate_tasks(const jpp_layer_config* cfg, int M, const jpp_task* tasks, int n, int* peak,
                   std::string& why) {
  const int V = cfg->n_virtual;
  if (M < 1 || n < 0 || (n > 0 && !tasks)) { why = "bad task array"; return JPP_ESCHED; }
  // state per (local stage, microbatch): 0 = nothing, 1 = forward done, 2 = backward done
  std::vector<uint8_t> state((size_t)V * M, 0);
  // Stashes in use.  With weight-gradient groups of g microbatches a group's g places are
  // taken from its first forward until its last backward (without: g = 1, a stash lives from
  // its forward to its backward).
  const int g = cfg->wgrad_group > 1 ? cfg->wgrad_group : 1;
  const int ng = (M + g - 1) / g;
  std::vector<int> grp_fwd((size_t)V * ng, 0), grp_bwd((size_t)V * ng, 0);
  int live = 0, hi = 0;
  for (int t = 0; t < n; ++t) {
    const jpp_task& k = tasks[t];
    int local = -1;
    for (int v = 0; v < V; ++v)
      if (cfg->stage_ids[v] == k.stage) local = v;
    if (local < 0) { why = "task " + std::to_string(t) + ": stage not owned by this actor"; return JPP_ESCHED; }
    if (k.i < 0 || k.i >= M) { why = "task " + std::to_string(t) + ": microbatch out of range"; return JPP_ESCHED; }
    uint8_t& s = state[(size_t)local * M + k.i];
    if (k.ty == JPP_FWD) {
      if (s != 0) { why = "task " + std::to_string(t) + ": duplicate forward"; return JPP_ESCHED; }
      s = 1;
      if (grp_fwd[(size_t)local * ng + k.i / g]++ == 0) live += g;
      if (live > hi) hi = live;
    } else if (k.ty == JPP_BWD) {
      if (s == 0) { why = "task " + std::to_string(t) + ": backward before its forward"; return JPP_ESCHED; }
      if (s == 2) { why = "task " + std::to_string(t) + ": duplicate backward"; return JPP_ESCHED; }
      s = 2;
      if (++grp_bwd[(size_t)local * ng + k.i / g] == std::min(g, M - k.i / g * g)) live -= g;
    } else {
      why = "task " + std::to_string(t) + ": unknown task type";
      return JPP_ESCHED;
    }
  }
  for (uint8_t s : state)
    if (s != 2) { why = "task list incomplete: some (microbatch, stage) lacks forward or backward"; return JPP_ESCHED; }
  if (peak) *peak = hi;
  return JPP_OK;
}

}  // namespace jpp

extern "C" {

int jpp_schedule_len(int kind, int P, int rank, int V, int M) {
  if (!jpp::sched_args_ok(kind, P, rank, V, M)) return -1;
  return 2 * M * V;
}

jpp_status jpp_schedule_make(int kind, int P, int rank, int V, int M, jpp_task* out, int cap) {
  if (!jpp::sched_args_ok(kind, P, rank, V, M)) return jpp::fail(JPP_EINVAL, "bad schedule arguments");
  if (!out || cap < 2 * M * V) return jpp::fail(JPP_EINVAL, "output array too small");
  std::vector<jpp_task> v;
  jpp::make_schedule(kind, P, rank, V, M, v);
  if ((int)v.size() != 2 * M * V) return jpp::fail(JPP_EINVAL, "internal: schedule length mismatch");
  for (size_t k = 0; k < v.size(); ++k) out[k] = v[k];
  return JPP_OK;
}

jpp_status jpp_schedule_validate(const jpp_layer_config* cfg, int M, const jpp_task* tasks, int n,
                                 int* peak_in_flight) {
  if (!cfg || cfg->n_virtual < 1 || cfg->n_virtual > JPP_MAX_VIRTUAL)
    return jpp::fail(JPP_EINVAL, "bad config");
  std::string why;
  int rc = jpp::validate_tasks(cfg, M, tasks, n, peak_in_flight, why);
  if (rc != JPP_OK) return jpp::fail((jpp_status)rc, why);
  return JPP_OK;
}

}  // extern "C"
