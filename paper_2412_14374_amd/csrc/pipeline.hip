// Several actors of one MPMD pipeline on one GPU.
//
// Section 4.2 of the paper: every actor has its own task list; the runtime walks the tasks in
// a topological order of the task graph and places each send, and the matching receive on
// the consuming actor, right after the task that produces the data; receives are
// asynchronous, so they act as prefetches.  Section 4.4: the actors are coordinated by
// send / receive dependencies only.
//
// Here every actor is a jpp_stage executor with its own streams, stage s lives on actor
// s mod P, and a hand-off is a pair of device-local copies through a boundary buffer owned
// by the pipeline: the producer's side stream copies into it and records an event, the
// consumer's side stream waits for that event and copies out of it.  jpp_pipeline_run merges
// the P lists on the host: round after round, every actor enqueues its next task if the task
// that produces its operand has already been enqueued.  That order is what makes the
// device-side waits sound (a stream can only wait for an event that has been recorded
// before, in host order) and it is also the deadlock check: if no actor can move, the lists
// wait for each other in a cycle and JPP_ESCHED is returned before anything is launched.
// Unlike NCCL point-to-point calls, these hand-offs are matched by buffer, not by call
// order, so the order-mismatch deadlock the paper warns about cannot occur; only the cyclic
// one can.
#include <algorithm>

#include "stage_impl.h"

using namespace jpp;

struct jpp_pipeline {
  std::vector<jpp_stage*> actors;
  int P = 0, V = 0, S = 0, M = 0;
  size_t bbytes = 0;
  bool head = false, embed = false;
  // boundary s (between stage s and s + 1), microbatch i -> index s * M + i
  std::vector<char*> act, cot;
  std::vector<hipEvent_t> act_ready, cot_ready;
  bool bound = false;
  bool ran = false;
};

namespace {

#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t _e = (expr);                             \
    if (_e != hipSuccess) return fail_hip(_e, #expr);   \
  } while (0)

size_t boundary_bytes(const jpp_layer_config& c) {
  return align_up((size_t)c.seq_len * c.microbatch * c.d_model * (c.dtype == JPP_BF16 ? 2 : 4));
}

// The producing task of `t`'s operand as (actor, key into that actor's tables), or actor -1.
struct Dep { int actor; size_t key; bool is_fwd; };
struct Shape { int P, V, M, S; };
Dep producer_of(const Shape& p, const jpp_task& t) {
  if (t.ty == JPP_FWD) {
    if (t.stage == 0) return {-1, 0, true};
    const int s = t.stage - 1;
    return {s % p.P, (size_t)(s / p.P) * p.M + t.i, true};
  }
  if (t.stage == p.S - 1) return {-1, 0, false};
  const int s = t.stage + 1;
  return {s % p.P, (size_t)(s / p.P) * p.M + t.i, false};
}

// Merges the lists: order[k] = actor that enqueues its next task at step k.  Fails with the
// blocked tasks named when the lists wait for each other.
jpp_status merge_lists(const Shape& p, const jpp_task* const* lists, const int* n, std::vector<int>& order) {
  std::vector<int> next(p.P, 0);
  std::vector<std::vector<char>> fwd_done(p.P), bwd_done(p.P);
  for (int r = 0; r < p.P; ++r) {
    fwd_done[r].assign((size_t)p.V * p.M, 0);
    bwd_done[r].assign((size_t)p.V * p.M, 0);
  }
  size_t total = 0;
  for (int r = 0; r < p.P; ++r) total += n[r];
  order.clear();
  while (order.size() < total) {
    bool moved = false;
    for (int r = 0; r < p.P; ++r) {
      if (next[r] == n[r]) continue;
      const jpp_task& t = lists[r][next[r]];
      const Dep d = producer_of(p, t);
      if (d.actor >= 0 && !(d.is_fwd ? fwd_done[d.actor][d.key] : bwd_done[d.actor][d.key])) continue;
      const size_t key = (size_t)(t.stage / p.P) * p.M + t.i;
      (t.ty == JPP_FWD ? fwd_done : bwd_done)[r][key] = 1;
      order.push_back(r);
      ++next[r];
      moved = true;
    }
    if (!moved) {
      std::string msg = "deadlock: the task lists wait for each other:";
      for (int r = 0; r < p.P; ++r)
        if (next[r] < n[r]) {
          const jpp_task& t = lists[r][next[r]];
          msg += " actor " + std::to_string(r) + " at (i=" + std::to_string(t.i) +
                 (t.ty == JPP_FWD ? ", fwd, stage " : ", bwd, stage ") + std::to_string(t.stage) + ")";
        }
      return fail(JPP_ESCHED, msg);
    }
  }
  return JPP_OK;
}

}  // namespace

extern "C" {

jpp_status jpp_pipeline_merge_order(int n_actors, int n_virtual, int n_microbatches, const jpp_task* const* task_lists,
                                    const int* n_tasks, int* order, int cap) {
  if (n_actors < 1 || n_virtual < 1 || n_microbatches < 1 || !task_lists || !n_tasks || !order)
    return fail(JPP_EINVAL, "bad arguments");
  const Shape sh{n_actors, n_virtual, n_microbatches, n_actors * n_virtual};
  long long total = 0;
  for (int r = 0; r < n_actors; ++r) {
    if (n_tasks[r] < 0 || (n_tasks[r] > 0 && !task_lists[r])) return fail(JPP_EINVAL, "null task list");
    for (int k = 0; k < n_tasks[r]; ++k) {
      const jpp_task& t = task_lists[r][k];
      if (t.i < 0 || t.i >= n_microbatches || t.stage < 0 || t.stage >= sh.S || t.stage % n_actors != r ||
          (t.ty != JPP_FWD && t.ty != JPP_BWD))
        return fail(JPP_ESCHED, "actor " + std::to_string(r) + ": task out of range or on the wrong actor");
    }
    total += n_tasks[r];
  }
  if (total > cap) return fail(JPP_EINVAL, "output array too small");
  std::vector<int> o;
  const jpp_status rc = merge_lists(sh, task_lists, n_tasks, o);
  if (rc != JPP_OK) return rc;
  std::copy(o.begin(), o.end(), order);
  return JPP_OK;
}

size_t jpp_pipeline_arena_bytes(const jpp_layer_config* cfg, int n_actors, int n_microbatches) {
  if (!cfg || n_actors < 1 || n_microbatches < 1 || cfg->n_virtual < 1) {
    fail(JPP_EINVAL, "bad pipeline shape");
    return 0;
  }
  const size_t S = (size_t)n_actors * cfg->n_virtual;
  return 2 * (S - 1) * n_microbatches * boundary_bytes(*cfg);
}

jpp_status jpp_pipeline_create(jpp_stage* const* actors, int n_actors, void* arena_dev, size_t arena_bytes,
                               jpp_pipeline** out) {
  if (!out) return fail(JPP_EINVAL, "null output pointer");
  *out = nullptr;
  if (!actors || n_actors < 1) return fail(JPP_EINVAL, "no actors");
  for (int r = 0; r < n_actors; ++r)
    if (!actors[r]) return fail(JPP_EINVAL, "null actor");
  const jpp_layer_config& c0 = actors[0]->cfg;
  const int V = c0.n_virtual, M = actors[0]->M;
  for (int r = 0; r < n_actors; ++r) {
    const jpp_stage& a = *actors[r];
    const jpp_layer_config& c = a.cfg;
    for (int q = 0; q < r; ++q)
      if (actors[q] == actors[r]) return fail(JPP_EINVAL, "the same actor twice");
    if (a.M != M || c.n_virtual != V || c.dtype != c0.dtype || c.d_model != c0.d_model || c.seq_len != c0.seq_len ||
        c.microbatch != c0.microbatch)
      return fail(JPP_EINVAL, "actors must agree on microbatches, virtual stages, dtype and boundary shape");
    for (int v = 0; v < V; ++v)
      if (c.stage_ids[v] != v * n_actors + r)
        return fail(JPP_EINVAL, "actor r must own the stages r, P + r, 2P + r, ... in that order");
    if (c.loss_head && r != n_actors - 1) return fail(JPP_EINVAL, "only the last actor can carry the loss head");
    if (c.embed && r != 0) return fail(JPP_EINVAL, "only the first actor can carry the token embedding");
    if (a.running) return fail(JPP_ESTATE, "actor is in the middle of a run");
  }
  const size_t need = jpp_pipeline_arena_bytes(&c0, n_actors, M);
  if (need > 0 && (!arena_dev || ((uintptr_t)arena_dev % kAlign) != 0))
    return fail(JPP_EINVAL, "arena must be 256-byte aligned");
  if (need > arena_bytes) return fail(JPP_EINVAL, "arena too small");
  jpp_pipeline* p = new jpp_pipeline;
  p->actors.assign(actors, actors + n_actors);
  p->P = n_actors; p->V = V; p->S = V * n_actors; p->M = M;
  p->bbytes = boundary_bytes(c0);
  p->head = actors[n_actors - 1]->cfg.loss_head != 0;
  p->embed = actors[0]->cfg.embed != 0;
  const size_t nb = (size_t)(p->S - 1) * M;
  p->act.resize(nb); p->cot.resize(nb);
  p->act_ready.assign(nb, nullptr); p->cot_ready.assign(nb, nullptr);
  char* base = (char*)arena_dev;
  for (size_t k = 0; k < nb; ++k) {
    p->act[k] = base + k * p->bbytes;
    p->cot[k] = base + (nb + k) * p->bbytes;
  }
  hipError_t e = hipSuccess;
  for (size_t k = 0; k < nb && e == hipSuccess; ++k) {
    e = hipEventCreateWithFlags(&p->act_ready[k], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p->cot_ready[k], hipEventDisableTiming);
  }
  if (e != hipSuccess) { jpp_pipeline_destroy(p); return fail_hip(e, "pipeline events"); }
  *out = p;
  return JPP_OK;
}

void jpp_pipeline_destroy(jpp_pipeline* p) {
  if (!p) return;
  for (jpp_stage* a : p->actors) {
    // the actors outlive the pipeline: wait for what it enqueued and unhook them
    if (a->cs) (void)hipStreamSynchronize(a->cs);
    if (a->ss) (void)hipStreamSynchronize(a->ss);
    a->wait_x.clear(); a->wait_cot.clear(); a->signal_y.clear(); a->signal_dx.clear();
    a->avail_x.clear(); a->avail_cot.clear();
  }
  for (hipEvent_t e : p->act_ready) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->cot_ready) if (e) (void)hipEventDestroy(e);
  delete p;
}

jpp_status jpp_pipeline_bind(jpp_pipeline* p, const void* const* x_in, void* const* dx_out,
                             const int32_t* const* targets, const void* const* cot_in, void* const* y_out) {
  if (!p || !x_in || (!dx_out && !p->embed)) return fail(JPP_EINVAL, "x_in and dx_out are required");
  if (p->head && !targets) return fail(JPP_EINVAL, "targets are required: the last stage has a loss head");
  if (!p->head && (!cot_in || !y_out)) return fail(JPP_EINVAL, "cot_in and y_out are required without a loss head");
  const int P = p->P, V = p->V, M = p->M, S = p->S;
  for (int i = 0; i < M; ++i) {
    if (!x_in[i] || (!p->embed && !dx_out[i])) return fail(JPP_EINVAL, "null boundary buffer");
    if (p->head ? !targets[i] : (!cot_in[i] || !y_out[i])) return fail(JPP_EINVAL, "null boundary buffer");
  }
  for (int r = 0; r < P; ++r) {
    jpp_stage* a = p->actors[r];
    const size_t n = (size_t)V * M;
    std::vector<const void*> in_x(n), in_c(n, nullptr);
    std::vector<void*> out_y(n, nullptr), out_dx(n);
    std::vector<const int32_t*> tg(n, nullptr);
    a->wait_x.assign(n, nullptr); a->wait_cot.assign(n, nullptr);
    a->signal_y.assign(n, nullptr); a->signal_dx.assign(n, nullptr);
    for (int v = 0; v < V; ++v) {
      const int s = v * P + r;
      for (int i = 0; i < M; ++i) {
        const size_t k = (size_t)v * M + i;
        const size_t below = s > 0 ? (size_t)(s - 1) * M + i : 0, above = (size_t)s * M + i;
        in_x[k] = s == 0 ? x_in[i] : p->act[below];
        out_dx[k] = s == 0 ? (p->embed ? nullptr : dx_out[i]) : (void*)p->cot[below];
        if (s > 0) { a->wait_x[k] = p->act_ready[below]; a->signal_dx[k] = p->cot_ready[below]; }
        if (s == S - 1) {
          if (p->head) tg[k] = targets[i];
          else { in_c[k] = cot_in[i]; out_y[k] = y_out[i]; }
        } else {
          in_c[k] = p->cot[above];
          out_y[k] = p->act[above];
          a->wait_cot[k] = p->cot_ready[above];
          a->signal_y[k] = p->act_ready[above];
        }
      }
    }
    // a head actor with several virtual stages still needs a non-null targets table
    const bool any_head = a->cfg.loss_head != 0;
    if (any_head)
      for (size_t k = 0; k < n; ++k)
        if (!tg[k]) tg[k] = targets[k % M];
    jpp_status rc = jpp_stage_bind_boundary(a, in_x.data(), in_c.data(), out_y.data(), out_dx.data(),
                                            any_head ? tg.data() : nullptr);
    if (rc != JPP_OK) return rc;
  }
  p->bound = true;
  return JPP_OK;
}

jpp_status jpp_pipeline_run(jpp_pipeline* p, const jpp_task* const* task_lists, const int* n_tasks,
                            void* const* compute_streams, void* const* side_streams) {
  if (!p || !task_lists || !n_tasks || !compute_streams || !side_streams) return fail(JPP_EINVAL, "null argument");
  if (!p->bound) return fail(JPP_ESTATE, "pipeline boundary buffers not bound");
  const int P = p->P;
  for (int r = 0; r < P; ++r) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    HIP_TRY(hipStreamIsCapturing((hipStream_t)compute_streams[r], &cap));
    if (cap != hipStreamCaptureStatusNone)
      return fail(JPP_ESTATE, "jpp_pipeline_run cannot be recorded into a HIP graph");
  }
  // everything that can be refused is checked before anything is enqueued
  for (int r = 0; r < P; ++r) {
    if (!task_lists[r] || n_tasks[r] < 0) return fail(JPP_EINVAL, "null task list");
    if (compute_streams[r] == side_streams[r]) return fail(JPP_EINVAL, "compute and side streams must differ");
    const jpp_stage& a = *p->actors[r];
    if (a.running) return fail(JPP_ESTATE, "actor is in the middle of a run");
    for (bool b : a.params_set)
      if (!b) return fail(JPP_ESTATE, "parameters not set for every virtual stage");
    std::string why;
    int peak = 0;
    const int rc = validate_tasks(&a.cfg, a.M, task_lists[r], n_tasks[r], &peak, why);
    if (rc != JPP_OK) return fail((jpp_status)rc, "actor " + std::to_string(r) + ": " + why);
    if (peak > a.max_in_flight)
      return fail(JPP_ECAPACITY, "actor " + std::to_string(r) + " keeps " + std::to_string(peak) +
                                     " stashes alive, its arena holds " + std::to_string(a.max_in_flight));
  }
  std::vector<int> order;
  jpp_status rc = merge_lists(Shape{p->P, p->V, p->M, p->S}, task_lists, n_tasks, order);
  if (rc != JPP_OK) return rc;

  // Boundary buffers are rewritten by this run: every actor starts after every actor's
  // previous run (device-side waits).
  for (int r = 0; r < P; ++r)
    for (int q = 0; q < P; ++q) {
      const jpp_stage& b = *p->actors[q];
      if (q == r || !b.end_compute.recorded) continue;
      HIP_TRY(hipStreamWaitEvent((hipStream_t)compute_streams[r], b.end_compute.ev, 0));
      HIP_TRY(hipStreamWaitEvent((hipStream_t)compute_streams[r], b.end_side.ev, 0));
      HIP_TRY(hipStreamWaitEvent((hipStream_t)side_streams[r], b.end_compute.ev, 0));
      HIP_TRY(hipStreamWaitEvent((hipStream_t)side_streams[r], b.end_side.ev, 0));
    }
  auto abort_run = [&](jpp_status code) {
    for (jpp_stage* a : p->actors) a->running = false;
    return code;
  };
  for (int r = 0; r < P; ++r) {
    jpp_stage* a = p->actors[r];
    // nothing of another actor has been enqueued yet; the pipeline's own inputs are there
    a->avail_x.assign((size_t)p->V * p->M, 0);
    a->avail_cot.assign((size_t)p->V * p->M, 0);
    for (int v = 0; v < p->V; ++v)
      for (int i = 0; i < p->M; ++i) {
        const int s = v * P + r;
        if (s == 0) a->avail_x[(size_t)v * p->M + i] = 1;
        if (s == p->S - 1) a->avail_cot[(size_t)v * p->M + i] = 1;
      }
    rc = run_begin(a, task_lists[r], n_tasks[r], compute_streams[r], side_streams[r]);
    if (rc != JPP_OK) return abort_run(rc);
  }
  for (int r : order) {
    jpp_stage* a = p->actors[r];
    const jpp_task t = a->run_tasks[a->run_next];
    rc = run_step(a);
    if (rc != JPP_OK) return abort_run(rc);
    // the task's send is enqueued: its consumer may now issue the matching receive
    if (t.ty == JPP_FWD && t.stage < p->S - 1) {
      const int s = t.stage + 1;
      p->actors[s % P]->avail_x[(size_t)(s / P) * p->M + t.i] = 1;
    } else if (t.ty == JPP_BWD && t.stage > 0) {
      const int s = t.stage - 1;
      p->actors[s % P]->avail_cot[(size_t)(s / P) * p->M + t.i] = 1;
    }
  }
  for (int r = 0; r < P; ++r) {
    rc = run_end(p->actors[r]);
    if (rc != JPP_OK) return abort_run(rc);
  }
  p->ran = true;
  return JPP_OK;
}

jpp_status jpp_pipeline_sum_tied_gradients(jpp_pipeline* p, void* stream) {
  if (!p) return fail(JPP_EINVAL, "null pipeline");
  jpp_stage* first = p->actors.front();
  jpp_stage* last = p->actors.back();
  if (!p->embed || !p->head) return fail(JPP_ESTATE, "tied weights need an embedding on the first stage and a loss head on the last");
  if (first->cfg.vocab != last->cfg.vocab) return fail(JPP_EINVAL, "embedding and head disagree on vocab");
  for (jpp_stage* a : p->actors)
    if (a->running) return fail(JPP_ESTATE, "an actor is in the middle of a run");
  hipStream_t s = (hipStream_t)stream;
  // after both actors' last runs (device-side waits)
  if (first->end_compute.recorded) HIP_TRY(hipStreamWaitEvent(s, first->end_compute.ev, 0));
  if (last->end_compute.recorded) HIP_TRY(hipStreamWaitEvent(s, last->end_compute.ev, 0));
  float* g1 = first->grads[0] + first->w_embed;
  float* g2 = last->grads[p->V - 1] + last->w_head;
  HIP_TRY(launch_tied_sum(g1, g2, (size_t)first->cfg.vocab * first->cfg.d_model, s));
  return JPP_OK;
}

jpp_status jpp_pipeline_sync(jpp_pipeline* p) {
  if (!p) return fail(JPP_EINVAL, "null pipeline");
  for (jpp_stage* a : p->actors) {
    if (a->cs) HIP_TRY(hipStreamSynchronize(a->cs));
    if (a->ss) HIP_TRY(hipStreamSynchronize(a->ss));
  }
  return JPP_OK;
}

}  // extern "C"
