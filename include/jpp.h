/* jpp.h -- C ABI of the MI355X pipeline-stage executor.
 *
 * One `jpp_stage` is one actor of an MPMD pipeline (paper, Section 2.2: an actor
 * is a group of devices executing the same logic; here: one gfx950 GPU).  It owns
 * one or more pipeline stages ("circular repeat", Section 2.2.1), each made of
 * transformer decoder layers, and executes a per-actor list of Task(i, ty, stage)
 * records (Section 4.2) in ONE call (Section 4.4, task fusion), accumulating
 * parameter gradients over the microbatches (Section 3.1: grads start at zero and
 * are summed, no 1/M; per-microbatch losses are collected as a vector).
 *
 * Conventions
 *  - Plain C.  No exception crosses the boundary; every entry point returns a
 *    jpp_status (or a size / pointer where stated) and records a message that
 *    jpp_last_error() returns (thread-local).
 *  - "dev" pointers are device (HBM) addresses on the current HIP device, "host"
 *    pointers are ordinary process memory.  Streams are hipStream_t passed as
 *    void*.  The library allocates no device memory: everything lives in the
 *    caller's arena and boundary buffers.
 *  - Storage type of parameters, activations and boundary tensors is given by
 *    jpp_layer_config.dtype; gradients and losses are always fp32.
 *  - Tensors are row-major.  A boundary tensor is [microbatch, seq_len, d_model].
 *    A linear weight is [out_features, in_features] (y = x W^T).
 */
#ifndef JPP_H
#define JPP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct jpp_stage jpp_stage; /* opaque; created and destroyed by the library */

typedef enum {
  JPP_OK = 0,
  JPP_EINVAL = 1,    /* bad config, NULL pointer, size mismatch, unsupported shape        */
  JPP_ESCHED = 2,    /* task list violates a rule of jpp_schedule_validate; nothing ran  */
  JPP_ECAPACITY = 3, /* task list needs more live stashes than max_in_flight             */
  JPP_EDEVICE = 4,   /* a HIP call failed (message holds the HIP error string)           */
  JPP_ESTATE = 5     /* e.g. run before parameters or boundary buffers were supplied     */
} jpp_status;

enum { JPP_FWD = 0, JPP_BWD = 1 };
enum { JPP_F32 = 0, JPP_BF16 = 1 };
enum { JPP_LAYERNORM = 0, JPP_RMSNORM = 1 };
enum { JPP_GELU = 0, JPP_GELU_TANH = 1, JPP_SWIGLU = 2 };
enum { JPP_GPIPE = 0, JPP_1F1B = 1, JPP_INTERLEAVED_1F1B = 2 };
#define JPP_MAX_VIRTUAL 8

/* Task(i, ty, stage) of Section 4.2: microbatch index, JPP_FWD/JPP_BWD, GLOBAL stage index. */
typedef struct { int32_t i; int32_t ty; int32_t stage; } jpp_task;

/* The paper does not define the layer (its Evaluation section only names GPT-3 and
 * Llama 2); a stage is n_layers pre-norm decoder layers
 *     n1 = Norm(x); [q|k|v] = n1 Wqkv^T (+b); q,k <- RoPE (opt); O = causal attention;
 *     x1 = x + O Wo^T (+b); n2 = Norm(x1);
 *     GeLU:   y = x1 + gelu(n2 W1^T + b1) W2^T + b2
 *     SwiGLU: [g|u] = n2 W1^T (W1 is [2*d_ffn, d_model], gate rows first); y = x1 + (silu(g)*u) W2^T
 * optionally followed (loss_head) by a final norm, an untied LM head [vocab, d_model]
 * and the mean-token cross-entropy, whose backward is seeded with dloss = 1.  With several
 * virtual stages the head belongs to the LAST one (local index n_virtual-1) only; the head's
 * parameter slots exist in every virtual stage's buffer and stay unused (zero gradient)
 * in the others. */
typedef struct {
  int32_t dtype;      /* JPP_F32: everything fp32.  JPP_BF16: bf16 storage, fp32 accumulate   */
  int32_t n_layers;   /* decoder layers per (virtual) stage                                   */
  int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, seq_len, microbatch;
  int32_t norm;       /* JPP_LAYERNORM (gain, offset) or JPP_RMSNORM (gain); biased variance  */
  int32_t act;        /* JPP_GELU (erf form), JPP_GELU_TANH, JPP_SWIGLU                       */
  int32_t use_bias;   /* 1: bqkv, bo, b1, b2 exist (and get gradients)                        */
  int32_t rope;       /* 1: rotate q,k; pairs (j, j+head_dim/2), angle pos*theta^(-2j/hd)     */
  float rope_theta;
  float norm_eps;
  int32_t loss_head;  /* 1: final norm + LM head + mean-token CE; output is loss[i]           */
  int32_t vocab;
  int32_t remat;      /* 1: rematerialisation (Section 2.2.1: trade memory for recomputation): a
                       * forward keeps only each layer's input; the backward re-runs the layer's
                       * forward (without its last GEMM) before differentiating it.  Same results,
                       * bit for bit; the stash shrinks from (8 d + 2 f) T to d T elements per layer */
  int32_t wgrad_group; /* 0 or 1: every backward task adds its own weight gradients.  g > 1: the
                       * microbatches g*k .. g*k+g-1 of a stage form a group (the last one may be
                       * smaller).  Their backward tasks run the input-gradient chain, the norm
                       * gradients and the send as usual and keep the operands of the
                       * weight-gradient GEMMs (activations and cotangents) in the stash; the task
                       * that completes the group runs one GEMM per weight (and one column sum per
                       * bias) over all the group's tokens, so the fp32 gradient is read and
                       * written once per group, not once per microbatch.  The sums are those of Section 3.1; only the rounding
                       * order differs from g = 1, and it depends on the microbatch indices alone,
                       * so the result is still the same for every schedule.  A group occupies g
                       * stash places from its first forward to its last backward
                       * (jpp_schedule_validate counts that).  Not together with remat.         */
  int32_t embed;      /* 1: the actor's FIRST virtual stage (local index 0) starts with a token
                       * embedding: its input is int32 token ids [microbatch, seq_len] and
                       * x = E[ids] with the table "embed.w" [vocab, d_model] (ids outside
                       * [0, vocab) read as a zero row and get no gradient).  Its backward adds the
                       * cotangent rows of x to the rows of the table's gradient, in position
                       * order, and sends nothing.  Needs vocab.  The table's parameter slots
                       * exist in every virtual stage's buffer and stay unused elsewhere.         */
  int32_t n_virtual;  /* stages owned by this actor                                           */
  int32_t stage_ids[JPP_MAX_VIRTUAL]; /* their global indices (interleaved: v*P + rank)       */
} jpp_layer_config;

/* ---- host-only schedule helpers (no GPU needed) ------------------------------------ */

/* Number of tasks of a schedule for one actor: 2*M*V (V = 1 for GPipe and 1F1B).
 * Returns -1 on invalid arguments (P<1, rank outside [0,P), V<1, M<1, interleaved with
 * M % P != 0). */
int jpp_schedule_len(int kind, int P, int rank, int V, int M);

/* Writes actor `rank`'s task list for a pipeline of P actors and M microbatches
 * (Section 2.2.1 for the three orders; Section 4.2 for the record format and the
 * interleaved example).  Every generator emits, per stage, backward tasks in ascending
 * microbatch order.  `out` (host) must hold `cap` >= jpp_schedule_len() records.
 * JPP_EINVAL on bad arguments or insufficient cap. */
jpp_status jpp_schedule_make(int kind, int P, int rank, int V, int M, jpp_task* out, int cap);

/* Checks a task list (host) against the rules that follow from Section 2.2.1: every
 * (i, ty, stage) with stage in cfg->stage_ids and 0 <= i < M appears exactly once, and
 * BWD(i, s) comes after FWD(i, s).  On success *peak_in_flight (optional) receives the
 * largest number of (microbatch, stage) activation stashes alive at once.
 * JPP_ESCHED on violation. */
jpp_status jpp_schedule_validate(const jpp_layer_config* cfg, int M, const jpp_task* tasks, int n,
                                 int* peak_in_flight);

/* ---- stage life cycle --------------------------------------------------------------- */

/* Bytes of device memory a stage needs for parameters, fp32 gradients, `max_in_flight`
 * activation stash slots (Section 2.2.1: GPipe needs M, 1F1B about the number of
 * stages), backward workspace and send/receive staging.  0 on invalid config. */
size_t jpp_stage_arena_bytes(const jpp_layer_config* cfg, int n_microbatches, int max_in_flight);

/* Creates the executor inside the caller-owned arena (`arena_dev`, 256-byte aligned,
 * at least jpp_stage_arena_bytes()).  The arena must outlive the stage; the library
 * never frees it.  Gradients and parameters are NOT initialised: call
 * jpp_stage_set_params and jpp_stage_zero_grads.  `max_in_flight` one above the
 * schedule's peak lets the next forward's input be prefetched while a slot is still held. */
jpp_status jpp_stage_create(const jpp_layer_config* cfg, int n_microbatches, int max_in_flight,
                            void* arena_dev, size_t arena_bytes, jpp_stage** out);
void jpp_stage_destroy(jpp_stage* st);

/* Parameter layout of one virtual stage: tensors 0..n-1 in order (layer by layer:
 * ln1_g [ln1_b] wqkv [bqkv] wo [bo] ln2_g [ln2_b] w1 [b1] w2 [b2]; then lnf_g [lnf_b]
 * w_head).  shape[1] = 0 for vectors.  elem_offset is the tensor's element offset in
 * the flat parameter buffer AND in the flat fp32 gradient buffer.  Returns the number
 * of tensors when idx < 0 (other outputs untouched), JPP_OK (0) otherwise; a negative
 * value (-JPP_EINVAL) on error. */
int jpp_stage_param_info(const jpp_stage* st, int idx, const char** name, int64_t shape[2],
                         size_t* elem_offset);
size_t jpp_stage_param_count(const jpp_stage* st); /* elements per virtual stage */

/* Copies one virtual stage's flat parameter buffer (storage dtype, param_count elements,
 * layout above) into the arena.  vstage is the LOCAL index 0..n_virtual-1.  `src` may be
 * a host or a device pointer (src_on_device).  Synchronous. */
jpp_status jpp_stage_set_params(jpp_stage* st, int vstage, const void* src, int src_on_device);

/* Section 4.2: a stage receives its input activation from the previous stage and its output's
 * cotangent from the next one, and sends its output and its input's cotangent the other way; on
 * one GPU the peers are buffers.  Boundary buffers, caller-owned, all device pointers to [microbatch, seq_len, d_model]
 * tensors of the storage dtype; each host array has n_virtual * M entries indexed
 * [vstage * M + i].  inbox_x[i]: activation received for FWD(i); inbox_cot[i]: cotangent
 * received for BWD(i) and outbox_y[i]: output sent after FWD(i) (entries of the virtual
 * stage that carries the loss head are ignored; the arrays may be NULL when that is the only
 * one); outbox_dx[i]: input cotangent sent after BWD(i).  For the virtual stage that carries
 * the token embedding inbox_x[i] points to int32 token ids [microbatch, seq_len], read in place
 * by FWD(i) and BWD(i) (they must stay valid for the run), and outbox_dx[i] is ignored.  targets[i] (loss_head only, read
 * for the head's virtual stage): device int32 [microbatch, seq_len] token ids in [0, vocab).
 * The host arrays are copied. */
jpp_status jpp_stage_bind_boundary(jpp_stage* st, const void* const* inbox_x,
                                   const void* const* inbox_cot, void* const* outbox_y,
                                   void* const* outbox_dx, const int32_t* const* targets);

/* Section 3.1: the accumulation loop starts from zero gradients (`grads = 0`, then every
 * backward adds its microbatch's share).  grads <- 0 and losses <- 0 for all virtual stages,
 * enqueued on `stream`. */
jpp_status jpp_stage_zero_grads(jpp_stage* st, void* stream);

/* Executes the task list (host array, read during the call only) in the order given:
 * validation first (JPP_ESCHED / JPP_ECAPACITY: nothing is launched), then every kernel
 * of every task is enqueued without any host synchronisation (Section 4.4): forward tasks
 * on compute_stream, backward tasks on two library-owned streams that start after the work
 * already queued on compute_stream and are joined back into it before the call returns, so
 * that a forward and a backward of different microbatches, and a layer's weight and input
 * gradients, may overlap (Section 2.2.1: any order that honours the data dependencies).
 * Receives are copies inbox -> stage input issued on side_stream ahead of their consumer
 * (prefetch), sends are copies stage output -> outbox issued on side_stream right after the
 * producing task (Section 4.2); staging buffers whose send has not completed are parked in a
 * pending-deletion queue and reclaimed later (Section 4.3).  Returns after enqueueing; the
 * side stream, too, is joined into compute_stream at the end, so the run is complete when
 * compute_stream is.  The two streams must differ and have the default priority.  Calls on
 * one stage must not overlap.
 * HIP graphs: JPP_ESTATE when compute_stream is capturing (the run queries event completion
 * and refers to events of earlier runs; recording it into a graph is not supported). */
jpp_status jpp_stage_run(jpp_stage* st, const jpp_task* tasks, int n_tasks, void* compute_stream,
                         void* side_stream);

/* Section 3.1: what the accumulation loop returns, the gradients summed over the microbatches
 * (no 1/M).  Synchronises the streams of the last run and returns a borrowed device pointer to the
 * flat fp32 gradient buffer of local virtual stage `vstage` (param_count elements, same
 * offsets as the parameters).  Valid until zero_grads / destroy. */
jpp_status jpp_stage_grads(jpp_stage* st, int vstage, const float** grads_dev, size_t* n_elems);

/* loss_head stages: borrowed device pointer to the fp32 loss vector [n_virtual * M], entry
 * [vstage * M + i]; only the head's virtual stage (the last) is written (Section 3.1: losses
 * are collected per microbatch, not averaged over microbatches). Synchronises. */
jpp_status jpp_stage_losses(jpp_stage* st, const float** loss_dev);

/* ---- parameter update after accumulation (Section 3.1: the step ends with
 * state.apply_gradient(grads, learning_rate); the paper names no optimizer) -----------
 * Per element, g = accumulated gradient (sum over microbatches, no 1/M: scale lr accordingly):
 *   JPP_OPT_SGD:   w <- w - lr (g + weight_decay w), computed in fp32 from the stored w and
 *                  rounded back to the storage dtype; no state.
 *   JPP_OPT_ADAMW: fp32 master weights and moments; step t = 1, 2, ...
 *                  m <- b1 m + (1-b1) g; v <- b2 v + (1-b2) g^2;
 *                  w <- w - lr (m/(1-b1^t) / (sqrt(v/(1-b2^t)) + eps) + weight_decay w);
 *                  the stored parameters become the master weights rounded to the storage dtype.
 * Every parameter is treated alike (weight decay included). */
enum { JPP_OPT_SGD = 0, JPP_OPT_ADAMW = 1 };
typedef struct {
  int32_t kind;       /* JPP_OPT_*                                  */
  float lr, beta1, beta2, eps, weight_decay;
  int32_t step;       /* AdamW: 1-based step count (bias correction) */
} jpp_optimizer_step;

/* Borrowed device pointer to the parameters of local virtual stage `vstage` (storage dtype,
 * param_count elements, layout of jpp_stage_param_info).  Waits for the compute stream. */
jpp_status jpp_stage_params(jpp_stage* st, int vstage, const void** params_dev, size_t* n_elems);

/* AdamW state: n_virtual x [master | m | v], param_count floats each, in caller-owned device
 * memory of jpp_stage_optimizer_bytes (0 for SGD), 16-byte aligned.  bind copies the current
 * parameters into the master weights and zeroes the moments (enqueued on `stream`). */
size_t jpp_stage_optimizer_bytes(const jpp_stage* st, int kind);
jpp_status jpp_stage_optimizer_bind(jpp_stage* st, int kind, void* state_dev, size_t state_bytes, void* stream);

/* Enqueues the update of every virtual stage's parameters from its gradient buffer on
 * `stream`; use the compute stream of jpp_stage_run so that it follows the accumulation and
 * precedes the next run.  Gradients are left as they are (call jpp_stage_zero_grads). */
jpp_status jpp_stage_apply_gradients(jpp_stage* st, const jpp_optimizer_step* step, void* stream);

/* Process-wide, read at the start of every run: which streams carry the backward tasks.
 * 0: input-gradient chain and weight-gradient GEMMs on two library-owned streams (three-way
 * overlap with the forward stream); 1: both on one library-owned stream; 2: everything on
 * compute_stream.  -1 (default): chosen per stage from its size: 2 when the layer's
 * smallest GEMM (the attention output projection, 2 T d n_q_heads head_dim flop) has at
 * least 5e10 flop, because kernels that fill the whole device on their own only disturb each
 * other's cache when they run side by side, else 0, where overlap fills the gaps that short
 * kernels leave.  Results are identical in every mode. */
void jpp_set_stream_mode(int mode);
/* Process-wide, read by every task: where GeLU (either form, bf16 storage) is evaluated.
 * Bit 0: by the epilogue of the FFN-up GEMM of a forward pass, which then stores h and
 * a = gelu(h); bit 1: by the epilogue of the FFN-down input-gradient GEMM of a backward pass,
 * which then stores dh = da * gelu'(h) and never da.  A clear bit leaves that direction to
 * the element-wise kernel after the GEMM.  Default (and any negative value): 3.  On MI355X
 * the choice moves the step of a GPT-3-175B-shaped stage (d 12288, 2048 tokens) by less than its run-to-run spread (all four values within
 * 0.15 %): the epilogue's extra arithmetic and second store come when a whole round of tiles
 * ends at once and no MFMA work is left to hide them, which costs about what the streaming
 * kernel did; fusing saves that kernel's 0.4 GB (forward) and 0.6 GB (backward) of HBM
 * traffic per layer and microbatch.  Results are identical for every value (both routes
 * round h, a and da to bf16 at the same points and share the GeLU arithmetic). */
void jpp_set_fused_activation(int mask);
/* The mode (0, 1 or 2) that the next run of `st` uses under the current setting. */
int jpp_stage_stream_mode(const jpp_stage* st);

/* Introspection of the last run (host bookkeeping, used by tests). */
int jpp_stage_peak_in_flight(const jpp_stage* st);   /* stash slots high-water mark            */
int jpp_stage_pending_peak(const jpp_stage* st);     /* pending-deletion queue high-water mark */
int jpp_stage_prefetched(const jpp_stage* st);       /* receives issued ahead of their consumer */

const char* jpp_last_error(void);

/* ---- several actors on one device (Sections 4.2 and 4.4) ----------------------------
 * A pipeline of P actors; actor r is a jpp_stage created by the caller whose stage_ids are
 * {r, P + r, 2P + r, ...} (circular placement), all with the same n_microbatches, dtype and
 * boundary shape; only actor P-1 may have loss_head = 1 (the last global stage then ends in
 * the loss).  The pipeline owns the boundary buffers between consecutive stages (in the
 * caller's arena) and wires them into the actors with jpp_stage_bind_boundary: stage s sends
 * y to stage s+1 and dx to stage s-1 right after the producing task, the receiver copies it
 * in ahead of its consumer when it can.  Parameters are set on the actors directly;
 * gradients and losses are read from them (jpp_stage_grads, jpp_stage_losses of actor P-1).
 * Destroy the pipeline before its actors. */
typedef struct jpp_pipeline jpp_pipeline;

/* Host-only (no GPU needed): the order in which jpp_pipeline_run enqueues the tasks of
 * n_actors lists (actor r owning the stages r, P + r, ...): order[k] = the actor whose next
 * task is enqueued at step k; cap >= the total number of tasks.  JPP_ESCHED, naming the
 * blocked tasks, when the lists wait for each other in a cycle (Section 4.2). */
jpp_status jpp_pipeline_merge_order(int n_actors, int n_virtual, int n_microbatches,
                                    const jpp_task* const* task_lists, const int* n_tasks, int* order, int cap);

/* Bytes of device memory for the boundary buffers: 2 * (P * n_virtual - 1) * M tensors. */
size_t jpp_pipeline_arena_bytes(const jpp_layer_config* cfg, int n_actors, int n_microbatches);

/* arena_dev: device pointer, 256-byte aligned, caller-owned, at least arena_bytes (may be
 * NULL when there is a single stage).  JPP_EINVAL if the actors do not fit together. */
jpp_status jpp_pipeline_create(jpp_stage* const* actors, int n_actors, void* arena_dev, size_t arena_bytes,
                               jpp_pipeline** out);
void jpp_pipeline_destroy(jpp_pipeline* p);

/* Outer boundary, device pointers, M entries each: x_in[i] input of stage 0, dx_out[i] its
 * cotangent (when actor 0 has `embed`: x_in[i] are int32 token ids [microbatch, seq_len] and
 * dx_out is ignored, may be NULL); with a loss head targets[i] (int32 [microbatch, seq_len]); without one cot_in[i]
 * (cotangent of the last stage's output) and y_out[i] (that output). */
jpp_status jpp_pipeline_bind(jpp_pipeline* p, const void* const* x_in, void* const* dx_out,
                             const int32_t* const* targets, const void* const* cot_in, void* const* y_out);

/* One training step of the whole pipeline: task_lists[r] / n_tasks[r] is actor r's list,
 * compute_streams[r] / side_streams[r] its two streams (all distinct, default priority).
 * Every list is validated as in jpp_stage_run, then the lists are merged in a topological
 * order of the task graph (Section 4.2): round after round each actor enqueues its next task
 * if the task producing its operand (FWD(i, s-1) for FWD(i, s); BWD(i, s+1) for BWD(i, s)) is
 * already enqueued.  If no actor can move the lists wait for each other in a cycle:
 * JPP_ESCHED, with the blocked tasks in jpp_last_error(), and nothing has been launched.
 * Asynchronous, no host synchronisation; gradients accumulate as in jpp_stage_run (call
 * jpp_stage_zero_grads on every actor's compute stream first). */
jpp_status jpp_pipeline_run(jpp_pipeline* p, const jpp_task* const* task_lists, const int* n_tasks,
                            void* const* compute_streams, void* const* side_streams);

/* Tied embedding and LM head (Section 3, "Weight Sharing and Gradient Accumulation"): when
 * actor 0 has `embed` and actor P-1 the loss head, and the caller has set the same values in
 * "embed.w" of stage 0 and "head.w_head" of the last stage, the two tables are one weight
 * used twice.  Each run accumulates the partial gradient of each use where it is produced
 * (the carried states of the commuted loop); this call is the one addition after the loop:
 * on `stream`, after both actors' runs, both gradient regions become their sum, so that the
 * same update applied on both actors keeps the two copies bit-identical.  Call it once per
 * step, before jpp_stage_apply_gradients: the table then crosses between the two actors
 * once per step, not once per microbatch.  JPP_ESTATE without embed + head. */
jpp_status jpp_pipeline_sum_tied_gradients(jpp_pipeline* p, void* stream);

/* Waits for everything the last jpp_pipeline_run enqueued. */
jpp_status jpp_pipeline_sync(jpp_pipeline* p);

/* ---- single operations (the kernels the executor is made of) ------------------------
 * Exposed for op-level parity at shapes the CPU oracle cannot run end to end, and for
 * per-kernel profiling.  All pointers are device pointers; work is enqueued on `stream`.
 * dtype is JPP_F32 or JPP_BF16 storage; accumulation is fp32. */

/* C[M,N] (op)= sum_k A(m,k) * B(n,k)  (+ bias[n]) (+ residual[m,n]).
 * a_kstrided = 0: A(m,k) at A[m*lda + k];  1: at A[k*lda + m]  (same for B).
 * out_mode 0: store in storage dtype; 1: store fp32; 2: C(fp32) += result.
 * bias (storage dtype, [N]) and residual (storage dtype, ldc) may be NULL.
 * bf16 path requires M, N, K and leading dimensions to be multiples of 8. */
jpp_status jpp_op_gemm(int dtype, int M, int N, int K, const void* A, int lda, int a_kstrided,
                       const void* B, int ldb, int b_kstrided, void* C, int ldc, int out_mode,
                       const void* bias, const void* residual, void* stream);

/* jpp_op_gemm with a scratch buffer (device, fp32, 16-byte aligned, caller-owned, not shared
 * by launches that may overlap).  The bf16 path uses it in two cases.  Every mode: when the
 * last round of output tiles would fill at most half of the GPU, those tiles are cut into 2..8
 * ranges of k, the partial tiles go to the scratch and a second kernel sums them in ascending k
 * order and applies bias / residual / rounding (or, out_mode 2, adds the sum to C, once).
 * Accumulating mode (out_mode 2) only: when the whole output is at most two rounds of tiles
 * (a weight gradient smaller than the chip with a long contraction), every tile is cut.
 * jpp_op_gemm_workspace_bytes returns the bytes a shape needs (0: never split); with less (or
 * NULL) the launch is the unsplit one.  The result does not depend on timing either way. */
size_t jpp_op_gemm_workspace_bytes(int dtype, int M, int N, int K, int out_mode);
jpp_status jpp_op_gemm_ws(int dtype, int M, int N, int K, const void* A, int lda, int a_kstrided,
                          const void* B, int ldb, int b_kstrided, void* C, int ldc, int out_mode,
                          const void* bias, const void* residual, void* workspace,
                          size_t workspace_bytes, void* stream);

/* The bf16 GEMM with GeLU fused into its epilogue, as the stage runs its feed-forward block
 * (act: JPP_GELU or JPP_GELU_TANH; aux has the shape, type and leading dimension of C; bias and
 * workspace as in jpp_op_gemm_ws, storage-type output).
 *   backward = 0: C receives h = A B^T (+ bias) and aux receives gelu(h), evaluated on the stored
 *                 (rounded) h: the bits of jpp_op_gemm followed by jpp_op_act_fwd.
 *   backward = 1: aux holds h; the product, rounded to bf16, is the cotangent da of gelu(h) and C
 *                 receives da * gelu'(h): the bits of jpp_op_gemm followed by jpp_op_act_bwd,
 *                 without da ever being stored. */
jpp_status jpp_op_gemm_gelu(int M, int N, int K, const void* A, int lda, int a_kstrided, const void* B, int ldb,
                            int b_kstrided, void* C, int ldc, const void* bias, int act, int backward, void* aux,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Benchmarking knob: 0 (default) lets the library pick the bf16 GEMM tile configuration
 * from the problem size; 1..7 force one (tile M x N x K-stage, LDS stages, waves):
 * 1 = 256x256x32, 4, 4;  2 = 256x256x32, 5, 4;  3 = 128x128x32, 4, 4;  4 = 256x256x64, 2, 4;
 * 5 = 256x256x64, 2, 8 (all with HBM->LDS direct loads);  6 = 256x256x64, 2, 8,
 * 7 = 128x128x64, 2, 4 and 8 = 256x256x64, 2, 4 (one wave per SIMD, 128x128 wave tiles with
 * the accumulators in the accumulation registers) with register-staged loads (0 picks 6 for
 * large outputs, else 7).  Process-wide; results are identical for every value. */
void jpp_set_gemm_variant(int variant);

/* Causal self-attention over a fused qkv tensor [mb*seq, (Hq + 2*Hkv)*hd] (q heads, then
 * k heads, then v heads; query head h reads kv head h / (Hq/Hkv)).  out: [mb*seq, Hq*hd];
 * lse: fp32 [mb, Hq, seq] natural-log-sum-exp of the scaled scores. */
jpp_status jpp_op_attention_fwd(int dtype, int mb, int seq, int Hq, int Hkv, int hd,
                                const void* qkv, void* out, float* lse, void* stream);
/* dqkv has the layout of qkv.  Deterministic: no floating-point atomics.  `delta` is
 * fp32 scratch [mb, Hq, seq]. */
jpp_status jpp_op_attention_bwd(int dtype, int mb, int seq, int Hq, int Hkv, int hd,
                                const void* qkv, const void* out, const float* lse,
                                const void* dout, void* dqkv, float* delta, void* stream);
/* The same with a scratch buffer (device, fp32, 16-byte aligned, caller-owned).  Grouped-query
 * attention in bf16 with head_dim 128 uses it: the query heads of a kv head are then spread
 * over workgroups, their dK / dV rows go to the scratch and a second kernel sums them in
 * ascending head order (still no atomics), instead of one workgroup walking the whole group.
 * jpp_op_attention_bwd_scratch_bytes returns the bytes a shape needs (0: no use for scratch);
 * with less (or NULL) the call is jpp_op_attention_bwd. */
size_t jpp_op_attention_bwd_scratch_bytes(int dtype, int mb, int seq, int Hq, int Hkv, int hd);
jpp_status jpp_op_attention_bwd_ws(int dtype, int mb, int seq, int Hq, int Hkv, int hd,
                                   const void* qkv, const void* out, const float* lse,
                                   const void* dout, void* dqkv, float* delta, void* scratch,
                                   size_t scratch_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): jpp_op_attention_bwd without the `delta` argument.
 * The fp32 scratch [mb, Hq, seq] lives in a device array that is part of the library itself
 * (JPP_STATIC_SCRATCH_BYTES per GPU, held from the moment the library is loaded on that GPU to
 * the end of the process); the call allocates and frees nothing, on the device or through any
 * library.  JPP_EINVAL, with nothing launched, when 4 * mb * Hq * seq exceeds
 * JPP_STATIC_SCRATCH_BYTES.  dqkv gets the bits that jpp_op_attention_bwd writes.  All calls
 * on one GPU share the one array (each call overwrites what it reads, nothing has to be
 * cleared): calls that may overlap on a GPU (different streams, different threads) race on it
 * and must be serialised by the caller. */
#define JPP_STATIC_SCRATCH_BYTES (4u << 20)
jpp_status jpp_op_attention_bwd_static(int dtype, int mb, int seq, int Hq, int Hkv, int hd,
                                       const void* qkv, const void* out, const float* lse,
                                       const void* dout, void* dqkv, void* stream);

/* Norm over the last axis of x [rows, d].  stats: fp32 [2*rows] (mean, rstd; mean = 0 for
 * RMSNorm).  beta may be NULL (RMSNorm). */
jpp_status jpp_op_norm_fwd(int dtype, int norm, int rows, int d, float eps, const void* x,
                           const void* gamma, const void* beta, void* y, float* stats,
                           void* stream);
/* dx = (optional dx_add) + Norm'(dy); g_gamma += sum_rows dy*xhat; g_beta += sum_rows dy
 * (fp32, deterministic two-stage column reduction through `partial`, fp32 scratch of
 * jpp_op_colreduce_scratch(rows, d) elements). */
jpp_status jpp_op_norm_bwd(int dtype, int norm, int rows, int d, const void* x, const void* gamma,
                           const float* stats, const void* dy, const void* dx_add, void* dx,
                           float* g_gamma, float* g_beta, float* partial, void* stream);
size_t jpp_op_colreduce_scratch(int rows, int d);

/* a = act(h): h [rows, f] (GeLU) or [rows, 2f] (SwiGLU, gate | up), a [rows, f]. */
jpp_status jpp_op_act_fwd(int dtype, int act, int rows, int f, const void* h, void* a, void* stream);
/* dh = da * act'(h), shaped like h. */
jpp_status jpp_op_act_bwd(int dtype, int act, int rows, int f, const void* h, const void* da,
                          void* dh, void* stream);

/* Mean-token cross-entropy of the loss head from fp32 logits z [rows, vocab]: row_loss[r] =
 * log sum_v exp(z[r, v]) - z[r, targets[r]] (NaN for a target outside [0, vocab)), *loss =
 * mean of row_loss, dz = (softmax(z) - onehot(targets)) / rows in the storage dtype.  All
 * device pointers; deterministic. */
jpp_status jpp_op_cross_entropy(int dtype, int rows, int vocab, const float* z, const int32_t* targets, void* dz,
                                float* row_loss, float* loss, void* stream);

/* Token embedding.  x[t] = table[ids[t]] for t < rows (table [vocab, d], storage dtype; an id
 * outside [0, vocab) gives a zero row).  Backward: g_table[v] (fp32 [vocab, d]) += the sum of
 * dx[t] over the positions with ids[t] == v, in ascending t, one writer per row, no atomics;
 * rows <= 393216. */
jpp_status jpp_op_embed_fwd(int dtype, int rows, int d, int vocab, const int32_t* ids, const void* table, void* x,
                            void* stream);
jpp_status jpp_op_embed_bwd(int dtype, int rows, int d, int vocab, const int32_t* ids, const void* dx, float* g_table,
                            void* stream);

#ifdef __cplusplus
}
#endif
#endif /* JPP_H */
