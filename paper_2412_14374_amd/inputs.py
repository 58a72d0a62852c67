"""Workload descriptions and seeded synthetic inputs.

This module is shared by the tests, the benchmark and the smoke check, and
feeds the SAME host arrays to the CPU oracle and to the HIP library.  It holds
no arithmetic of the method: only shapes, random draws and rounding of the
drawn values to the storage type.

The paper's Evaluation section trains GPT-3 175B (sequence 2048, 32
microbatches, 8 pipeline ranks, interleaved 1F1B) and Llama2 70B (sequence
4096, 16 microbatches, 4 pipeline ranks) in BF16 on text data that is not
available here; throughput and parity depend only on shapes and value
distributions, so normal/uniform synthetic tensors of those shapes stand in.
"""
from dataclasses import dataclass, field, asdict, replace
import numpy as np

SEED = 20241214

NORM_LAYERNORM, NORM_RMSNORM = 0, 1
ACT_GELU, ACT_GELU_TANH, ACT_SWIGLU = 0, 1, 2
DT_F32, DT_BF16 = 0, 1
SCHED_GPIPE, SCHED_1F1B, SCHED_INTERLEAVED = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: int
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    seq_len: int
    microbatch: int
    n_microbatches: int
    norm: int = NORM_LAYERNORM
    act: int = ACT_GELU
    use_bias: int = 1
    rope: int = 0
    rope_theta: float = 10000.0
    norm_eps: float = 1e-5
    loss_head: int = 0
    vocab: int = 0
    remat: int = 0                   # 1: keep only each layer's input, recompute in the backward
    wgrad_group: int = 0             # g > 1: one weight-gradient GEMM per group of g microbatches
    embed: int = 0                   # 1: the first stage starts with a token embedding [vocab, d_model]
    # schedule: kind, pipeline depth P, this actor's rank, virtual stages V
    sched: int = SCHED_GPIPE
    P: int = 1
    rank: int = 0
    V: int = 1
    # value distributions
    w_std: float = 0.02
    cot_std: float = 1e-2
    scale_out_proj: bool = False     # Wo, W2 ~ N(0, w_std / sqrt(2 * n_layers))

    @property
    def stage_ids(self):
        return [v * self.P + self.rank for v in range(self.V)]

    @property
    def tokens(self):
        return self.microbatch * self.seq_len


# The five benchmark configurations.
C1 = Workload("C1-tiny-gpt-fp32-gpipe", DT_F32, 2, 128, 4, 4, 32, 512, 64, 2, 4,
              sched=SCHED_GPIPE, P=1, rank=0, cot_std=1.0, scale_out_proj=True)
C2 = Workload("C2-gpt-d2048-bf16-1f1b", DT_BF16, 4, 2048, 16, 16, 128, 8192, 2048, 4, 8,
              sched=SCHED_1F1B, P=4, rank=0)
C3 = Workload("C3-llama-d8192-gqa-bf16-1f1b", DT_BF16, 2, 8192, 64, 8, 128, 28672, 4096, 1, 16,
              norm=NORM_RMSNORM, act=ACT_SWIGLU, use_bias=0, rope=1,
              sched=SCHED_1F1B, P=4, rank=0)
C4 = Workload("C4-gpt3-175b-stage-bf16-interleaved", DT_BF16, 1, 12288, 96, 96, 128, 49152, 2048, 1, 32,
              sched=SCHED_INTERLEAVED, P=8, rank=0, V=2)
C5 = Workload("C5-last-stage-loss-bf16-1f1b", DT_BF16, 2, 4096, 32, 32, 128, 16384, 2048, 2, 16,
              loss_head=1, vocab=50304, sched=SCHED_1F1B, P=4, rank=3)

CONFIGS = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}


def shrunk_twin(w, d_model, seq_len, d_ffn=None, vocab=None, n_q_heads=None, n_microbatches=None):
    """Same structure (head_dim, GQA ratio, norm/act/rope/bias, schedule) at a
    size the CPU oracle finishes in seconds."""
    ratio = w.n_q_heads // w.n_kv_heads
    hq = n_q_heads if n_q_heads is not None else max(ratio, d_model // w.head_dim)
    return replace(w, name=w.name + "-twin", d_model=d_model, seq_len=seq_len,
                   d_ffn=d_ffn if d_ffn is not None else 4 * d_model,
                   n_q_heads=hq, n_kv_heads=hq // ratio,
                   vocab=(vocab if vocab is not None else w.vocab),
                   n_microbatches=n_microbatches if n_microbatches is not None else w.n_microbatches)


def round_to_dtype(a, dtype):
    """Round float64 values to the storage grid (fp32, or bf16 with
    round-to-nearest-even) and return them as float64."""
    if dtype == DT_F32:
        return a.astype(np.float32).astype(np.float64)
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.to(torch.float64).numpy()


def draw_params(shapes, rng, w, perturb=False):
    """shapes: list of (name, shape) for one layer or the loss head.
    Norm gains are 1, norm offsets and biases 0, matrices ~ N(0, w_std); with
    perturb=True the gains/offsets/biases get random values too (test-only, so
    that a misapplied bias or gain cannot hide behind its zero/one value)."""
    out = {}
    for name, shape in shapes:
        if len(shape) == 2:
            std = w.w_std
            if w.scale_out_proj and name in ("wo", "w2"):
                std = w.w_std / np.sqrt(2.0 * w.n_layers)
            a = rng.standard_normal(shape) * std
        elif name.endswith("_g"):
            a = np.ones(shape)
            if perturb:
                a = a + 0.1 * rng.standard_normal(shape)
        else:
            a = np.zeros(shape)
            if perturb:
                a = 0.05 * rng.standard_normal(shape)
        out[name] = round_to_dtype(a, w.dtype)
    return out


def draw_stage_inputs(w, layer_shapes, head_shapes=None, seed=SEED, perturb=False):
    """Draw everything one actor needs, in a fixed order: per owned stage the
    parameters (layer by layer, then the head), then x_0..x_{M-1}, then
    c_0..c_{M-1}; finally the targets.  Returns
    (params_by_stage, x, cot, targets) with float64 arrays already rounded to
    the storage type."""
    rng = np.random.default_rng(seed)
    M = w.n_microbatches
    shp = (w.microbatch, w.seq_len, w.d_model)
    params, x, cot = {}, {}, {}
    for s in w.stage_ids:
        p = {"layers": [draw_params(layer_shapes, rng, w, perturb) for _ in range(w.n_layers)]}
        if w.loss_head:
            p["head"] = draw_params(head_shapes, rng, w, perturb)
        params[s] = p
        x[s] = [round_to_dtype(rng.standard_normal(shp), w.dtype) for _ in range(M)]
        cot[s] = [round_to_dtype(rng.standard_normal(shp) * w.cot_std, w.dtype) for _ in range(M)]
    targets = None
    if w.loss_head:
        targets = [rng.integers(0, w.vocab, size=(w.microbatch, w.seq_len)).astype(np.int32)
                   for _ in range(M)]
    return params, x, cot, targets


def draw_pipeline_inputs(w, n_stages, layer_shapes, head_shapes=None, seed=SEED, perturb=False):
    """Draw what a whole pipeline of `n_stages` stages needs, in a fixed order: per stage the
    parameters (layer by layer; the head on the last stage if w.loss_head), then the inputs
    x_0..x_{M-1} of stage 0, then either the targets (loss head) or the cotangents
    c_0..c_{M-1} of the last stage's output.  Returns (params_by_stage, x0, cot_last, targets)
    with float64 arrays already rounded to the storage type."""
    rng = np.random.default_rng(seed)
    M = w.n_microbatches
    shp = (w.microbatch, w.seq_len, w.d_model)
    params = {}
    for s in range(n_stages):
        p = {"layers": [draw_params(layer_shapes, rng, w, perturb) for _ in range(w.n_layers)]}
        if w.loss_head and s == n_stages - 1:
            p["head"] = draw_params(head_shapes, rng, w, perturb)
        params[s] = p
    x0 = [round_to_dtype(rng.standard_normal(shp), w.dtype) for _ in range(M)]
    cot_last, targets = None, None
    if w.loss_head:
        targets = [rng.integers(0, w.vocab, size=(w.microbatch, w.seq_len)).astype(np.int32) for _ in range(M)]
    else:
        cot_last = [round_to_dtype(rng.standard_normal(shp) * w.cot_std, w.dtype) for _ in range(M)]
    return params, x0, cot_last, targets


def draw_tied_inputs(w, n_stages, layer_shapes, head_shapes, seed=SEED, perturb=False, distinct_ids=None):
    """Draw what a pipeline with a tied embedding / LM head needs, in a fixed order: per stage
    the layer parameters, the head's norm parameters (head_shapes without w_head), the shared
    table E [vocab, d_model], then token ids and targets per microbatch.  `distinct_ids`
    limits the ids to that many values, so that positions collide in the table's gradient
    (natural text repeats tokens; a uniform draw over a large vocabulary would not).
    Returns (params_by_stage, E, tokens, targets), floats already on the storage grid."""
    rng = np.random.default_rng(seed)
    M = w.n_microbatches
    params = {}
    for s in range(n_stages):
        params[s] = {"layers": [draw_params(layer_shapes, rng, w, perturb) for _ in range(w.n_layers)]}
    params[n_stages - 1]["head"] = draw_params([(k, shp) for k, shp in head_shapes if k != "w_head"], rng, w, perturb)
    E = round_to_dtype(rng.standard_normal((w.vocab, w.d_model)) * w.w_std, w.dtype)
    hi = w.vocab if distinct_ids is None else min(w.vocab, distinct_ids)
    ids = rng.permutation(w.vocab)[:hi]
    tokens = [ids[rng.integers(0, hi, size=(w.microbatch, w.seq_len))].astype(np.int32) for _ in range(M)]
    targets = [rng.integers(0, w.vocab, size=(w.microbatch, w.seq_len)).astype(np.int32) for _ in range(M)]
    return params, E, tokens, targets
