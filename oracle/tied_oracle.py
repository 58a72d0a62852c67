"""CPU oracle for a model whose token embedding and LM head share one weight (tied
embeddings), trained through the gradient accumulation loop.

TEST INFRASTRUCTURE ONLY.  Plain float64 numpy; shares nothing with the HIP library.  Only
tests, the smoke check and the benchmark's CPU leg may import this module.

What it computes is a plain definition.  The model is

    a_0 = E[tokens_i]                      (row lookup in the table E [vocab, d_model])
    a_{s+1} = F_s(theta_s, a_s)            (the stages of oracle/stage_oracle.py)
    loss_i = CE(Norm(a_S) E^T, targets_i)  (the head of stage_oracle with w_head = E)

and the result of a step is the loss vector, every stage's gradient summed over the
microbatches without 1/M (Section 3.1) and the gradient of E.  E is used twice, so each
microbatch yields two partial gradients of it: g1_i through the lookup (row tokens[t] of g1
collects the cotangent of a_0 at position t; repeated tokens add up) and g2_i through the
head.  Section 3, "Weight Sharing and Gradient Accumulation", states the loop as written
by the user,

    g = sum_i (g1_i + g2_i)                                   (`uncommuted`)

and the rewrite that carries the partial gradients separately and adds them once after the
loop,

    g = (sum_i g1_i) + (sum_i g2_i)                           (`commuted`)

which is what lets each partial sum stay on the actor that produces it.  Both are returned;
they are equal up to the rounding order of the additions.  No schedule appears here: the
microbatches are taken one after the other through the whole model, which is what every
valid schedule computes.

Pinned by tests/test_tied_oracle_pins.py: the lookup's backward against a dense one-hot
product, the gradient of E against central finite differences of the summed loss (which
fails if either use of E is dropped), the two accumulation orders against each other
(bit-equal on integer-valued data), and the untied limit against oracle/pipeline_oracle.py.
"""
from dataclasses import replace

import numpy as np

from . import stage_oracle as so


def embed_forward(E, tokens):
    """tokens: int [mb, seq] -> [mb, seq, d]: row tokens[b, t] of E."""
    return E[tokens]


def embed_backward(vocab, tokens, dx):
    """Gradient of the lookup with respect to E: row v is the sum, in position order, of the
    cotangent rows dx[b, t] with tokens[b, t] == v."""
    d = dx.shape[-1]
    g = np.zeros((vocab, d), dtype=np.float64)
    flat = tokens.reshape(-1)
    rows = dx.reshape(-1, d)
    for t in range(flat.shape[0]):
        g[flat[t]] += rows[t]
    return g


def accumulate_uncommuted(g1s, g2s):
    """The loop as the user writes it: one carried total, every microbatch adds both partial
    gradients."""
    g = np.zeros_like(g1s[0])
    for g1, g2 in zip(g1s, g2s):
        g = g + (g1 + g2)
    return g


def accumulate_commuted(g1s, g2s):
    """After the loop-commuting rewrite: one carried state per use of the weight, one final
    addition."""
    a = np.zeros_like(g1s[0])
    b = np.zeros_like(g2s[0])
    for g1, g2 in zip(g1s, g2s):
        a = a + g1
        b = b + g2
    return a + b


def run_tied_model(spec, params_by_stage, E, tokens, targets):
    """spec: StageSpec of one stage (the last stage ends with the loss head whose w_head is
    E; params_by_stage[S-1]["head"] holds the head's norm parameters only).
    tokens[i], targets[i]: int [mb, seq].
    Returns dict: loss[i]; grads[s] (as stage_oracle, the last stage's head without w_head);
    g1[i], g2[i] (the partial gradients of E per microbatch); gE_uncommuted, gE_commuted."""
    S = len(params_by_stage)
    M = len(tokens)
    body = replace(spec, loss_head=False)
    last = replace(spec, loss_head=True)
    out = {"loss": [None] * M, "grads": {s: None for s in range(S)}, "g1": [], "g2": []}
    for i in range(M):
        a = embed_forward(E, tokens[i])
        caches = []
        for s in range(S):
            sp = last if s == S - 1 else body
            p = params_by_stage[s]
            if s == S - 1:
                p = {"layers": p["layers"], "head": dict(p["head"], w_head=E)}
            a, c = so.stage_forward(sp, p, a, targets[i] if s == S - 1 else None)
            caches.append((sp, p, c))
        out["loss"][i] = a
        cot = None
        for s in reversed(range(S)):
            sp, p, c = caches[s]
            cot, g = so.stage_backward(sp, p, c, cot)
            if s == S - 1:
                out["g2"].append(g["head"].pop("w_head"))
            out["grads"][s] = so._tree_add(out["grads"][s], g)
        out["g1"].append(embed_backward(E.shape[0], tokens[i], cot))
    out["gE_uncommuted"] = accumulate_uncommuted(out["g1"], out["g2"])
    out["gE_commuted"] = accumulate_commuted(out["g1"], out["g2"])
    return out


def total_loss(spec, params_by_stage, E, tokens, targets):
    """sum_i loss_i, forward only (for finite differences)."""
    S = len(params_by_stage)
    body = replace(spec, loss_head=False)
    last = replace(spec, loss_head=True)
    tot = 0.0
    for i in range(len(tokens)):
        a = embed_forward(E, tokens[i])
        for s in range(S):
            p = params_by_stage[s]
            if s == S - 1:
                p = {"layers": p["layers"], "head": dict(p["head"], w_head=E)}
                a, _ = so.stage_forward(last, p, a, targets[i])
            else:
                a, _ = so.stage_forward(body, p, a)
        tot += a
    return tot
