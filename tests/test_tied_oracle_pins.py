"""Pins of oracle/tied_oracle.py (CPU only): a tied embedding / LM head through the
gradient accumulation loop, and the loop-commuting rewrite of Section 3, "Weight Sharing
and Gradient Accumulation"."""
import numpy as np
import pytest

from oracle import pipeline_oracle as po
from oracle import stage_oracle as so
from oracle import tied_oracle as to


def tiny(seed=0, S=2, M=3, vocab=11, repeat_tokens=True):
    spec = so.StageSpec(n_layers=1, d_model=8, n_q_heads=2, n_kv_heads=1, head_dim=4, d_ffn=12, seq_len=5,
                        microbatch=2, loss_head=True, vocab=vocab)
    rng = np.random.default_rng(seed)
    params = {}
    for s in range(S):
        params[s] = {"layers": [{k: rng.standard_normal(shp) * 0.3 for k, shp in so.layer_param_shapes(spec)}]}
    params[S - 1]["head"] = {k: 1.0 + 0.1 * rng.standard_normal(shp) for k, shp in so.head_param_shapes(spec)
                             if k != "w_head"}
    E = rng.standard_normal((vocab, spec.d_model)) * 0.5
    hi = 4 if repeat_tokens else vocab      # few distinct ids: positions collide in the lookup's backward
    tokens = [rng.integers(0, hi, size=(spec.microbatch, spec.seq_len)) for _ in range(M)]
    targets = [rng.integers(0, vocab, size=(spec.microbatch, spec.seq_len)) for _ in range(M)]
    return spec, params, E, tokens, targets


def test_lookup_backward_is_the_one_hot_product():
    rng = np.random.default_rng(1)
    vocab, d = 7, 5
    tokens = rng.integers(0, vocab, size=(3, 6))
    dx = rng.standard_normal((3, 6, d))
    onehot = np.zeros((tokens.size, vocab))
    onehot[np.arange(tokens.size), tokens.reshape(-1)] = 1.0
    want = onehot.T @ dx.reshape(-1, d)
    got = to.embed_backward(vocab, tokens, dx)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    # rows of ids that do not occur stay zero; distinct ids just move rows
    assert np.all(got[np.setdiff1d(np.arange(vocab), tokens)] == 0.0)
    perm = rng.permutation(vocab)[:6].reshape(1, 6)
    g = to.embed_backward(vocab, perm, dx[:1])
    assert np.array_equal(g[perm[0]], dx[0])
    # the lookup itself
    E = rng.standard_normal((vocab, d))
    assert np.array_equal(to.embed_forward(E, tokens)[2, 4], E[tokens[2, 4]])


def test_gradient_of_the_shared_table_matches_finite_differences():
    """Both uses of E contribute: the check fails if the lookup's or the head's partial
    gradient is dropped (the second assert shows each alone is far off)."""
    spec, params, E, tokens, targets = tiny(seed=2)
    ref = to.run_tied_model(spec, params, E, tokens, targets)
    g = ref["gE_uncommuted"]
    rng = np.random.default_rng(3)
    eps = 1e-6
    picks = [(int(tokens[0][0, 0]), 1), (int(tokens[1][1, 2]), 5), (int(targets[0][0, 1]), 0)]
    picks += [(int(rng.integers(0, E.shape[0])), int(rng.integers(0, E.shape[1]))) for _ in range(5)]
    for (v, j) in picks:
        Ep, Em = E.copy(), E.copy()
        Ep[v, j] += eps
        Em[v, j] -= eps
        fd = (to.total_loss(spec, params, Ep, tokens, targets) - to.total_loss(spec, params, Em, tokens, targets)) / (2 * eps)
        assert abs(fd - g[v, j]) <= 1e-6 * max(1.0, abs(fd)), (v, j, fd, g[v, j])
    g1 = sum(ref["g1"])
    g2 = sum(ref["g2"])
    used = np.unique(np.concatenate([t.reshape(-1) for t in tokens]))
    assert np.linalg.norm(g1[used]) > 1e-3 * np.linalg.norm(g[used])
    assert np.linalg.norm(g2) > 1e-3 * np.linalg.norm(g)
    assert np.linalg.norm(g - g1) > 1e-3 * np.linalg.norm(g) and np.linalg.norm(g - g2) > 1e-3 * np.linalg.norm(g)


def test_commuted_and_uncommuted_accumulation_agree():
    """The rewrite rule: sum_i (g1_i + g2_i) = (sum_i g1_i) + (sum_i g2_i).  Bit-equal when
    every partial sum is exact (integer-valued data), equal to rounding otherwise."""
    rng = np.random.default_rng(4)
    g1s = [rng.integers(-50, 50, size=(6, 4)).astype(np.float64) for _ in range(9)]
    g2s = [rng.integers(-50, 50, size=(6, 4)).astype(np.float64) for _ in range(9)]
    assert np.array_equal(to.accumulate_uncommuted(g1s, g2s), to.accumulate_commuted(g1s, g2s))
    assert np.array_equal(to.accumulate_commuted(g1s, g2s), sum(g1s) + sum(g2s))
    spec, params, E, tokens, targets = tiny(seed=5)
    ref = to.run_tied_model(spec, params, E, tokens, targets)
    a, b = ref["gE_uncommuted"], ref["gE_commuted"]
    assert np.linalg.norm(a - b) <= 1e-14 * np.linalg.norm(a)
    # one microbatch: nothing to commute
    one = to.run_tied_model(spec, params, E, tokens[:1], targets[:1])
    assert np.array_equal(one["gE_uncommuted"], one["gE_commuted"])


def test_untied_limit_is_the_pipeline_oracle():
    """With the lookup done by hand and the head's weight a separate parameter the same
    numbers must come out of oracle/pipeline_oracle.py: losses, stage gradients, the head's
    weight gradient (= sum of g2) and the cotangent of the embedded input (whose scatter is
    g1)."""
    spec, params, E, tokens, targets = tiny(seed=6, S=3, M=2)
    ref = to.run_tied_model(spec, params, E, tokens, targets)
    S = len(params)
    pp = {s: {"layers": params[s]["layers"]} for s in range(S)}
    pp[S - 1]["head"] = dict(params[S - 1]["head"], w_head=E.copy())
    x0 = [to.embed_forward(E, t) for t in tokens]
    lists = [[(i, "fwd", s) for i in range(len(tokens))] + [(i, "bwd", s) for i in range(len(tokens))] for s in range(S)]
    pipe = po.run_pipeline(spec, pp, lists, x0, targets=targets)
    for i in range(len(tokens)):
        assert abs(pipe["loss"][i] - ref["loss"][i]) <= 1e-13 * abs(ref["loss"][i])
        g1 = to.embed_backward(E.shape[0], tokens[i], pipe["dx"][i])
        assert np.allclose(g1, ref["g1"][i], rtol=1e-12, atol=1e-14)
    assert np.allclose(pipe["grads"][S - 1]["head"]["w_head"], sum(ref["g2"]), rtol=1e-12, atol=1e-14)
    for s in range(S):
        for la, lb in zip(pipe["grads"][s]["layers"], ref["grads"][s]["layers"]):
            for k in la:
                assert np.allclose(la[k], lb[k], rtol=1e-12, atol=1e-14), (s, k)
    assert "w_head" not in ref["grads"][S - 1]["head"]
