"""Pins for oracle/pipeline_oracle.py (several actors, one task list each): checked against
the single deep stage of oracle/stage_oracle.py (itself pinned by finite differences and
closed forms), a finite difference through the whole pipeline, the example printed in the
paper's Section 4.2, bitwise schedule invariance and hand-made deadlocks.  CPU only; nothing
here touches the HIP path.
"""
import os
from dataclasses import replace

import numpy as np
import pytest

from oracle import pipeline_oracle as po
from oracle import schedules as sch
from oracle import stage_oracle as so
from paper_2412_14374_amd import inputs as inp


def workload(head, **kw):
    base = dict(name="tiny-pipe", dtype=inp.DT_F32, n_layers=1, d_model=16, n_q_heads=2, n_kv_heads=2,
                head_dim=8, d_ffn=32, seq_len=8, microbatch=2, n_microbatches=4, cot_std=1.0, w_std=0.3)
    if head:
        base.update(loss_head=1, vocab=29)
    base.update(kw)
    return inp.Workload(**base)


def spec_of(w):
    return so.StageSpec(n_layers=w.n_layers, d_model=w.d_model, n_q_heads=w.n_q_heads,
                        n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, d_ffn=w.d_ffn,
                        seq_len=w.seq_len, microbatch=w.microbatch, norm=w.norm, act=w.act,
                        use_bias=bool(w.use_bias), rope=bool(w.rope), rope_theta=w.rope_theta,
                        norm_eps=w.norm_eps, loss_head=bool(w.loss_head), vocab=w.vocab)


def draw(w, S, seed=3):
    spec = spec_of(w)
    return (spec,) + inp.draw_pipeline_inputs(w, S, so.layer_param_shapes(spec),
                                              so.head_param_shapes(spec) if w.loss_head else None,
                                              seed=seed, perturb=True)


def interleaved_lists(P, V, M):
    return [sch.interleaved_1f1b(P, r, V, M) for r in range(P)]


def flat_lists(P, V, M):
    """Every actor: all forwards of its stages in ascending stage order, then all backwards
    in descending stage order (GPipe on a circular placement)."""
    out = []
    for r in range(P):
        st = [v * P + r for v in range(V)]
        out.append([(i, "fwd", s) for s in st for i in range(M)] +
                   [(i, "bwd", s) for s in reversed(st) for i in range(M)])
    return out


@pytest.mark.parametrize("head", [False, True])
def test_pipeline_equals_one_deep_stage(head):
    """S stages of L layers chained through the actors' hand-offs are the same function as
    one stage of S*L layers: outputs, input cotangents and summed gradients must agree."""
    P, V, M = 2, 2, 4
    S = P * V
    w = workload(head, n_layers=2)
    spec, params, x0, cot_last, tg = draw(w, S)
    res = po.run_pipeline(spec, params, interleaved_lists(P, V, M), x0, tg, cot_last)
    deep_spec = replace(spec, n_layers=S * w.n_layers)
    deep = {"layers": [l for s in range(S) for l in params[s]["layers"]]}
    if head:
        deep["head"] = params[S - 1]["head"]
    acc = None
    for i in range(M):
        out, cache = so.stage_forward(deep_spec, deep, x0[i], tg[i] if head else None)
        if head:
            assert abs(out - res["loss"][i]) <= 1e-12 * abs(out)
        else:
            np.testing.assert_allclose(res["y"][i], out, rtol=1e-12, atol=1e-13)
        dx, g = so.stage_backward(deep_spec, deep, cache, None if head else cot_last[i])
        np.testing.assert_allclose(res["dx"][i], dx, rtol=1e-11, atol=1e-13)
        acc = so._tree_add(acc, g)
    for s in range(S):
        for li in range(w.n_layers):
            for k, v in acc["layers"][s * w.n_layers + li].items():
                np.testing.assert_allclose(res["grads"][s]["layers"][li][k], v, rtol=1e-11, atol=1e-13)
    if head:
        for k, v in acc["head"].items():
            np.testing.assert_allclose(res["grads"][S - 1]["head"][k], v, rtol=1e-11, atol=1e-13)


def test_finite_difference_through_the_whole_pipeline():
    """d(sum_i loss_i)/d(theta of stage 0) by central differences: the gradient must have
    crossed every hand-off, and must be the plain sum over microbatches."""
    P, V, M = 2, 2, 2
    S = P * V
    w = workload(True, n_microbatches=M)
    spec, params, x0, _, tg = draw(w, S)
    lists = interleaved_lists(P, V, M)
    res = po.run_pipeline(spec, params, lists, x0, tg)

    def total():
        return sum(po.run_pipeline(spec, params, lists, x0, tg)["loss"])

    rng = np.random.default_rng(0)
    for s, name in ((0, "wqkv"), (0, "b2"), (1, "w1"), (3, "ln1_g")):
        a = params[s]["layers"][0][name]
        idx = tuple(rng.integers(0, n) for n in a.shape)
        old = a[idx]
        h = 1e-5
        a[idx] = old + h
        up = total()
        a[idx] = old - h
        dn = total()
        a[idx] = old
        fd = (up - dn) / (2 * h)
        an = res["grads"][s]["layers"][0][name][idx]
        assert abs(fd - an) <= 2e-6 * max(abs(an), abs(fd)) + 2e-7, (s, name, fd, an)


def test_results_do_not_depend_on_the_schedule_bitwise():
    """Section 2.2.1: schedules only reorder.  Interleaved 1F1B, all-forward-then-all-backward
    and (V = 1) plain 1F1B give the same bits; each actor's stash peak is the one its own
    list implies."""
    P, V, M = 2, 2, 4
    S = P * V
    w = workload(True)
    spec, params, x0, _, tg = draw(w, S)
    a = po.run_pipeline(spec, params, interleaved_lists(P, V, M), x0, tg)
    b = po.run_pipeline(spec, params, flat_lists(P, V, M), x0, tg)
    assert a["loss"] == b["loss"]
    for s in range(S):
        for k, v in a["grads"][s]["layers"][0].items():
            assert np.array_equal(v, b["grads"][s]["layers"][0][k])
    for i in range(M):
        assert np.array_equal(a["dx"][i], b["dx"][i])
    for r in range(P):
        assert a["peak_live"][r] == sch.validate(interleaved_lists(P, V, M)[r], [v * P + r for v in range(V)], M)
        assert b["peak_live"][r] == M * V
    # V = 1: 1F1B on 4 actors against GPipe on 4 actors
    P1 = 4
    c = po.run_pipeline(spec, params, [sch.one_f_one_b(P1, r, M) for r in range(P1)], x0, tg)
    d = po.run_pipeline(spec, params, [[(i, ty, r) for (i, ty, _) in sch.gpipe(P1, r, M)] for r in range(P1)], x0, tg)
    assert c["loss"] == d["loss"] == a["loss"]
    for s in range(S):
        for k, v in a["grads"][s]["layers"][0].items():
            assert np.array_equal(v, c["grads"][s]["layers"][0][k])
            assert np.array_equal(v, d["grads"][s]["layers"][0][k])
    assert c["peak_live"] == [min(P1 - r, M) for r in range(P1)]


def test_the_paper_example_runs_in_a_topological_order():
    """The two-actor, four-stage lists of Section 4.2 (their printed beginning is the golden
    file) merge into one order in which every task follows its producer."""
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_sec4_2_task_lists.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, i, ty, s = line.split()
            rows.append((int(a), (int(i), ty, int(s))))
    P, V, M = 2, 2, 4
    lists = interleaved_lists(P, V, M)
    for r in range(P):
        assert lists[r][:3] == [t for (a, t) in rows if a == r]
    order = po.global_order(lists, P * V)
    assert len(order) == sum(len(l) for l in lists)
    pos = {t: k for k, (_, t) in enumerate(order)}
    for r, t in order:
        assert po.actor_of(t[2], P) == r
        need = po.producer_of(t, P * V)
        if need is not None:
            assert pos[need] < pos[t]
    for r in range(P):      # every actor's own order is kept
        own = [t for (a, t) in order if a == r]
        assert own == lists[r]


def test_deadlock_is_reported():
    """Lists that are each valid for their actor but wait for each other in a cycle."""
    P, V, M = 2, 2, 1
    lists = flat_lists(P, V, M)
    assert len(po.global_order(lists, 4)) == 8
    # actor 0 wants stage 2 (fed by actor 1's stage 1, fed by actor 0's stage 0) before stage 0
    bad0 = [(0, "fwd", 2), (0, "fwd", 0), (0, "bwd", 2), (0, "bwd", 0)]
    for r, lst in enumerate((bad0, lists[1])):
        sch.validate(lst, [v * P + r for v in range(V)], M)     # locally fine
    with pytest.raises(po.Deadlock):
        po.global_order([bad0, lists[1]], 4)
    # backward side: actor 1 wants bwd of stage 1 before bwd of stage 3
    bad1 = [(0, "fwd", 1), (0, "fwd", 3), (0, "bwd", 1), (0, "bwd", 3)]
    with pytest.raises(po.Deadlock):
        po.global_order([lists[0], bad1], 4)


def test_producers():
    assert po.producer_of((3, "fwd", 0), 4) is None
    assert po.producer_of((3, "fwd", 2), 4) == (3, "fwd", 1)
    assert po.producer_of((3, "bwd", 3), 4) is None
    assert po.producer_of((3, "bwd", 1), 4) == (3, "bwd", 2)
