"""GPU parity of weight-gradient groups (jpp_layer_config.wgrad_group = g > 1): the backward
tasks of g consecutive microbatches of a stage keep their GEMM operands, and the task that
completes the group runs one weight-gradient GEMM per parameter over all g*T tokens.

What must hold: the sums are those of Section 3.1, so everything matches the fp64 oracle to
the usual tolerances; outputs and input cotangents are the bits of the ungrouped run (the
input-gradient chain is untouched); gradients are the same bits for every schedule that
keeps the per-stage backward order, because the association depends on the microbatch
indices alone; a group occupies its g stash places from its first forward to its last
backward.
"""
from dataclasses import replace

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import stage_oracle as so
from paper_2412_14374_amd import binding as B
from paper_2412_14374_amd import inputs as inp
from paper_2412_14374_amd.harness import Stage
from test_gpu_parity import FP32_VARIANTS, TOL, TWINS, compare, oracle_tasks, rel_l2, spec_of

pytestmark = pytest.mark.gpu


def grouped_peak(tasks, stage_ids, M, g):
    """Stash places in use at once when a group holds g places from its first forward to its
    last backward: brute force over the task list."""
    first, done, live, hi = set(), {}, 0, 0
    for (i, ty, s) in tasks:
        key = (s, i // g)
        if ty == B.JPP_FWD:
            if key not in first:
                first.add(key)
                live += g
            hi = max(hi, live)
        else:
            done[key] = done.get(key, 0) + 1
            if done[key] == min(g, M - (i // g) * g):
                live -= g
    assert live == 0
    return hi


def run_stage(w, params, x, cot, tg, tasks=None):
    st = Stage(w, tasks=tasks)
    st.set_params_host(params)
    st.bind(x, cot, tg)
    st.zero_grads()
    st.run()
    st.sync()
    torch.cuda.synchronize()
    return st


def draw(w, seed):
    spec = spec_of(w)
    return spec, inp.draw_stage_inputs(w, so.layer_param_shapes(spec),
                                       so.head_param_shapes(spec) if w.loss_head else None, seed=seed, perturb=True)


FP32_GROUPS = [("gpt-perturbed", 2), ("llama", 3), ("head", 2), ("gelu-tanh-ragged", 4), ("interleaved", 3)]


@pytest.mark.parametrize("name,g", FP32_GROUPS)
def test_fp32_groups_match_oracle(name, g):
    """Every executor path in fp32 storage with groups of g (3 with 4 microbatches: a full
    group and a ragged one; 4: the whole run is one group)."""
    w = replace(inp.C1, name="fp32-group-" + name, wgrad_group=g, **FP32_VARIANTS[name])
    spec, (params, x, cot, tg) = draw(w, seed=13)
    st = run_stage(w, params, x, cot, tg)
    got = st.results()
    ref = so.run_task_list(spec, params, oracle_tasks(st.tasks), x, cot, tg)
    worst, err = compare(w, got, ref)
    print(name, g, "worst", worst, err)
    assert err <= TOL[w.dtype], (worst, err)
    peak = grouped_peak(st.tasks, w.stage_ids, w.n_microbatches, g)
    assert B.jpp_schedule_validate(st.cfg, st.M, st.tasks) == peak
    assert B.jpp_stage_peak_in_flight(st.h) == peak
    st.close()


@pytest.mark.parametrize("name,g", [("C2", 2), ("C3", 4), ("C4", 4), ("C5", 2)])
def test_bf16_twin_groups_match_oracle_and_the_ungrouped_run(name, g):
    w = TWINS[name]
    if name == "C4":
        w = replace(w, P=2, rank=0)
    spec, (params, x, cot, tg) = draw(w, seed=7)
    runs = []
    for gg in (0, g):
        st = run_stage(replace(w, wgrad_group=gg), params, x, cot, tg)
        runs.append(([st.grads_tensor(v).cpu() for v in range(len(w.stage_ids))],
                     [t.cpu().clone() for t in st.out_y], [t.cpu().clone() for t in st.out_dx],
                     st.losses() if w.loss_head else None, st.results() if gg else None, list(st.tasks)))
        st.close()
    ref = so.run_task_list(spec, params, oracle_tasks(runs[1][5]), x, cot, tg)
    worst, err = compare(w, runs[1][4], ref)
    print(name, g, "worst", worst, err)
    assert err <= TOL[w.dtype], (worst, err)
    # the input-gradient chain, the outputs and the losses do not know about groups
    for k in (1, 2):
        for a, b in zip(runs[0][k], runs[1][k]):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    if w.loss_head:
        assert np.array_equal(runs[0][3], runs[1][3])
    # the gradients are the same sums in another association of fp32 additions
    for a, b in zip(runs[0][0], runs[1][0]):
        assert rel_l2(b.double().numpy(), a.double().numpy()) < 1e-5
        assert not torch.equal(a, b)


def test_grouped_gradients_bit_identical_across_schedules():
    """GPipe, 1F1B at every rank and a repeated run: with groups fixed by microbatch index
    the association is one and the same."""
    w = replace(TWINS["C2"], n_layers=2, wgrad_group=2)
    spec, (params, x, cot, tg) = draw(w, seed=3)
    s0 = w.stage_ids[0]
    M = w.n_microbatches
    lists = [B.jpp_schedule_make(inp.SCHED_GPIPE, 4, w.rank, 1, M)]
    lists += [B.jpp_schedule_make(inp.SCHED_1F1B, 4, r, 1, M) for r in range(4)]
    lists.append(lists[0])
    ref = None
    for tasks in lists:
        tasks = [(i, ty, s0) for (i, ty, _) in tasks]
        st = run_stage(w, params, x, cot, tg, tasks=tasks)
        g = st.grads_tensor(0).cpu()
        dxs = torch.stack([t.cpu() for t in st.out_dx])
        if ref is None:
            ref = (g, dxs)
        else:
            assert torch.equal(g.view(torch.int32), ref[0].view(torch.int32))
            assert torch.equal(dxs.view(torch.int16), ref[1].view(torch.int16))
        st.close()


def test_one_group_does_not_care_about_the_backward_order():
    """With the whole run in one group the weight gradients are one GEMM over the rows in
    microbatch-index order, whichever backward comes last: a reversed backward order gives
    the weight gradients' bits (norm gradients still add per task, in task order)."""
    w = replace(inp.C1, wgrad_group=inp.C1.n_microbatches)
    spec, (params, x, cot, tg) = draw(w, seed=17)
    s0, M = w.stage_ids[0], w.n_microbatches
    fwd = [(i, B.JPP_FWD, s0) for i in range(M)]
    orders = [fwd + [(i, B.JPP_BWD, s0) for i in range(M)], fwd + [(i, B.JPP_BWD, s0) for i in reversed(range(M))]]
    grads = []
    for tasks in orders:
        st = run_stage(w, params, x, cot, tg, tasks=tasks)
        grads.append(st.grads_tensor(0).cpu())
        info = st.info
        st.close()
    for name, shp, off in info:
        n = int(np.prod(shp))
        a, b = grads[0][off:off + n], grads[1][off:off + n]
        if len(shp) == 2 and shp[1] > 0 and name.split(".")[-1] in ("wqkv", "wo", "w1", "w2"):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32)), name
        else:
            assert rel_l2(b.double().numpy(), a.double().numpy()) < 1e-5, name


@pytest.mark.parametrize("name", ["C4", "C2"])
def test_full_size_groups_are_schedule_invariant(name):
    """The benchmark's configurations and launch paths (C4: one compute stream; C2: forward,
    input-gradient chain and weight gradients on three) with groups of 4 of 8 microbatches:
    the configuration's own schedule and all-forwards-then-all-backwards give identical bits,
    and equal the ungrouped run to fp32 rounding."""
    w = replace(inp.CONFIGS[name], n_microbatches=8, wgrad_group=4)
    M = w.n_microbatches
    inter = B.jpp_schedule_make(w.sched, w.P, w.rank, w.V, M)
    flat = [(i, B.JPP_FWD, s) for s in w.stage_ids for i in range(M)]
    flat += [(i, B.JPP_BWD, s) for s in reversed(w.stage_ids) for i in range(M)]
    outs = []
    for ww, lists in ((w, (inter, flat)), (replace(w, wgrad_group=0), (inter,))):
        st = Stage(ww, tasks=flat)
        st.set_params_random(seed=5)
        st.bind(seed=6)
        for tasks in lists:
            st.zero_grads()
            st.run(tasks)
            st.sync()
            outs.append(([st.grads_tensor(v).clone() for v in range(len(w.stage_ids))],
                         [t.clone() for t in st.out_dx]))
            torch.cuda.synchronize()
        st.close()
    for a, b in zip(outs[0][0], outs[1][0]):
        assert bool(torch.isfinite(a).all())
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    for a, b in zip(outs[0][1], outs[1][1]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    for a, c in zip(outs[0][0], outs[2][0]):
        num = float((a.double() - c.double()).norm())
        assert num / float(c.double().norm()) < 1e-5
    for a, c in zip(outs[0][1], outs[2][1]):
        assert torch.equal(a.view(torch.int16), c.view(torch.int16))


def test_group_configuration_errors():
    w = replace(inp.C1, wgrad_group=2)
    for bad in (replace(w, remat=1), replace(w, wgrad_group=w.n_microbatches + 1), replace(w, wgrad_group=-1)):
        with pytest.raises(B.JppError) as e:
            B.jpp_stage_arena_bytes(B.make_config(bad), bad.n_microbatches, 8)
        assert e.value.status == B.JPP_EINVAL
    with pytest.raises(B.JppError) as e:
        B.jpp_stage_arena_bytes(B.make_config(w), w.n_microbatches, 1)   # less than one group
    assert e.value.status == B.JPP_EINVAL
    # 1F1B at rank 0 of 2 keeps 2 stashes alive, with groups of 2 it keeps 2 groups = 4 places
    w = replace(inp.C1, wgrad_group=2, sched=inp.SCHED_1F1B, P=2, rank=0)
    spec, (params, x, cot, tg) = draw(w, seed=1)
    st = Stage(w, max_in_flight=2)
    st.set_params_host(params)
    st.bind(x, cot, tg)
    arr, n = B.tasks_array(st.tasks)
    with pytest.raises(B.JppError) as e:
        B.jpp_stage_run(st.h, arr, n, st.compute.cuda_stream, st.side.cuda_stream)
    assert e.value.status == B.JPP_ECAPACITY
    st.close()


@pytest.mark.parametrize("name,g", [("gpt-fp32-loss-interleaved", 2), ("gpt-fp32-cot-1f1b", 3),
                                    ("gpt-bf16-loss-interleaved", 4)])
def test_pipeline_with_groups_matches_oracle(name, g):
    """Several actors on one device, every one with weight-gradient groups: a task of one
    actor may complete a group while its neighbour still prefetches; losses, input cotangents
    and every stage's gradients against the pipeline oracle."""
    import test_gpu_pipeline as tp
    w, lists = tp.PIPES[name]
    w = replace(w, wgrad_group=g)
    pipe, got, ref = tp.run_both(w, lists)
    worst = tp.worst_error(w, got, ref)
    for r, a in enumerate(pipe.actors):
        own = [(i, B.JPP_FWD if ty == "fwd" else B.JPP_BWD, s) for (i, ty, s) in lists[r]]
        assert B.jpp_stage_peak_in_flight(a.h) == grouped_peak(own, None, w.n_microbatches, g)
    pipe.close()
    assert worst[1] < tp.TOL[w.dtype], worst
