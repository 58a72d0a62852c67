"""GPU parity of a whole pipeline (several actors on one device, real stage-to-stage
hand-offs) against oracle/pipeline_oracle.py, through the C ABI.  Same tolerances as the
single-stage tests: 1e-5 (fp32 storage), 2e-2 (bf16 storage), relative L2 per tensor.
"""
from dataclasses import replace

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pipeline_oracle as po
from oracle import schedules as osch
from oracle import stage_oracle as so
from paper_2412_14374_amd import binding as B
from paper_2412_14374_amd import inputs as inp
from paper_2412_14374_amd.harness import Pipeline

pytestmark = pytest.mark.gpu

TOL = {inp.DT_F32: 1e-5, inp.DT_BF16: 2e-2}


def spec_of(w):
    return so.StageSpec(n_layers=w.n_layers, d_model=w.d_model, n_q_heads=w.n_q_heads,
                        n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, d_ffn=w.d_ffn,
                        seq_len=w.seq_len, microbatch=w.microbatch, norm=w.norm, act=w.act,
                        use_bias=bool(w.use_bias), rope=bool(w.rope), rope_theta=w.rope_theta,
                        norm_eps=w.norm_eps, loss_head=bool(w.loss_head), vocab=w.vocab)


def rel_l2(a, b):
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a)


def interleaved(P, V, M):
    return [osch.interleaved_1f1b(P, r, V, M) for r in range(P)]


def flat(P, V, M):
    out = []
    for r in range(P):
        st = [v * P + r for v in range(V)]
        out.append([(i, "fwd", s) for s in st for i in range(M)] +
                   [(i, "bwd", s) for s in reversed(st) for i in range(M)])
    return out


def one_f_one_b(P, M):
    return [osch.one_f_one_b(P, r, M) for r in range(P)]


PIPES = {
    # small GPT pipeline in fp32 ending in the loss: 2 actors x 2 virtual stages
    "gpt-fp32-loss-interleaved": (inp.Workload("p1", inp.DT_F32, 1, 64, 2, 2, 32, 128, 32, 2, 4, loss_head=1,
                                               vocab=96, w_std=0.1, P=2, V=2, sched=inp.SCHED_INTERLEAVED),
                                  interleaved(2, 2, 4)),
    # three actors, one stage each, two layers per stage, no loss head: outer cotangents
    "gpt-fp32-cot-1f1b": (inp.Workload("p2", inp.DT_F32, 2, 64, 2, 2, 32, 128, 24, 1, 5, w_std=0.1, cot_std=1.0,
                                       P=3, V=1, sched=inp.SCHED_1F1B),
                          one_f_one_b(3, 5)),
    # Llama-style layers (RMSNorm, SwiGLU, RoPE, GQA, no biases)
    "llama-fp32-loss-interleaved": (inp.Workload("p3", inp.DT_F32, 1, 64, 4, 2, 16, 96, 32, 1, 4, norm=inp.NORM_RMSNORM,
                                                 act=inp.ACT_SWIGLU, use_bias=0, rope=1, loss_head=1, vocab=64,
                                                 w_std=0.1, P=2, V=2, sched=inp.SCHED_INTERLEAVED),
                                    interleaved(2, 2, 4)),
    # bf16 storage, MFMA kernels (head_dim 128), 2 actors x 2 virtual stages, loss head
    "gpt-bf16-loss-interleaved": (inp.Workload("p4", inp.DT_BF16, 1, 256, 2, 2, 128, 512, 136, 1, 4, loss_head=1,
                                               vocab=520, P=2, V=2, sched=inp.SCHED_INTERLEAVED),
                                  interleaved(2, 2, 4)),
}


def run_both(w, lists, seed=11):
    spec = spec_of(w)
    S = w.P * w.V
    params, x0, cot_last, tg = inp.draw_pipeline_inputs(
        w, S, so.layer_param_shapes(spec), so.head_param_shapes(spec) if w.loss_head else None,
        seed=seed, perturb=True)
    pipe = Pipeline(w, [[(i, ty, s) for (i, ty, s) in l] for l in lists])
    pipe.set_params_host(params)
    pipe.bind(x0, cot_last, tg)
    pipe.zero_grads()
    pipe.run()
    got = pipe.results()
    ref = po.run_pipeline(spec, params, lists, x0, tg, cot_last)
    return pipe, got, ref


def worst_error(w, got, ref):
    worst = ("", 0.0)

    def upd(name, a, b):
        nonlocal worst
        a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
        assert a.shape == b.shape, name
        assert np.all(np.isfinite(a)), name
        e = rel_l2(a, b)
        if e > worst[1]:
            worst = (name, e)

    M, S = w.n_microbatches, w.P * w.V
    for i in range(M):
        if w.loss_head:
            upd(f"loss[{i}]", got["loss"][i], ref["loss"][i])
        else:
            upd(f"y[{i}]", got["y"][i], ref["y"][i])
        upd(f"dx[{i}]", got["dx"][i], ref["dx"][i])
    for s in range(S):
        for li, lg in enumerate(ref["grads"][s]["layers"]):
            for k, v in lg.items():
                upd(f"G[{s}].layer{li}.{k}", got["grads"][s]["layers"][li][k], v)
        if "head" in ref["grads"][s]:
            for k, v in ref["grads"][s]["head"].items():
                upd(f"G[{s}].head.{k}", got["grads"][s]["head"][k], v)
    return worst


@pytest.mark.parametrize("name", sorted(PIPES))
def test_pipeline_matches_oracle(name):
    w, lists = PIPES[name]
    pipe, got, ref = run_both(w, lists)
    worst = worst_error(w, got, ref)
    for r, a in enumerate(pipe.actors):
        assert B.jpp_stage_peak_in_flight(a.h) == ref["peak_live"][r]
    pipe.close()
    assert worst[1] < TOL[w.dtype], worst


def test_pipeline_bits_do_not_depend_on_the_schedule_or_the_run():
    """Section 2.2.1: interleaved 1F1B and all-forward-then-all-backward only reorder the
    tasks; with the per-stage backward order kept the accumulated gradients, the losses and
    the input cotangents are identical bit for bit, also when the run is repeated."""
    w, lists = PIPES["gpt-bf16-loss-interleaved"]
    spec = spec_of(w)
    S = w.P * w.V
    params, x0, _, tg = inp.draw_pipeline_inputs(w, S, so.layer_param_shapes(spec), so.head_param_shapes(spec), seed=5)
    flat_lists = flat(w.P, w.V, w.n_microbatches)
    pipe = Pipeline(w, flat_lists)          # sized for the list that keeps most stashes alive
    pipe.set_params_host(params)
    pipe.bind(x0, None, tg)
    ref = None
    for lst in (lists, flat_lists, lists):
        pipe.zero_grads()
        pipe.run(lst)
        pipe.sync()
        torch.cuda.synchronize()
        g = [a.grads_tensor(v).cpu() for a in pipe.actors for v in range(w.V)]
        l = pipe.actors[-1].losses()
        dx = [t.cpu().clone() for t in pipe.dx_out]
        if ref is None:
            ref = (g, l, dx)
            continue
        for a, b in zip(g, ref[0]):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32))
        assert np.array_equal(l, ref[1])
        for a, b in zip(dx, ref[2]):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # a second run without zeroing adds the same gradients again (Section 3.1)
    pipe.run(lists)
    pipe.sync()
    g2 = [a.grads_tensor(v).cpu() for a in pipe.actors for v in range(w.V)]
    for a, b in zip(g2, ref[0]):
        assert rel_l2(a.double().numpy(), 2 * b.double().numpy()) < 1e-6
    pipe.close()


def test_pipeline_deadlock_and_bad_arguments_are_refused_before_anything_runs():
    w, lists = PIPES["gpt-fp32-loss-interleaved"]
    spec = spec_of(w)
    S, M = w.P * w.V, w.n_microbatches
    params, x0, _, tg = inp.draw_pipeline_inputs(w, S, so.layer_param_shapes(spec), so.head_param_shapes(spec), seed=2)
    good = flat(w.P, w.V, M)
    pipe = Pipeline(w, good)
    # not bound yet
    with pytest.raises(B.JppError) as e:
        pipe.run()
    assert e.value.status == B.JPP_ESTATE
    pipe.set_params_host(params)
    pipe.bind(x0, None, tg)
    pipe.zero_grads()
    # actor 0 asks for stage 2 (fed through actor 1 by its own stage 0) first: a cycle
    bad0 = [(i, "fwd", s) for s in (2, 0) for i in range(M)] + [(i, "bwd", s) for s in (2, 0) for i in range(M)]
    with pytest.raises(po.Deadlock):
        po.global_order([bad0, good[1]], S)
    with pytest.raises(B.JppError) as e:
        pipe.run([bad0, good[1]])
    assert e.value.status == B.JPP_ESCHED and "deadlock" in str(e.value)
    # a list that is wrong for its own actor is named as such
    with pytest.raises(B.JppError) as e:
        pipe.run([good[0][:-1], good[1]])
    assert e.value.status == B.JPP_ESCHED and "actor 0" in str(e.value)
    # nothing ran: the gradients are still the zeros written above, and a good run works
    pipe.sync()
    for a in pipe.actors:
        for v in range(w.V):
            assert float(a.grads_tensor(v).abs().max()) == 0.0
    pipe.run(good)
    got = pipe.results()
    ref = po.run_pipeline(spec, params, good, x0, tg)
    assert worst_error(w, got, ref)[1] < TOL[w.dtype]
    pipe.close()


def test_pipeline_rejects_actors_that_do_not_fit_together():
    from paper_2412_14374_amd.harness import Stage
    w = replace(PIPES["gpt-fp32-cot-1f1b"][0], P=2)
    a0 = Stage(replace(w, rank=0), tasks=osch.one_f_one_b(2, 0, w.n_microbatches))
    a1 = Stage(replace(w, rank=1), tasks=osch.one_f_one_b(2, 1, w.n_microbatches))
    nbytes = B.jpp_pipeline_arena_bytes(a0.cfg, 2, w.n_microbatches)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda:0")
    base = (arena.data_ptr() + 255) // 256 * 256
    with pytest.raises(B.JppError) as e:
        B.jpp_pipeline_create([a1.h, a0.h], base, nbytes)        # wrong order of ranks
    assert e.value.status == B.JPP_EINVAL
    with pytest.raises(B.JppError):
        B.jpp_pipeline_create([a0.h, a0.h], base, nbytes)        # the same actor twice
    with pytest.raises(B.JppError):
        B.jpp_pipeline_create([a0.h, a1.h], base, nbytes - 256)  # arena too small
    h = B.jpp_pipeline_create([a0.h, a1.h], base, nbytes)
    B.jpp_pipeline_destroy(h)
    a0.close()
    a1.close()
