"""GPU parity of the token embedding stage and of a tied embedding / LM head across the first
and the last stage of a pipeline (Section 3, "Weight Sharing and Gradient Accumulation"),
against oracle/tied_oracle.py, through the C ABI.

Each actor accumulates the partial gradient of its own use of the shared table during the
run (the carried states of the commuted loop); jpp_pipeline_sum_tied_gradients is the one
addition after the loop.  Checked: the partial sums against the oracle's, the final sum
against the oracle's loop as the user writes it (uncommuted), the two copies of the gradient
(and, after an update, of the table) bit for bit against each other.
Tolerances as everywhere: 1e-5 (fp32 storage), 2e-2 (bf16 storage), relative L2 per tensor.
"""
from dataclasses import replace

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import optimizer_oracle as oo
from oracle import schedules as osch
from oracle import stage_oracle as so
from oracle import tied_oracle as to
from paper_2412_14374_amd import binding as B
from paper_2412_14374_amd import inputs as inp
from paper_2412_14374_amd.harness import Pipeline, Stage

pytestmark = pytest.mark.gpu

TOL = {inp.DT_F32: 1e-5, inp.DT_BF16: 2e-2}


def spec_of(w):
    return so.StageSpec(n_layers=w.n_layers, d_model=w.d_model, n_q_heads=w.n_q_heads,
                        n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, d_ffn=w.d_ffn,
                        seq_len=w.seq_len, microbatch=w.microbatch, norm=w.norm, act=w.act,
                        use_bias=bool(w.use_bias), rope=bool(w.rope), rope_theta=w.rope_theta,
                        norm_eps=w.norm_eps, loss_head=bool(w.loss_head), vocab=w.vocab)


def rel_l2(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape
    assert np.all(np.isfinite(a))
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a)


def lists_for(w):
    if w.V > 1:
        return [osch.interleaved_1f1b(w.P, r, w.V, w.n_microbatches) for r in range(w.P)]
    return [osch.one_f_one_b(w.P, r, w.n_microbatches) for r in range(w.P)]


TIED = {
    # 2 actors x 2 virtual stages, fp32, few distinct ids: positions collide in the table's gradient
    "gpt-fp32-interleaved": (inp.Workload("t1", inp.DT_F32, 1, 64, 2, 2, 32, 128, 32, 2, 4, loss_head=1, embed=1,
                                          vocab=96, w_std=0.1, P=2, V=2, sched=inp.SCHED_INTERLEAVED), 7),
    # the same with rematerialisation: the embedding's output is the first layer's kept input
    "gpt-fp32-interleaved-remat": (inp.Workload("t1r", inp.DT_F32, 1, 64, 2, 2, 32, 128, 32, 2, 4, loss_head=1, embed=1,
                                                remat=1, vocab=96, w_std=0.1, P=2, V=2, sched=inp.SCHED_INTERLEAVED), 7),
    # a single actor that holds both uses of the table
    "gpt-fp32-one-actor": (inp.Workload("t2", inp.DT_F32, 2, 64, 2, 2, 32, 128, 24, 1, 3, loss_head=1, embed=1,
                                        vocab=40, w_std=0.1, P=1, V=1, sched=inp.SCHED_1F1B), None),
    # Llama-style layers, three actors
    "llama-fp32-1f1b": (inp.Workload("t3", inp.DT_F32, 1, 64, 4, 2, 16, 96, 32, 1, 5, norm=inp.NORM_RMSNORM,
                                     act=inp.ACT_SWIGLU, use_bias=0, rope=1, loss_head=1, embed=1, vocab=64,
                                     w_std=0.1, P=3, V=1, sched=inp.SCHED_1F1B), 9),
    # bf16 storage, MFMA kernels, ragged sizes, weight-gradient groups of 2
    "gpt-bf16-interleaved-groups": (inp.Workload("t4", inp.DT_BF16, 1, 256, 2, 2, 128, 512, 136, 1, 4, loss_head=1,
                                                 embed=1, vocab=520, wgrad_group=2, P=2, V=2,
                                                 sched=inp.SCHED_INTERLEAVED), 50),
}


def build(w, distinct, seed=23):
    spec = spec_of(w)
    S = w.P * w.V
    params, E, tokens, targets = inp.draw_tied_inputs(w, S, so.layer_param_shapes(spec), so.head_param_shapes(spec),
                                                      seed=seed, perturb=True, distinct_ids=distinct)
    dev_params = {s: dict(params[s]) for s in range(S)}
    dev_params[0] = dict(dev_params[0], embed={"w": E})
    dev_params[S - 1] = dict(dev_params[S - 1], head=dict(params[S - 1]["head"], w_head=E))
    lists = lists_for(w)
    pipe = Pipeline(w, lists)
    pipe.set_params_host(dev_params)
    pipe.bind(tokens, None, targets)
    return spec, params, E, tokens, targets, pipe


@pytest.mark.parametrize("name", sorted(TIED))
def test_tied_pipeline_matches_oracle(name):
    w, distinct = TIED[name]
    spec, params, E, tokens, targets, pipe = build(w, distinct)
    S = w.P * w.V
    ref = to.run_tied_model(spec, params, E, tokens, targets)
    tol = TOL[w.dtype]
    pipe.zero_grads()
    pipe.run()
    got = pipe.results()
    # the carried partial sums, each where it is produced
    assert rel_l2(got["grads"][0]["embed"]["w"], sum(ref["g1"])) < tol
    assert rel_l2(got["grads"][S - 1]["head"]["w_head"], sum(ref["g2"])) < tol
    for i in range(w.n_microbatches):
        assert abs(got["loss"][i] - ref["loss"][i]) <= tol * abs(ref["loss"][i]), i
    for s in range(S):
        for li, lg in enumerate(ref["grads"][s]["layers"]):
            for k, v in lg.items():
                assert rel_l2(got["grads"][s]["layers"][li][k], v) < tol, (s, li, k)
    for k, v in ref["grads"][S - 1]["head"].items():
        assert rel_l2(got["grads"][S - 1]["head"][k], v) < tol, k
    # the one addition after the loop
    pipe.sum_tied_gradients()
    after = pipe.results()
    a, b = after["grads"][0]["embed"]["w"], after["grads"][S - 1]["head"]["w_head"]
    assert np.array_equal(a, b)
    assert rel_l2(a, ref["gE_uncommuted"]) < tol
    assert rel_l2(a, ref["gE_commuted"]) < tol
    # fp32 partial sums added once: exactly the fp32 sum of what was there before
    want = (got["grads"][0]["embed"]["w"].astype(np.float32) + got["grads"][S - 1]["head"]["w_head"].astype(np.float32))
    assert np.array_equal(a.astype(np.float32), want)
    pipe.close()


def test_embedding_stage_alone_matches_oracle():
    """One actor, no head: y = F(E[ids]) and the table's gradient from the incoming
    cotangents; every id occurs several times per microbatch (5 distinct ids, 48 positions)."""
    w = inp.Workload("e1", inp.DT_F32, 1, 64, 2, 2, 32, 128, 24, 2, 3, embed=1, vocab=32, w_std=0.2, cot_std=1.0)
    spec = spec_of(w)
    rng = np.random.default_rng(31)
    params = {0: {"layers": [inp.draw_params(so.layer_param_shapes(spec), rng, w, True)]}}
    E = inp.round_to_dtype(rng.standard_normal((w.vocab, w.d_model)), w.dtype)
    ids = rng.permutation(w.vocab)[:5]
    M = w.n_microbatches
    tokens = [ids[rng.integers(0, 5, size=(w.microbatch, w.seq_len))].astype(np.int32) for _ in range(M)]
    cot = [inp.round_to_dtype(rng.standard_normal((w.microbatch, w.seq_len, w.d_model)), w.dtype) for _ in range(M)]
    st = Stage(w)
    st.set_params_host({0: dict(params[0], embed={"w": E})})
    st.bind({0: tokens}, {0: cot}, None)
    st.zero_grads()
    st.run()
    got = st.results()
    x = {0: [to.embed_forward(E, t) for t in tokens]}
    ref = so.run_task_list(spec, params, [(i, "fwd" if ty == B.JPP_FWD else "bwd", s) for (i, ty, s) in st.tasks],
                           x, {0: cot}, None)
    for i in range(M):
        assert rel_l2(got["y"][0][i], ref["y"][0][i]) < 1e-5
    gE = sum(to.embed_backward(w.vocab, tokens[i], ref["dx"][0][i]) for i in range(M))
    assert rel_l2(got["grads"][0]["embed"]["w"], gE) < 1e-5
    unused = np.setdiff1d(np.arange(w.vocab), ids)
    assert np.all(got["grads"][0]["embed"]["w"][unused] == 0.0)
    for k, v in ref["grads"][0]["layers"][0].items():
        assert rel_l2(got["grads"][0]["layers"][0][k], v) < 1e-5, k
    st.close()


def test_update_keeps_the_two_copies_of_the_table_identical():
    """Sum, then the same SGD step on both actors: the table of stage 0 and the head's weight
    of the last stage stay the same bits, and equal the oracle's step on the shared weight."""
    w, distinct = TIED["gpt-fp32-interleaved"]
    spec, params, E, tokens, targets, pipe = build(w, distinct, seed=29)
    ref = to.run_tied_model(spec, params, E, tokens, targets)
    pipe.zero_grads()
    pipe.run()
    pipe.sum_tied_gradients()
    first, last = pipe.actors[0], pipe.actors[-1]
    # the sum ran on actor 0's compute stream: the last actor's update must follow it
    first.compute.synchronize()
    lr, wd = 0.05, 0.01
    for a in (first, last):
        a.apply_gradients(B.JPP_OPT_SGD, lr=lr, weight_decay=wd)
    pipe.sync()
    torch.cuda.synchronize()
    off = {n: (o, int(np.prod(s)), s) for n, s, o in first.info}
    o1, n1, shp = off["embed.w"]
    o2, n2, _ = {n: (o, int(np.prod(s)), s) for n, s, o in last.info}["head.w_head"]
    e_new = first.params_tensor(0)[o1:o1 + n1].cpu()
    h_new = last.params_tensor(w.V - 1)[o2:o2 + n2].cpu()
    assert torch.equal(e_new, h_new)
    want = oo.sgd_step(E, ref["gE_uncommuted"], lr=lr, weight_decay=wd)
    assert rel_l2(e_new.double().numpy().reshape(shp), want) < 1e-5
    pipe.close()


def test_tied_sum_errors():
    # no embedding: nothing is tied
    w = replace(TIED["gpt-fp32-interleaved"][0], embed=0)
    lists = lists_for(w)
    pipe = Pipeline(w, lists)
    with pytest.raises(B.JppError) as e:
        pipe.sum_tied_gradients()
    assert e.value.status == B.JPP_ESTATE
    pipe.close()
    # the embedding belongs to the first global stage: an actor other than 0 cannot carry it
    w = TIED["gpt-fp32-interleaved"][0]
    a0 = Stage(replace(w, rank=0, loss_head=0, embed=0), tasks=lists[0])
    a1 = Stage(replace(w, rank=1, embed=1), tasks=lists[1])
    with pytest.raises(B.JppError) as e:
        B.jpp_pipeline_create([a0.h, a1.h], 0, 0)
    assert e.value.status == B.JPP_EINVAL
    a0.close()
    a1.close()
    with pytest.raises(B.JppError) as e:
        B.jpp_stage_arena_bytes(B.make_config(replace(w, vocab=0, loss_head=0)), 4, 4)
    assert e.value.status == B.JPP_EINVAL


def test_full_size_embedding_kernels_on_sampled_rows():
    """The kernels at a production shape (4096 tokens, GPT-2 vocabulary 50304, d_model 4096,
    bf16) with a Zipf-like id distribution, so that a few ids occur hundreds of times and most
    never: the forward against the table's rows, the gradient's rows for the most frequent, a
    few rare and a few absent ids against the oracle's position-ordered sum, accumulated onto
    a non-zero gradient."""
    rows, d, vocab = 4096, 4096, 50304
    rng = np.random.default_rng(41)
    ids = np.minimum((rng.pareto(1.1, size=rows) * 3).astype(np.int64), vocab - 1).astype(np.int32)
    bad = [7, 1000, 4095]                       # ids outside the table: a zero row, no gradient
    ids[bad] = [-1, vocab, 2 ** 31 - 1]
    g = torch.Generator(device="cuda:0")
    g.manual_seed(3)
    table = (torch.randn((vocab, d), generator=g, device="cuda:0") * 0.02).to(torch.bfloat16)
    dx = torch.randn((rows, d), generator=g, device="cuda:0").to(torch.bfloat16)
    G0 = torch.randn((vocab, d), generator=g, device="cuda:0")
    ids_d = torch.from_numpy(ids).to("cuda:0")
    x = torch.empty((rows, d), dtype=torch.bfloat16, device="cuda:0")
    G = G0.clone()
    torch.cuda.synchronize()
    s = torch.cuda.current_stream().cuda_stream
    B.jpp_op_embed_fwd(B.JPP_BF16, rows, d, vocab, ids_d.data_ptr(), table.data_ptr(), x.data_ptr(), s)
    B.jpp_op_embed_bwd(B.JPP_BF16, rows, d, vocab, ids_d.data_ptr(), dx.data_ptr(), G.data_ptr(), s)
    torch.cuda.synchronize()
    valid = torch.from_numpy((ids >= 0) & (ids < vocab)).to("cuda:0")
    assert torch.equal(x[valid].view(torch.int16), table[ids_d[valid].long()].view(torch.int16))
    assert bool((x[~valid] == 0).all()) and int((~valid).sum()) == len(bad)
    ids = np.where((ids >= 0) & (ids < vocab), ids, 0 * ids - 1)
    counts = np.bincount(ids[ids >= 0], minlength=vocab)
    frequent = list(np.argsort(-counts)[:4])
    rare = list(np.flatnonzero(counts == 1)[:4])
    absent = list(np.flatnonzero(counts == 0)[:4])
    assert counts[frequent[0]] > 100 and rare and absent
    dx_h = dx.double().cpu().numpy()
    for v in frequent + rare:
        pos = np.flatnonzero(ids == v)
        want = to.embed_backward(1, np.zeros((1, len(pos)), dtype=np.int64), dx_h[pos][None])[0]
        got = (G[v].double() - G0[v].double()).cpu().numpy()
        assert rel_l2(got, want) < 1e-5, (v, len(pos))
    for v in absent:
        assert torch.equal(G[v], G0[v])
    # untouched rows in bulk: every row whose id never occurs keeps its bits
    mask = torch.from_numpy(counts == 0).to("cuda:0")
    assert torch.equal(G[mask], G0[mask])
