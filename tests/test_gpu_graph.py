"""HIP-graph capture of a step.  Recording jpp_stage_run into a graph was implemented once (fork
of the side stream, no completion queries, no waits for events outside the graph); the first GPU
run of the replay test ended in a segmentation fault inside the HIP runtime when the capture was
closed (torch.cuda.graph -> capture_end), with no cause found in this repository's code.  The
code path is therefore switched off (jpp_stage_run and jpp_pipeline_run return JPP_ESTATE while
their compute stream is capturing) and the tests below stay skipped until a cause is shown."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import stage_oracle as so
from paper_2412_14374_amd import binding as B
from paper_2412_14374_amd import inputs as inp
from paper_2412_14374_amd.harness import Stage

pytestmark = pytest.mark.gpu


def spec_of(w):
    return so.StageSpec(n_layers=w.n_layers, d_model=w.d_model, n_q_heads=w.n_q_heads,
                        n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, d_ffn=w.d_ffn,
                        seq_len=w.seq_len, microbatch=w.microbatch, norm=w.norm, act=w.act,
                        use_bias=bool(w.use_bias), rope=bool(w.rope), rope_theta=w.rope_theta,
                        norm_eps=w.norm_eps, loss_head=bool(w.loss_head), vocab=w.vocab)


def snapshot(st, w):
    st.sync()
    torch.cuda.synchronize()
    return ([st.grads_tensor(v).cpu() for v in range(len(w.stage_ids))],
            [t.cpu().clone() for t in st.out_y], [t.cpu().clone() for t in st.out_dx])


def same(a, b):
    return all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for ka, kb in zip(a, b) for x, y in zip(ka, kb))


CASES = {
    "C1 gpipe fp32": inp.C1,
    "bf16 1f1b twin": inp.shrunk_twin(inp.C2, d_model=256, seq_len=64, d_ffn=512, n_q_heads=2, n_microbatches=6),
}


@pytest.mark.skip(reason="closing the capture of a run crashed inside the HIP runtime (segmentation fault in "
                         "capture_end); the capture path is switched off, see the module docstring")
@pytest.mark.parametrize("name", sorted(CASES))
def test_graph_replays_equal_the_eager_step(name):
    w = CASES[name]
    spec = spec_of(w)
    params, x, cot, tg = inp.draw_stage_inputs(w, so.layer_param_shapes(spec), None, seed=8, perturb=True)
    st = Stage(w)
    st.set_params_host(params)
    st.bind(x, cot, tg)
    st.zero_grads()
    st.run()
    eager = snapshot(st, w)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st.compute):
        st.zero_grads()
        st.run()
    # the recording executed nothing and must not have disturbed the results of the eager run
    assert same(snapshot(st, w), eager)
    for k in range(3):
        for t in st.out_y + st.out_dx:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        assert same(snapshot(st, w), eager), k
        # eager work of the program itself between the replays
        st.zero_grads()
        st.run()
        assert same(snapshot(st, w), eager), k
    # replay after replay, no eager step in between
    graph.replay()
    graph.replay()
    assert same(snapshot(st, w), eager)
    del graph
    st.close()


@pytest.mark.skip(reason="needs an open stream capture; no capture is opened on the GPU box until the crash "
                         "described in the module docstring is understood")
def test_pipeline_run_refuses_to_be_captured():
    from oracle import schedules as osch
    from paper_2412_14374_amd.harness import Pipeline
    w = inp.Workload("g", inp.DT_F32, 1, 64, 2, 2, 32, 128, 16, 1, 2, w_std=0.1, cot_std=1.0, P=2, V=1,
                     sched=inp.SCHED_1F1B)
    lists = [osch.one_f_one_b(2, r, 2) for r in range(2)]
    pipe = Pipeline(w, lists)
    pipe.set_params_random(seed=1)
    pipe.bind_random(seed=2)
    g = torch.cuda.CUDAGraph()
    err = None
    with torch.cuda.graph(g, stream=pipe.actors[0].compute):
        try:
            pipe.run()
        except B.JppError as e:
            err = e
    assert err is not None and err.status == B.JPP_ESTATE
    pipe.zero_grads()
    pipe.run()            # still usable
    pipe.sync()
    pipe.close()
