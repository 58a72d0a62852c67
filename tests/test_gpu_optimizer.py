"""GPU parity of the parameter update that follows gradient accumulation (Section 3.1 of the
paper: the step ends with apply_gradient) against oracle/optimizer_oracle.py, and of a short
training loop (run, update, run, ...) against the oracle's."""
from dataclasses import replace

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import optimizer_oracle as oo
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


def rel_l2(a, b):
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a)


def oracle_tasks(tasks):
    return [(i, "fwd" if ty == B.JPP_FWD else "bwd", s) for (i, ty, s) in tasks]


def tree_map2(f, a, b):
    out = {"layers": [{k: f(la[k], lb[k]) for k in la} for la, lb in zip(a["layers"], b["layers"])]}
    if "head" in a:
        out["head"] = {k: f(a["head"][k], b["head"][k]) for k in a["head"]}
    return out


W = inp.Workload("opt-tiny", inp.DT_F32, 2, 64, 2, 2, 32, 128, 24, 2, 3, loss_head=1, vocab=80, w_std=0.1,
                 sched=inp.SCHED_1F1B, P=2, rank=1)


@pytest.mark.parametrize("kind", ["sgd", "adamw"])
def test_three_training_steps_match_the_oracle(kind):
    """fp32 storage: run the task list, update, three times; the losses of every step and the
    final parameters follow the oracle's loop (float64) to 1e-5 / 2e-5."""
    w = W
    spec = spec_of(w)
    params, x, cot, tg = inp.draw_stage_inputs(w, so.layer_param_shapes(spec), so.head_param_shapes(spec), seed=4,
                                               perturb=True)
    s0 = w.stage_ids[0]
    st = Stage(w)
    st.set_params_host(params)
    st.bind(x, cot, tg)
    hyper = dict(lr=2e-3, beta1=0.9, beta2=0.95, eps=1e-6, weight_decay=0.01)
    k = B.JPP_OPT_ADAMW if kind == "adamw" else B.JPP_OPT_SGD
    st.optimizer_bind(k)
    ref_p = params[s0]
    zeros = tree_map2(lambda a, b: np.zeros_like(a), ref_p, ref_p)
    ref_m, ref_v = zeros, tree_map2(lambda a, b: np.zeros_like(a), ref_p, ref_p)
    for t in (1, 2, 3):
        st.zero_grads()
        st.run()
        if kind == "adamw":
            st.apply_gradients(k, step=t, **hyper)
        else:
            st.apply_gradients(k, lr=5e-3, weight_decay=0.01)
        got_loss = st.losses()[:w.n_microbatches]
        ref = so.run_task_list(spec, {s0: ref_p}, oracle_tasks(st.tasks), x, cot, tg)
        assert rel_l2(got_loss, np.array(ref["loss"][s0])) < 1e-5, t
        g = ref["grads"][s0]
        if kind == "adamw":
            new = tree_map2(lambda a, b: a, ref_p, ref_p)
            for grp in (["head"] if "head" in g else []) + list(range(len(g["layers"]))):
                gp = g["head"] if grp == "head" else g["layers"][grp]
                for name in gp:
                    pp = ref_p["head"] if grp == "head" else ref_p["layers"][grp]
                    mm = ref_m["head"] if grp == "head" else ref_m["layers"][grp]
                    vv = ref_v["head"] if grp == "head" else ref_v["layers"][grp]
                    nn = new["head"] if grp == "head" else new["layers"][grp]
                    nn[name], mm[name], vv[name] = oo.adamw_step(pp[name], mm[name], vv[name], gp[name], t,
                                                                 hyper["lr"], hyper["beta1"], hyper["beta2"],
                                                                 hyper["eps"], hyper["weight_decay"])
            ref_p = new
        else:
            ref_p = tree_map2(lambda p_, g_: oo.sgd_step(p_, g_, 5e-3, 0.01), ref_p, g)
    got = st.unpack_grads(st.params_tensor(0).double().cpu().numpy())     # same layout as the gradients
    worst = 0.0
    for li, lp in enumerate(ref_p["layers"]):
        for name, v in lp.items():
            worst = max(worst, rel_l2(got["layers"][li][name], v))
    for name, v in ref_p["head"].items():
        worst = max(worst, rel_l2(got["head"][name], v))
    st.close()
    # SGD is linear in the gradient, so the parameters inherit its 1e-5.  AdamW divides by
    # sqrt(v): an element moves by about lr * g / (|g| + eps) per step, so the relative error
    # of that single gradient element (far above 1e-5 for the smallest elements of a tensor)
    # enters with weight lr; three steps of lr = 2e-3 on parameters of size ~0.1 bound the
    # effect by about 2e-4.  The update's own arithmetic is pinned to 1e-6 in the next test,
    # where the oracle is fed the very gradients the kernel read.
    assert worst < (2e-4 if kind == "adamw" else 2e-5)


def test_bf16_adamw_keeps_fp32_master_weights():
    """bf16 storage: the stored parameters are the fp32 master weights rounded to bf16 (bit for
    bit), and the master weights follow the oracle applied to the GPU's own fp32 gradients."""
    w = replace(inp.shrunk_twin(inp.C2, d_model=256, seq_len=64, d_ffn=512, n_q_heads=2, n_microbatches=2), n_layers=1)
    st = Stage(w)
    st.set_params_random(seed=3)
    st.bind(seed=4)
    st.optimizer_bind(B.JPP_OPT_ADAMW)
    p0 = st.params_tensor(0).float().cpu().numpy().astype(np.float64)
    n = p0.size
    master, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    # the hyper-parameters cross the C boundary as floats: the oracle gets those very values
    lr, b1, b2, eps, wd = (float(np.float32(x)) for x in (1e-3, 0.9, 0.999, 1e-8, 0.1))
    for t in (1, 2):
        st.zero_grads()
        st.run()
        g = st.grads_tensor(0).cpu().numpy().astype(np.float64)
        st.apply_gradients(B.JPP_OPT_ADAMW, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1, step=t)
        st.sync()
        master, m, v = oo.adamw_step(master, m, v, g, t, lr, b1, b2, eps, wd)
        state = st.opt_state.cpu().numpy().astype(np.float64)
        assert rel_l2(state[:n], master) < 1e-6
        assert rel_l2(state[n:2 * n], m) < 1e-6
        assert rel_l2(state[2 * n:3 * n], v) < 1e-6
        stored = st.params_tensor(0).cpu()
        assert torch.equal(stored.view(torch.int16), st.opt_state[:n].to(torch.bfloat16).cpu().view(torch.int16))
        master = state[:n]          # continue from the GPU's fp32 values: no drift between the two
        m, v = state[n:2 * n], state[2 * n:3 * n]
    st.close()


def test_optimizer_errors():
    st = Stage(W)
    with pytest.raises(B.JppError) as e:
        st.apply_gradients(B.JPP_OPT_ADAMW, lr=1e-3, step=1)       # no state bound
    assert e.value.status == B.JPP_ESTATE
    with pytest.raises(B.JppError) as e:
        st.optimizer_bind(B.JPP_OPT_ADAMW)                         # parameters not set yet
    assert e.value.status == B.JPP_ESTATE
    st.set_params_random(seed=0)
    st.optimizer_bind(B.JPP_OPT_ADAMW)
    with pytest.raises(B.JppError):
        st.apply_gradients(B.JPP_OPT_ADAMW, lr=1e-3, step=0)
    with pytest.raises(B.JppError):
        st.apply_gradients(7, lr=1e-3)
    assert B.jpp_stage_optimizer_bytes(st.h, B.JPP_OPT_SGD) == 0
    assert B.jpp_stage_optimizer_bytes(st.h, B.JPP_OPT_ADAMW) == 3 * 4 * st.pcount
    st.close()
