"""Pins for the fp64 CPU oracle: everything here checks oracle/ against facts
fixed by mathematics or by the paper, never against the HIP path.

* central finite differences of Phi = sum_i <y_i, c_i> (or sum_i loss_i);
* the accumulation semantics of the paper's Section 3.1 (sum over microbatches
  equals the gradient of the one big batch, no 1/M; losses as a vector);
* schedule invariance (Section 2.2.1: any order that honours the data
  dependencies computes the same thing);
* closed forms and special cases of the layer mathematics;
* an independent float64 computation with a library autograd.
"""
import math

import numpy as np
import pytest

from oracle import stage_oracle as so
from oracle import schedules as sch
from paper_2412_14374_amd import inputs as inp


def tiny(kind, **kw):
    base = dict(name="tiny", dtype=inp.DT_F32, n_layers=2, d_model=16, n_q_heads=2, n_kv_heads=2,
                head_dim=8, d_ffn=32, seq_len=8, microbatch=2, n_microbatches=3, cot_std=1.0,
                w_std=0.3)
    if kind == "llama":
        base.update(n_q_heads=4, n_kv_heads=2, head_dim=4, norm=inp.NORM_RMSNORM,
                    act=inp.ACT_SWIGLU, use_bias=0, rope=1)
    if kind == "head":
        base.update(loss_head=1, vocab=37)
    if kind == "gelu_tanh":
        base.update(act=inp.ACT_GELU_TANH)
    base.update(kw)
    return inp.Workload(**base)


def spec_of(w):
    return so.StageSpec(n_layers=w.n_layers, d_model=w.d_model, n_q_heads=w.n_q_heads,
                        n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, d_ffn=w.d_ffn,
                        seq_len=w.seq_len, microbatch=w.microbatch, norm=w.norm, act=w.act,
                        use_bias=bool(w.use_bias), rope=bool(w.rope), rope_theta=w.rope_theta,
                        norm_eps=w.norm_eps, loss_head=bool(w.loss_head), vocab=w.vocab)


def draw(w, seed=1, perturb=True):
    spec = spec_of(w)
    params, x, cot, tg = inp.draw_stage_inputs(
        w, so.layer_param_shapes(spec), so.head_param_shapes(spec) if w.loss_head else None,
        seed=seed, perturb=perturb)
    # pins work on un-rounded float64 values: undo nothing, just use them as is
    return spec, params, x, cot, tg


def phi(spec, params, xs, cots, tgs):
    tot = 0.0
    for i, x in enumerate(xs):
        out, _ = so.stage_forward(spec, params, x, None if tgs is None else tgs[i])
        tot += out if spec.loss_head else float((out * cots[i]).sum())
    return tot


def accumulate(spec, params, xs, cots, tgs):
    G = None
    dxs = []
    for i, x in enumerate(xs):
        _, cache = so.stage_forward(spec, params, x, None if tgs is None else tgs[i])
        dx, g = so.stage_backward(spec, params, cache, None if spec.loss_head else cots[i])
        G = so._tree_add(G, g)
        dxs.append(dx)
    return G, dxs


def leaves(params):
    for li, lp in enumerate(params["layers"]):
        for k in lp:
            yield ("layers", li, k), lp[k]
    if "head" in params:
        for k in params["head"]:
            yield ("head", None, k), params["head"][k]


def get_leaf(tree, key):
    return tree["head"][key[2]] if key[0] == "head" else tree["layers"][key[1]][key[2]]


@pytest.mark.parametrize("kind", ["gpt", "llama", "head", "gelu_tanh"])
def test_finite_differences_all_parameters_and_inputs(kind):
    w = tiny(kind)
    spec, params, x, cot, tg = draw(w)
    s = w.stage_ids[0]
    P, xs, cs = params[s], x[s], cot[s]
    G, dxs = accumulate(spec, P, xs, cs, tg)
    rng = np.random.default_rng(7)
    for key, arr in leaves(P):
        g = get_leaf(G, key)
        flat = arr.reshape(-1)
        idxs = range(flat.size) if flat.size <= 48 else rng.choice(flat.size, 24, replace=False)
        for j in idxs:
            old = flat[j]
            h = 1e-6 * max(1.0, abs(old))
            flat[j] = old + h
            fp = phi(spec, P, xs, cs, tg)
            flat[j] = old - h
            fm = phi(spec, P, xs, cs, tg)
            flat[j] = old
            fd = (fp - fm) / (2 * h)
            an = g.reshape(-1)[j]
            # 2e-7 absolute: rounding noise of Phi (~1e-14) divided by the step
            assert abs(fd - an) <= 2e-6 * max(abs(an), abs(fd)) + 2e-7, (key, j, fd, an)
    # input cotangent dx_0
    x0 = xs[0].reshape(-1)
    for j in rng.choice(x0.size, 24, replace=False):
        old = x0[j]
        h = 1e-6 * max(1.0, abs(old))
        x0[j] = old + h
        fp = phi(spec, P, xs, cs, tg)
        x0[j] = old - h
        fm = phi(spec, P, xs, cs, tg)
        x0[j] = old
        fd = (fp - fm) / (2 * h)
        an = dxs[0].reshape(-1)[j]
        assert abs(fd - an) <= 2e-6 * max(abs(an), abs(fd)) + 2e-7


@pytest.mark.parametrize("kind", ["gpt", "llama", "head"])
def test_accumulation_equals_one_big_batch_no_averaging(kind):
    """Section 3.1: grads are summed, not averaged.  The sum over M microbatches
    must equal the gradient of sum_i <F(x_i), c_i> evaluated as one batch of
    M*mb sequences (for the loss head: M times the big batch's mean loss)."""
    w = tiny(kind)
    spec, params, x, cot, tg = draw(w)
    s = w.stage_ids[0]
    G, _ = accumulate(spec, params[s], x[s], cot[s], tg)
    M = w.n_microbatches
    big = so.StageSpec(**{**spec.__dict__, "microbatch": spec.microbatch * M})
    X = np.concatenate(x[s], axis=0)
    C = np.concatenate(cot[s], axis=0)
    TG = None if tg is None else np.concatenate(tg, axis=0)
    out, cache = so.stage_forward(big, params[s], X, TG)
    _, gbig = so.stage_backward(big, params[s], cache, C)
    scale = float(M) if spec.loss_head else 1.0
    for key, _ in leaves(params[s]):
        a, b = get_leaf(G, key), get_leaf(gbig, key) * scale
        assert np.linalg.norm(a - b) <= 1e-12 * max(1.0, np.linalg.norm(b)), key
    if spec.loss_head:
        losses = [so.stage_forward(spec, params[s], x[s][i], tg[i])[0] for i in range(M)]
        assert abs(np.mean(losses) - out) < 1e-13


def test_schedule_invariance_bitwise_and_peak_live():
    """GPipe, 1F1B at every rank and interleaved 1F1B give identical fp64 bits
    for y, dx and G; peak live stashes follow Section 2.2.1 (GPipe: number of
    microbatches; 1F1B: bounded by the number of stages)."""
    w = tiny("gpt", n_microbatches=4, n_layers=1)
    spec, params, x, cot, tg = draw(w)
    s0 = w.stage_ids[0]
    P = 4

    def run(tasks, stage):
        remap = [(i, ty, s0) for (i, ty, _) in tasks]
        return so.run_task_list(spec, {s0: params[s0]}, remap, x, cot, tg)

    ref = run(sch.gpipe(P, 0, 4), 0)
    assert ref["peak_live"] == 4
    for r in range(P):
        out = run(sch.one_f_one_b(P, r, 4), r)
        assert out["peak_live"] == min(P - r, 4)
        for i in range(4):
            assert np.array_equal(out["y"][s0][i], ref["y"][s0][i])
            assert np.array_equal(out["dx"][s0][i], ref["dx"][s0][i])
        for key, _ in leaves(params[s0]):
            assert np.array_equal(get_leaf(out["grads"][s0], key), get_leaf(ref["grads"][s0], key))

    # two virtual stages with their own parameters and inputs
    w2 = tiny("gpt", n_microbatches=4, n_layers=1, sched=inp.SCHED_INTERLEAVED, P=2, rank=1, V=2)
    spec2, p2, x2, c2, _ = draw(w2)
    il = so.run_task_list(spec2, p2, sch.interleaved_1f1b(2, 1, 2, 4), x2, c2)
    for s in w2.stage_ids:
        solo = so.run_task_list(spec2, {s: p2[s]}, [(i, ty, s) for (i, ty, _) in sch.gpipe(2, 1, 4)],
                                x2, c2)
        for key, _ in leaves(p2[s]):
            assert np.array_equal(get_leaf(il["grads"][s], key), get_leaf(solo["grads"][s], key))
        for i in range(4):
            assert np.array_equal(il["dx"][s][i], solo["dx"][s][i])


def test_reverse_backward_order_agrees_to_rounding_only():
    w = tiny("gpt", n_microbatches=4)
    spec, params, x, cot, tg = draw(w)
    s = w.stage_ids[0]
    fwd = [(i, "fwd", s) for i in range(4)]
    a = so.run_task_list(spec, params, fwd + [(i, "bwd", s) for i in range(4)], x, cot)
    b = so.run_task_list(spec, params, fwd + [(i, "bwd", s) for i in reversed(range(4))], x, cot)
    for key, _ in leaves(params[s]):
        ga, gb = get_leaf(a["grads"][s], key), get_leaf(b["grads"][s], key)
        assert np.linalg.norm(ga - gb) <= 1e-13 * max(1.0, np.linalg.norm(ga))


# ---------------------------------------------------------------- closed forms

def test_seq_len_one_attention_returns_v():
    w = tiny("gpt", seq_len=1)
    spec = spec_of(w)
    rng = np.random.default_rng(0)
    q, k, v = (rng.standard_normal((2, 1, 2, 8)) for _ in range(3))
    O, P = so.attention_forward(spec, q, k, v)
    assert np.array_equal(O, v) and np.all(P == 1.0)


def test_zero_output_projections_make_layer_identity():
    w = tiny("gpt", n_layers=1)
    spec, params, x, cot, _ = draw(w, perturb=False)
    s = w.stage_ids[0]
    p = params[s]["layers"][0]
    p["wo"][:] = 0
    p["w2"][:] = 0
    y, cache = so.layer_forward(spec, p, x[s][0])
    assert np.array_equal(y, x[s][0])
    dx, g = so.layer_backward(spec, p, cache, cot[s][0])
    assert np.array_equal(dx, cot[s][0])
    assert np.all(g["wqkv"] == 0) and np.all(g["w1"] == 0)
    assert np.linalg.norm(g["w2"]) > 0 and np.linalg.norm(g["wo"]) > 0


def test_gqa_with_equal_head_counts_is_mha_and_group_sharing():
    """Query heads of one group read the same kv head: duplicating a kv head
    into an MHA layout gives the same output, and dK/dV of the shared head is
    the sum over the group."""
    w = tiny("llama", rope=0)
    spec = spec_of(w)                      # Hq=4, Hkv=2
    rng = np.random.default_rng(3)
    q = rng.standard_normal((2, 8, 4, 4))
    k = rng.standard_normal((2, 8, 2, 4))
    v = rng.standard_normal((2, 8, 2, 4))
    dO = rng.standard_normal((2, 8, 4, 4))
    O, P = so.attention_forward(spec, q, k, v)
    mha = so.StageSpec(**{**spec.__dict__, "n_kv_heads": 4})
    kk, vv = np.repeat(k, 2, axis=2), np.repeat(v, 2, axis=2)
    O2, P2 = so.attention_forward(mha, q, kk, vv)
    assert np.array_equal(O, O2)
    dq, dk, dv = so.attention_backward(spec, q, k, v, P, dO)
    dq2, dk2, dv2 = so.attention_backward(mha, q, kk, vv, P2, dO)
    assert np.array_equal(dq, dq2)
    assert np.allclose(dk, dk2[:, :, 0::2] + dk2[:, :, 1::2], rtol=0, atol=1e-14)
    assert np.allclose(dv, dv2[:, :, 0::2] + dv2[:, :, 1::2], rtol=0, atol=1e-14)


def test_attention_matches_bruteforce_scalar_loops():
    """Definition written out with scalar loops on a tiny case."""
    w = tiny("gpt", seq_len=5)
    spec = spec_of(w)
    rng = np.random.default_rng(5)
    q, k, v = (rng.standard_normal((1, 5, 2, 8)) for _ in range(3))
    O, _ = so.attention_forward(spec, q, k, v)
    for h in range(2):
        for t in range(5):
            sc = [sum(q[0, t, h, e] * k[0, u, h, e] for e in range(8)) / math.sqrt(8) for u in range(t + 1)]
            m = max(sc)
            ex = [math.exp(s - m) for s in sc]
            z = sum(ex)
            for e in range(8):
                o = sum(ex[u] / z * v[0, u, h, e] for u in range(t + 1))
                assert abs(o - O[0, t, h, e]) < 1e-14


def test_softmax_rows_and_ds_rows():
    w = tiny("gpt")
    spec = spec_of(w)
    rng = np.random.default_rng(6)
    q, k, v, dO = (rng.standard_normal((2, 8, 2, 8)) for _ in range(4))
    O, P = so.attention_forward(spec, q, k, v)
    assert np.allclose(P.sum(-1), 1.0, atol=1e-14)
    assert np.all(np.triu(P, 1) == 0)
    # dS rows sum to zero <=> dq is unchanged when a constant is added to all scores:
    # equivalently sum_u dS_tu = 0; check through dK: shifting every k_u by the same
    # vector delta changes S_tu by q_t.delta for all u, which softmax ignores.
    delta = rng.standard_normal((1, 1, 2, 8))
    O2, _ = so.attention_forward(spec, q, k + delta, v)
    assert np.allclose(O, O2, atol=1e-12)
    _, dk, _ = so.attention_backward(spec, q, k, v, P, dO)
    assert np.allclose(dk.sum(axis=1), 0.0, atol=1e-12)


def test_causality_and_batch_independence():
    w = tiny("gpt")
    spec, params, x, _, _ = draw(w)
    s = w.stage_ids[0]
    x0 = x[s][0]
    y0, _ = so.stage_forward(spec, params[s], x0)
    x1 = x0.copy()
    x1[0, 5, :] += 1.0
    y1, _ = so.stage_forward(spec, params[s], x1)
    assert np.array_equal(y0[0, :5], y1[0, :5])
    assert not np.array_equal(y0[0, 5:], y1[0, 5:])
    assert np.array_equal(y0[1], y1[1])


def test_rope_properties():
    w = tiny("llama")
    spec = spec_of(w)
    rng = np.random.default_rng(9)
    q = rng.standard_normal((2, 8, 4, 4))
    k = rng.standard_normal((2, 8, 2, 4))
    rq = so.rope_apply(spec, q)
    assert np.array_equal(rq[:, 0], q[:, 0])                       # t = 0 is the identity
    assert np.allclose((rq ** 2).sum(-1), (q ** 2).sum(-1), atol=1e-13)
    assert np.allclose(so.rope_apply(spec, rq, transpose=True), q, atol=1e-14)
    # explicit angle of one element: position 3, pair j=1 of hd=4 -> 3 * theta^(-2/4)
    ang = 3.0 * 10000.0 ** (-0.5)
    exp0 = q[0, 3, 0, 1] * math.cos(ang) - q[0, 3, 0, 3] * math.sin(ang)
    exp1 = q[0, 3, 0, 1] * math.sin(ang) + q[0, 3, 0, 3] * math.cos(ang)
    assert abs(rq[0, 3, 0, 1] - exp0) < 1e-15 and abs(rq[0, 3, 0, 3] - exp1) < 1e-15
    # scores depend on relative position only: shift all positions by 2
    big = so.StageSpec(**{**spec.__dict__, "seq_len": 10})
    qpad = np.concatenate([np.zeros((2, 2, 4, 4)), q], axis=1)
    kpad = np.concatenate([np.zeros((2, 2, 2, 4)), k], axis=1)
    rk = so.rope_apply(spec, k)
    rq2, rk2 = so.rope_apply(big, qpad)[:, 2:], so.rope_apply(big, kpad)[:, 2:]
    s1 = np.einsum("bthe,buhe->bhtu", rq[:, :, :2], rk)
    s2 = np.einsum("bthe,buhe->bhtu", rq2[:, :, :2], rk2)
    assert np.allclose(s1, s2, atol=1e-12)


def test_layernorm_closed_forms():
    w = tiny("gpt")
    spec = spec_of(w)
    rng = np.random.default_rng(11)
    x = rng.standard_normal((3, 5, 16)) * 2 + 0.7
    g, b = np.ones(16), np.zeros(16)
    y, xhat, rstd = so.norm_forward(spec, x, g, b)
    var = x.var(axis=-1)
    assert np.allclose(y.mean(-1), 0, atol=1e-14)
    assert np.allclose(y.var(-1), var / (var + 1e-5), atol=1e-13)
    dy = rng.standard_normal(x.shape)
    gg = 1 + 0.1 * rng.standard_normal(16)
    dx, dg, db = so.norm_backward(spec, dy, xhat, rstd, gg)
    assert np.allclose(dx.sum(-1), 0, atol=1e-13)                   # orthogonal to 1
    # dx . xhat = rstd * (dxhat . xhat) * eps/(var+eps)
    lhs = (dx * xhat).sum(-1)
    rhs = rstd[..., 0] * ((dy * gg) * xhat).sum(-1) * (1e-5 / (var + 1e-5))
    assert np.allclose(lhs, rhs, atol=1e-12)
    assert np.allclose(db, dy.sum((0, 1))) and np.allclose(dg, (dy * xhat).sum((0, 1)))


def test_rmsnorm_closed_forms():
    w = tiny("llama")
    spec = spec_of(w)
    rng = np.random.default_rng(12)
    x = rng.standard_normal((2, 3, 16))
    y, xhat, rstd = so.norm_forward(spec, x, np.ones(16), 0.0)
    ms = (x ** 2).mean(-1)
    assert np.allclose((y ** 2).mean(-1), ms / (ms + 1e-5), atol=1e-14)
    # scale invariance up to eps: norm(ax) ~ norm(x); exact with eps -> handled via big x
    y2, _, _ = so.norm_forward(spec, x * 1e4, np.ones(16), 0.0)
    assert np.allclose(y2, x / np.sqrt(ms)[..., None], atol=1e-9)


def test_gelu_and_silu_values():
    spec = spec_of(tiny("gpt"))
    t = np.array([0.0, 1.0, -1.0, 3.0])
    # Phi(1) = 0.841344746068543 (standard normal table)
    assert np.allclose(so.act_forward(spec, t), [0.0, 0.841344746068543, -0.158655253931457,
                                                 3 * 0.998650101968370], atol=1e-14)
    # derivative at 0 is 1/2; at 1: Phi(1) + phi(1) = 0.8413447 + 0.2419707
    assert np.allclose(so.act_backward(spec, t[:2], np.ones(2)), [0.5, 0.841344746068543 + 0.241970724519143],
                       atol=1e-14)
    sw = spec_of(tiny("llama"))
    sw.d_ffn = 1
    # silu(1) = 1/(1+e^-1) = 0.731058578630005
    assert np.allclose(so.act_forward(sw, np.array([1.0, 2.0])), [2 * 0.731058578630005], atol=1e-14)


def test_gelu_tanh_values():
    """The tanh form 0.5 t (1 + tanh(sqrt(2/pi) (t + 0.044715 t^3))), pinned by values that do
    not come from this repository: at t = 1 the argument is 0.7978845608 * 1.044715 =
    0.8335619..., tanh of it 0.6823839812, so gelu_tanh(1) = 0.8411919906; the identity
    gelu_tanh(t) - gelu_tanh(-t) = t (tanh is odd) gives the value at -1; the library's
    float64 implementation covers a grid, and its autograd the derivative.  A mistyped
    0.044715 or sqrt(2/pi), or the erf form in its place (0.8413447 at 1), fails here."""
    torch = pytest.importorskip("torch")
    w = tiny("gelu_tanh")
    spec = spec_of(w)
    got = so.act_forward(spec, np.array([0.0, 1.0, -1.0]))
    assert np.allclose(got, [0.0, 0.8411919906, 0.8411919906 - 1.0], atol=2e-10)
    assert abs(got[1] - 0.841344746068543) > 1e-4          # not the erf form
    t = np.linspace(-6.0, 6.0, 241)
    tt = torch.tensor(t, dtype=torch.float64, requires_grad=True)
    lib = torch.nn.functional.gelu(tt, approximate="tanh")
    assert np.allclose(so.act_forward(spec, t), lib.detach().numpy(), atol=1e-14)
    lib.sum().backward()
    assert np.allclose(so.act_backward(spec, t, np.ones_like(t)), tt.grad.numpy(), atol=1e-13)


def test_cross_entropy_closed_forms():
    w = tiny("head", vocab=50304 // 64)            # 786
    spec, params, x, _, tg = draw(w, perturb=False)
    s = w.stage_ids[0]
    hp = params[s]["head"]
    hp["w_head"][:] = 0
    rng = np.random.default_rng(1)
    y = rng.standard_normal((2, 8, 16))
    loss, c = so.head_forward(spec, hp, y, tg[0])
    assert abs(loss - math.log(786)) < 1e-13
    hp["w_head"][:] = rng.standard_normal(hp["w_head"].shape)
    loss, c = so.head_forward(spec, hp, y, tg[0])
    dz = c["prob"].copy()
    dz[np.arange(16), c["tg"]] -= 1
    assert np.allclose(dz.sum(-1), 0, atol=1e-13)
    # full vocabulary size named by the workload: ln(50304)
    assert abs(math.log(50304) - 10.825840) < 1e-6


# ---------------------------------------------------------------- independent autograd

@pytest.mark.parametrize("kind", ["gpt", "llama", "head"])
def test_against_library_autograd_float64(kind):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    w = tiny(kind, seq_len=12)
    spec, params, x, cot, tg = draw(w)
    s = w.stage_ids[0]
    P = params[s]
    tp = {"layers": [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in lp.items()}
                     for lp in P["layers"]]}
    if "head" in P:
        tp["head"] = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in P["head"].items()}

    def norm(t, g, b):
        if w.norm == inp.NORM_LAYERNORM:
            return F.layer_norm(t, (w.d_model,), g, b, eps=w.norm_eps)
        return F.rms_norm(t, (w.d_model,), g, eps=w.norm_eps)

    def rope(t):
        hd = w.head_dim
        inv = 1.0 / (w.rope_theta ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
        ang = torch.outer(torch.arange(w.seq_len, dtype=torch.float64), inv)
        cs, sn = torch.cos(ang)[None, :, None, :], torch.sin(ang)[None, :, None, :]
        cs, sn = torch.cat([cs, cs], -1), torch.cat([sn, sn], -1)
        rot = torch.cat([-t[..., hd // 2:], t[..., :hd // 2]], -1)
        return t * cs + rot * sn

    def fwd(xt, tgt):
        mb, seq, d = xt.shape
        Hq, Hkv, hd = w.n_q_heads, w.n_kv_heads, w.head_dim
        for lp in tp["layers"]:
            n1 = norm(xt, lp["ln1_g"], lp.get("ln1_b"))
            qkv = F.linear(n1, lp["wqkv"], lp.get("bqkv"))
            q, k, v = torch.split(qkv, [Hq * hd, Hkv * hd, Hkv * hd], dim=-1)
            q = q.reshape(mb, seq, Hq, hd)
            k = k.reshape(mb, seq, Hkv, hd)
            v = v.reshape(mb, seq, Hkv, hd)
            if w.rope:
                q, k = rope(q), rope(k)
            k = k.repeat_interleave(Hq // Hkv, dim=2)
            v = v.repeat_interleave(Hq // Hkv, dim=2)
            o = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2),
                                               is_causal=True).transpose(1, 2).reshape(mb, seq, Hq * hd)
            x1 = xt + F.linear(o, lp["wo"], lp.get("bo"))
            n2 = norm(x1, lp["ln2_g"], lp.get("ln2_b"))
            h = F.linear(n2, lp["w1"], lp.get("b1"))
            if w.act == inp.ACT_SWIGLU:
                a = F.silu(h[..., :w.d_ffn]) * h[..., w.d_ffn:]
            else:
                a = F.gelu(h)
            xt = x1 + F.linear(a, lp["w2"], lp.get("b2"))
        if w.loss_head:
            hp = tp["head"]
            nf = norm(xt, hp["lnf_g"], hp.get("lnf_b"))
            z = F.linear(nf, hp["w_head"])
            return F.cross_entropy(z.reshape(mb * seq, -1), torch.tensor(tgt.reshape(-1), dtype=torch.long))
        return xt

    total = 0.0
    xts = []
    for i in range(w.n_microbatches):
        xt = torch.tensor(x[s][i], dtype=torch.float64, requires_grad=True)
        xts.append(xt)
        out = fwd(xt, None if tg is None else tg[i])
        total = total + (out if w.loss_head else (out * torch.tensor(cot[s][i])).sum())
    total.backward()
    G, dxs = accumulate(spec, P, x[s], cot[s], tg)
    for key, _ in leaves(P):
        ref = get_leaf(tp, key).grad.numpy()
        mine = get_leaf(G, key)
        assert np.linalg.norm(mine - ref) <= 1e-11 * max(1e-3, np.linalg.norm(ref)), key
    for i in range(w.n_microbatches):
        ref = xts[i].grad.numpy()
        assert np.linalg.norm(dxs[i] - ref) <= 1e-11 * np.linalg.norm(ref)


# ---------------------------------------------------------------- schedules

def test_interleaved_matches_paper_example():
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_sec4_2_task_lists.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, i, ty, s = line.split()
            rows.append((int(a), int(i), ty, int(s)))
    for actor in (0, 1):
        got = sch.interleaved_1f1b(2, actor, 2, 4)[:3]
        want = [(i, ty, s) for (a, i, ty, s) in rows if a == actor]
        assert got == want


@pytest.mark.parametrize("P,V,M", [(2, 2, 4), (4, 2, 8), (8, 2, 32), (4, 3, 8), (1, 2, 3)])
def test_interleaved_is_valid_for_every_rank(P, V, M):
    for r in range(P):
        tasks = sch.interleaved_1f1b(P, r, V, M)
        peak = sch.validate(tasks, [v * P + r for v in range(V)], M)
        assert len(tasks) == 2 * M * V
        assert peak <= min(M * V, (P - r - 1) * 2 + (V - 1) * P + 1)
        for s in {t[2] for t in tasks}:
            order = [i for (i, ty, st) in tasks if ty == "bwd" and st == s]
            assert order == sorted(order)


@pytest.mark.parametrize("P,M", [(4, 8), (4, 2), (8, 32), (1, 5)])
def test_1f1b_and_gpipe_are_valid_with_expected_peaks(P, M):
    for r in range(P):
        t = sch.one_f_one_b(P, r, M)
        assert sch.validate(t, [r], M) == min(P - r, M)
        assert [i for (i, ty, _) in t if ty == "bwd"] == list(range(M))
        g = sch.gpipe(P, r, M)
        assert sch.validate(g, [r], M) == M
    # last rank alternates strictly
    t = sch.one_f_one_b(P, P - 1, M)
    assert [ty for (_, ty, _) in t] == ["fwd", "bwd"] * M


def test_validator_rejects_bad_lists():
    good = sch.gpipe(1, 0, 2)
    with pytest.raises(ValueError):
        sch.validate(good[:-1], [0], 2)
    with pytest.raises(ValueError):
        sch.validate([(0, "bwd", 0), (0, "fwd", 0)], [0], 1)
    with pytest.raises(ValueError):
        sch.validate(good + [good[0]], [0], 2)
    with pytest.raises(ValueError):
        sch.validate([(0, "fwd", 1), (0, "bwd", 1)], [0], 1)


def test_flop_count_matches_hand_computed_values():
    """GPT-3-shaped layer: 2*T*(d*3d + d*d + 2*d*f) = 7.422 TF forward GEMMs and
    2*96*2048^2*128 = 0.103 TF causal attention per microbatch; x3 for fwd+bwd."""
    w = inp.C4
    f = so.algorithmic_flops_per_microbatch(spec_of(w))
    T, d, ff = 2048, 12288, 49152
    hand = 3 * (2 * T * (3 * d * d + d * d + 2 * d * ff) + 2 * 96 * 2048 ** 2 * 128)
    assert f == hand
    assert abs(2 * f / 1e12 - 45.15) < 0.01
