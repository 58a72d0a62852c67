"""fp64 CPU oracle for one pipeline stage (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It shares no code with the HIP library and never calls it.

What it defines.  The paper (Section 3.1, "Gradient Accumulation Loop") states
the semantics of the accumulation loop: gradients start at zero, each
microbatch's gradients are added (no 1/M), and per-microbatch losses are
collected as a vector.  Section 2.2.1 states that a schedule only changes the
order in which forward and backward tasks of (microbatch, stage) pairs run, and
that the backward of a stage runs where its forward ran.  The result of running
a task list is therefore, for every owned stage s with parameters theta_s,
inputs x_i and upstream cotangents c_i:

    y_i  = F_s(theta_s, x_i)
    dx_i = (dF_s/dx)^T c_i
    G_s  = sum_{i ascending} (dF_s/dtheta)^T c_i
    loss_i (last stage only) = CE(F_s(theta_s, x_i), targets_i), seeded by 1.

The paper does not define the layer mathematics (it only names GPT-3 and
Llama 2 in its Evaluation section); F_s is the standard pre-norm decoder
layer of those model families:

    n1 = Norm(x);  [q|k|v] = n1 Wqkv^T (+ bqkv);  q,k <- RoPE (optional)
    O  = causal softmax(q k^T / sqrt(hd)) v       (GQA: query head h reads
                                                    kv head h // (Hq/Hkv))
    x1 = x + O Wo^T (+ bo);  n2 = Norm(x1)
    GeLU:   y = x1 + gelu(n2 W1^T + b1) W2^T + b2       (gelu(t) = t Phi(t))
    SwiGLU: [g|u] = n2 W1^T;  y = x1 + (silu(g) * u) W2^T

with an optional loss head  nf = Norm(y_L); z = nf Whead^T; mean-token CE.

Everything is float64, written step by step with explicit per-(batch, head)
loops; score matrices are materialised in full; backward passes are written by
hand from the chain rule.  numpy's matmul and scipy's erf serve as library
steps.  Parity pins (finite differences, closed forms, invariants, an
independent autograd computation) live in tests/test_oracle_*.py.
"""
from dataclasses import dataclass, field
import math

import numpy as np
from scipy.special import erf as _erf

NORM_LAYERNORM = 0
NORM_RMSNORM = 1
ACT_GELU = 0        # exact, erf-based
ACT_GELU_TANH = 1
ACT_SWIGLU = 2


@dataclass
class StageSpec:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    seq_len: int
    microbatch: int
    norm: int = NORM_LAYERNORM
    act: int = ACT_GELU
    use_bias: bool = True
    rope: bool = False
    rope_theta: float = 10000.0
    norm_eps: float = 1e-5
    loss_head: bool = False
    vocab: int = 0


# --------------------------------------------------------------------------
# parameter naming / shapes (the oracle's own statement of the layout)
# --------------------------------------------------------------------------

def layer_param_shapes(spec):
    d, f = spec.d_model, spec.d_ffn
    nq = spec.n_q_heads * spec.head_dim
    nkv = spec.n_kv_heads * spec.head_dim
    f1 = 2 * f if spec.act == ACT_SWIGLU else f
    ln = spec.norm == NORM_LAYERNORM
    out = [("ln1_g", (d,))]
    if ln:
        out.append(("ln1_b", (d,)))
    out.append(("wqkv", (nq + 2 * nkv, d)))
    if spec.use_bias:
        out.append(("bqkv", (nq + 2 * nkv,)))
    out.append(("wo", (d, nq)))
    if spec.use_bias:
        out.append(("bo", (d,)))
    out.append(("ln2_g", (d,)))
    if ln:
        out.append(("ln2_b", (d,)))
    out.append(("w1", (f1, d)))
    if spec.use_bias:
        out.append(("b1", (f1,)))
    out.append(("w2", (d, f)))
    if spec.use_bias:
        out.append(("b2", (d,)))
    return out


def head_param_shapes(spec):
    out = [("lnf_g", (spec.d_model,))]
    if spec.norm == NORM_LAYERNORM:
        out.append(("lnf_b", (spec.d_model,)))
    out.append(("w_head", (spec.vocab, spec.d_model)))
    return out


# --------------------------------------------------------------------------
# elementwise pieces
# --------------------------------------------------------------------------

def norm_forward(spec, x, g, b):
    """LayerNorm: (x - mean)/sqrt(var + eps) * g + b with the biased variance;
    RMSNorm: x / sqrt(mean(x^2) + eps) * g.  Returns (y, xhat, rstd)."""
    if spec.norm == NORM_LAYERNORM:
        mu = x.mean(axis=-1, keepdims=True)
        var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
        rstd = 1.0 / np.sqrt(var + spec.norm_eps)
        xhat = (x - mu) * rstd
        return xhat * g + b, xhat, rstd
    ms = (x ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(ms + spec.norm_eps)
    xhat = x * rstd
    return xhat * g, xhat, rstd


def norm_backward(spec, dy, xhat, rstd, g):
    """Returns (dx, dg, db-or-None).  With dxhat = dy*g:
    LayerNorm: dx = rstd*(dxhat - mean(dxhat) - xhat*mean(dxhat*xhat));
    RMSNorm:   dx = rstd*(dxhat - xhat*mean(dxhat*xhat))."""
    dxhat = dy * g
    red = tuple(range(dy.ndim - 1))
    dg = (dy * xhat).sum(axis=red)
    proj = (dxhat * xhat).mean(axis=-1, keepdims=True)
    if spec.norm == NORM_LAYERNORM:
        db = dy.sum(axis=red)
        dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True) - xhat * proj)
        return dx, dg, db
    dx = rstd * (dxhat - xhat * proj)
    return dx, dg, None


def _phi_cdf(t):
    return 0.5 * (1.0 + _erf(t / math.sqrt(2.0)))


def _phi_pdf(t):
    return np.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)


_K0 = math.sqrt(2.0 / math.pi)
_K1 = 0.044715


def act_forward(spec, h):
    """h is [.., f] (GeLU) or [.., 2f] = [gate | up] (SwiGLU)."""
    if spec.act == ACT_GELU:
        return h * _phi_cdf(h)
    if spec.act == ACT_GELU_TANH:
        return 0.5 * h * (1.0 + np.tanh(_K0 * (h + _K1 * h ** 3)))
    f = spec.d_ffn
    gte, up = h[..., :f], h[..., f:]
    sig = 1.0 / (1.0 + np.exp(-gte))
    return gte * sig * up


def act_backward(spec, h, da):
    if spec.act == ACT_GELU:
        return da * (_phi_cdf(h) + h * _phi_pdf(h))
    if spec.act == ACT_GELU_TANH:
        u = _K0 * (h + _K1 * h ** 3)
        th = np.tanh(u)
        du = _K0 * (1.0 + 3.0 * _K1 * h * h)
        return da * (0.5 * (1.0 + th) + 0.5 * h * (1.0 - th * th) * du)
    f = spec.d_ffn
    gte, up = h[..., :f], h[..., f:]
    sig = 1.0 / (1.0 + np.exp(-gte))
    silu = gte * sig
    dsilu = sig * (1.0 + gte * (1.0 - sig))
    return np.concatenate([da * up * dsilu, da * silu], axis=-1)


def rope_tables(spec):
    """cos/sin of angle(t, j) = t * theta^(-2j/hd), t = position in the
    sequence (0-based), j in [0, hd/2)."""
    half = spec.head_dim // 2
    j = np.arange(half, dtype=np.float64)
    inv = spec.rope_theta ** (-2.0 * j / spec.head_dim)
    ang = np.arange(spec.seq_len, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(spec, t, transpose=False):
    """t: [mb, seq, H, hd].  Pairs element j with j + hd/2 (half-split) and
    rotates the pair by angle(t, j); transpose=True applies the inverse
    rotation, which is the backward pass of the forward rotation."""
    half = spec.head_dim // 2
    c, s = rope_tables(spec)
    c = c[None, :, None, :]
    s = s[None, :, None, :]
    if transpose:
        s = -s
    a, b = t[..., :half], t[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------

def attention_forward(spec, q, k, v):
    """q: [mb, seq, Hq, hd]; k, v: [mb, seq, Hkv, hd].
    Returns O [mb, seq, Hq, hd] and the probabilities P [mb, Hq, seq, seq]."""
    mb, seq, Hq, hd = q.shape
    group = Hq // spec.n_kv_heads
    scale = 1.0 / math.sqrt(hd)
    mask = np.tril(np.ones((seq, seq), dtype=bool))
    O = np.zeros_like(q)
    P = np.zeros((mb, Hq, seq, seq))
    for b in range(mb):
        for h in range(Hq):
            kv = h // group
            S = (q[b, :, h, :] @ k[b, :, kv, :].T) * scale
            S = np.where(mask, S, -np.inf)
            S = S - S.max(axis=-1, keepdims=True)
            e = np.exp(S)
            p = e / e.sum(axis=-1, keepdims=True)
            P[b, h] = p
            O[b, :, h, :] = p @ v[b, :, kv, :]
    return O, P


def attention_backward(spec, q, k, v, P, dO):
    mb, seq, Hq, hd = q.shape
    group = Hq // spec.n_kv_heads
    scale = 1.0 / math.sqrt(hd)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(mb):
        for h in range(Hq):
            kv = h // group
            p = P[b, h]
            do = dO[b, :, h, :]
            dv[b, :, kv, :] += p.T @ do
            dp = do @ v[b, :, kv, :].T
            ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
            dq[b, :, h, :] = (ds @ k[b, :, kv, :]) * scale
            dk[b, :, kv, :] += (ds.T @ q[b, :, h, :]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------
# one decoder layer
# --------------------------------------------------------------------------

def layer_forward(spec, p, x):
    """x: [mb, seq, d].  Returns (y, cache)."""
    mb, seq, d = x.shape
    Hq, Hkv, hd = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    nq, nkv = Hq * hd, Hkv * hd
    c = {"x": x}
    n1, c["xhat1"], c["rstd1"] = norm_forward(spec, x, p["ln1_g"], p.get("ln1_b", 0.0))
    c["n1"] = n1
    qkv = n1 @ p["wqkv"].T
    if spec.use_bias:
        qkv = qkv + p["bqkv"]
    q = qkv[..., :nq].reshape(mb, seq, Hq, hd)
    k = qkv[..., nq:nq + nkv].reshape(mb, seq, Hkv, hd)
    v = qkv[..., nq + nkv:].reshape(mb, seq, Hkv, hd)
    if spec.rope:
        q = rope_apply(spec, q)
        k = rope_apply(spec, k)
    c["q"], c["k"], c["v"] = q, k, v
    O, c["P"] = attention_forward(spec, q, k, v)
    O = O.reshape(mb, seq, nq)
    c["O"] = O
    x1 = x + O @ p["wo"].T
    if spec.use_bias:
        x1 = x1 + p["bo"]
    n2, c["xhat2"], c["rstd2"] = norm_forward(spec, x1, p["ln2_g"], p.get("ln2_b", 0.0))
    c["n2"] = n2
    h = n2 @ p["w1"].T
    if spec.use_bias:
        h = h + p["b1"]
    c["h"] = h
    a = act_forward(spec, h)
    c["a"] = a
    y = x1 + a @ p["w2"].T
    if spec.use_bias:
        y = y + p["b2"]
    return y, c


def layer_backward(spec, p, c, dy):
    """Returns (dx, grads) with grads keyed like the parameters."""
    mb, seq, d = dy.shape
    Hq, Hkv, hd = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    nq, nkv = Hq * hd, Hkv * hd
    T = mb * seq
    g = {}
    flat = lambda t: t.reshape(T, -1)
    # FFN down
    g["w2"] = flat(dy).T @ flat(c["a"])
    if spec.use_bias:
        g["b2"] = flat(dy).sum(axis=0)
    da = dy @ p["w2"]
    dh = act_backward(spec, c["h"], da)
    g["w1"] = flat(dh).T @ flat(c["n2"])
    if spec.use_bias:
        g["b1"] = flat(dh).sum(axis=0)
    dn2 = dh @ p["w1"]
    dx1n, g["ln2_g"], db = norm_backward(spec, dn2, c["xhat2"], c["rstd2"], p["ln2_g"])
    if db is not None:
        g["ln2_b"] = db
    dx1 = dy + dx1n
    # attention output projection
    g["wo"] = flat(dx1).T @ flat(c["O"])
    if spec.use_bias:
        g["bo"] = flat(dx1).sum(axis=0)
    dO = (dx1 @ p["wo"]).reshape(mb, seq, Hq, hd)
    dq, dk, dv = attention_backward(spec, c["q"], c["k"], c["v"], c["P"], dO)
    if spec.rope:
        dq = rope_apply(spec, dq, transpose=True)
        dk = rope_apply(spec, dk, transpose=True)
    dqkv = np.concatenate([dq.reshape(mb, seq, nq), dk.reshape(mb, seq, nkv),
                           dv.reshape(mb, seq, nkv)], axis=-1)
    g["wqkv"] = flat(dqkv).T @ flat(c["n1"])
    if spec.use_bias:
        g["bqkv"] = flat(dqkv).sum(axis=0)
    dn1 = dqkv @ p["wqkv"]
    dxn, g["ln1_g"], db = norm_backward(spec, dn1, c["xhat1"], c["rstd1"], p["ln1_g"])
    if db is not None:
        g["ln1_b"] = db
    return dx1 + dxn, g


# --------------------------------------------------------------------------
# loss head: final norm -> untied LM head -> mean token cross-entropy
# --------------------------------------------------------------------------

def head_forward(spec, hp, y, targets):
    """targets: int [mb, seq].  loss = -(1/T) sum_t log softmax(z_t)[tgt_t],
    T = tokens of this microbatch."""
    mb, seq, d = y.shape
    c = {}
    nf, c["xhat"], c["rstd"] = norm_forward(spec, y, hp["lnf_g"], hp.get("lnf_b", 0.0))
    c["nf"] = nf
    z = nf.reshape(mb * seq, d) @ hp["w_head"].T
    z = z - z.max(axis=-1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=-1, keepdims=True))
    tg = targets.reshape(-1)
    c["prob"] = np.exp(logp)
    c["tg"] = tg
    loss = -logp[np.arange(mb * seq), tg].mean()
    return loss, c


def head_backward(spec, hp, c, shape, dloss=1.0):
    mb, seq, d = shape
    T = mb * seq
    dz = c["prob"].copy()
    dz[np.arange(T), c["tg"]] -= 1.0
    dz *= dloss / T
    g = {"w_head": dz.T @ c["nf"].reshape(T, d)}
    dnf = (dz @ hp["w_head"]).reshape(mb, seq, d)
    dy, g["lnf_g"], db = norm_backward(spec, dnf, c["xhat"], c["rstd"], hp["lnf_g"])
    if db is not None:
        g["lnf_b"] = db
    return dy, g


# --------------------------------------------------------------------------
# one stage = n_layers layers (+ head); params = {"layers": [dict...], "head": dict}
# --------------------------------------------------------------------------

def stage_forward(spec, params, x, targets=None):
    caches = []
    for p in params["layers"]:
        x, c = layer_forward(spec, p, x)
        caches.append(c)
    if spec.loss_head:
        loss, hc = head_forward(spec, params["head"], x, targets)
        return loss, {"layers": caches, "head": hc, "shape": x.shape}
    return x, {"layers": caches}


def stage_backward(spec, params, cache, cot=None):
    """cot: cotangent of the stage output y (ignored when the stage ends in the
    loss, whose backward is seeded with dloss = 1)."""
    grads = {"layers": [None] * len(params["layers"])}
    if spec.loss_head:
        dy, grads["head"] = head_backward(spec, params["head"], cache["head"], cache["shape"])
    else:
        dy = cot
    for li in reversed(range(len(params["layers"]))):
        dy, grads["layers"][li] = layer_backward(spec, params["layers"][li], cache["layers"][li], dy)
    return dy, grads


def _tree_add(acc, g):
    """acc <- acc + g, leaf by leaf (the `grads += mugrads` of Section 3.1)."""
    if acc is None:
        return {"layers": [{k: v.copy() for k, v in lg.items()} for lg in g["layers"]],
                **({"head": {k: v.copy() for k, v in g["head"].items()}} if "head" in g else {})}
    for la, lg in zip(acc["layers"], g["layers"]):
        for k in la:
            la[k] = la[k] + lg[k]
    if "head" in g:
        for k in acc["head"]:
            acc["head"][k] = acc["head"][k] + g["head"][k]
    return acc


def run_task_list(spec, params_by_stage, tasks, x, cot=None, targets=None):
    """Execute a per-actor task list in the order given (Section 4.2).

    params_by_stage: {stage: params}; x[stage][i], cot[stage][i] are the
    activations and cotangents that other actors would have sent; targets[i]
    for a loss-head stage.  Forward tasks stash what the backward needs; the
    stash is dropped when the backward has run (Section 4.3).  Gradients start
    from zero and are summed over microbatches, losses are collected per
    microbatch (Section 3.1).

    Returns dict with y[stage][i] (or loss[stage][i]), dx[stage][i],
    grads[stage], peak_live."""
    stages = sorted(params_by_stage)
    M = len(next(iter(x.values())))
    out = {"y": {s: [None] * M for s in stages}, "dx": {s: [None] * M for s in stages},
           "loss": {s: [None] * M for s in stages}, "grads": {s: None for s in stages}}
    stash = {}
    peak = 0
    for (i, ty, s) in tasks:
        if ty == "fwd":
            assert (i, s) not in stash
            res, cache = stage_forward(spec, params_by_stage[s], x[s][i],
                                       None if targets is None else targets[i])
            if spec.loss_head:
                out["loss"][s][i] = res
            else:
                out["y"][s][i] = res
            stash[(i, s)] = cache
            peak = max(peak, len(stash))
        else:
            cache = stash.pop((i, s))
            c = None if spec.loss_head else cot[s][i]
            dx, g = stage_backward(spec, params_by_stage[s], cache, c)
            out["dx"][s][i] = dx
            out["grads"][s] = _tree_add(out["grads"][s], g)
    assert not stash
    out["peak_live"] = peak
    return out


# --------------------------------------------------------------------------
# FLOP count used for reporting (not part of the method)
# --------------------------------------------------------------------------

def algorithmic_flops_per_microbatch(spec):
    """2*T*d_in*d_out per linear map, x3 (forward, input grad, weight grad);
    causal attention counted at half of the full score matrix: forward
    2*mb*Hq*seq^2*hd, backward twice that; norms/activations not counted."""
    T = spec.microbatch * spec.seq_len
    total = 0.0
    for name, shp in layer_param_shapes(spec):
        if len(shp) == 2:
            total += 2.0 * T * shp[0] * shp[1]
    total *= 3.0
    total += 3.0 * 2.0 * spec.microbatch * spec.n_q_heads * spec.seq_len ** 2 * spec.head_dim
    total *= spec.n_layers
    if spec.loss_head:
        total += 3.0 * 2.0 * T * spec.d_model * spec.vocab
    return total
