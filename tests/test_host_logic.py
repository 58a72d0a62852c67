"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host-side schedule generators / validator behave as the paper's
Sections 2.2.1 and 4.2 require.  No compute entry point is called here."""
import ctypes as C
import os
import re

import numpy as np

import pytest

from oracle import schedules as osch
from paper_2412_14374_amd import binding as B
from paper_2412_14374_amd import inputs as inp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "jpp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(jpp_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert "jpp_stage_create" in names and "jpp_stage_run" in names and "jpp_stage_grads" in names
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in jpp.h but not exported"
    assert set(names) == set(B.exported_names()), "binding and header disagree"


def as_oracle(tasks):
    return [(i, "fwd" if ty == B.JPP_FWD else "bwd", s) for (i, ty, s) in tasks]


def test_interleaved_generator_reproduces_paper_example():
    rows = []
    with open(os.path.join(ROOT, "tests", "golden", "paper_sec4_2_task_lists.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, i, ty, s = line.split()
            rows.append((int(a), int(i), ty, int(s)))
    for actor in (0, 1):
        got = as_oracle(B.jpp_schedule_make(inp.SCHED_INTERLEAVED, 2, actor, 2, 4))[:3]
        assert got == [(i, ty, s) for (a, i, ty, s) in rows if a == actor]


@pytest.mark.parametrize("P,M", [(1, 1), (1, 5), (4, 8), (4, 2), (8, 32), (3, 7)])
def test_gpipe_and_1f1b_agree_with_independent_generators(P, M):
    for r in range(P):
        assert as_oracle(B.jpp_schedule_make(inp.SCHED_GPIPE, P, r, 1, M)) == osch.gpipe(P, r, M)
        assert as_oracle(B.jpp_schedule_make(inp.SCHED_1F1B, P, r, 1, M)) == osch.one_f_one_b(P, r, M)


@pytest.mark.parametrize("P,V,M", [(2, 2, 4), (4, 2, 8), (8, 2, 32), (4, 3, 8), (1, 2, 3), (8, 6, 32)])
def test_interleaved_agrees_with_independent_generator(P, V, M):
    for r in range(P):
        assert as_oracle(B.jpp_schedule_make(inp.SCHED_INTERLEAVED, P, r, V, M)) == osch.interleaved_1f1b(P, r, V, M)


def cfg_for(stage_ids):
    class W:
        pass
    w = W()
    for k, v in dict(dtype=0, n_layers=1, d_model=16, n_q_heads=2, n_kv_heads=2, head_dim=8, d_ffn=32, seq_len=8,
                     microbatch=1, norm=0, act=0, use_bias=1, rope=0, rope_theta=10000.0, norm_eps=1e-5,
                     loss_head=0, vocab=0).items():
        setattr(w, k, v)
    w.stage_ids = stage_ids
    return B.make_config(w)


def test_validator_peaks_follow_section_2_2_1():
    """GPipe keeps M stashes alive, 1F1B min(P - rank, M)."""
    for P, M in [(4, 8), (8, 32), (4, 2)]:
        for r in range(P):
            cfg = cfg_for([r])
            assert B.jpp_schedule_validate(cfg, M, B.jpp_schedule_make(inp.SCHED_GPIPE, P, r, 1, M)) == M
            assert B.jpp_schedule_validate(cfg, M, B.jpp_schedule_make(inp.SCHED_1F1B, P, r, 1, M)) == min(P - r, M)
    cfg = cfg_for([0, 8])
    peak = B.jpp_schedule_validate(cfg, 32, B.jpp_schedule_make(inp.SCHED_INTERLEAVED, 8, 0, 2, 32))
    assert peak == osch.validate(osch.interleaved_1f1b(8, 0, 2, 32), [0, 8], 32) == 23


def test_validator_counts_group_places():
    """With weight-gradient groups of g a group holds g stash places from its first forward to
    its last backward; checked against a brute-force count over the generated lists."""
    def brute(tasks, M, g):
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
        return hi
    for kind, P, r, V, M in [(inp.SCHED_GPIPE, 4, 1, 1, 7), (inp.SCHED_1F1B, 4, 0, 1, 8), (inp.SCHED_1F1B, 4, 3, 1, 5),
                             (inp.SCHED_INTERLEAVED, 8, 0, 2, 32), (inp.SCHED_INTERLEAVED, 2, 1, 3, 6)]:
        ids = [v * P + r for v in range(V)]
        tasks = B.jpp_schedule_make(kind, P, r, V, M)
        for g in (1, 2, 3, 4, 8, M):
            if g > M:
                continue
            cfg = cfg_for(ids)
            cfg.wgrad_group = g
            assert B.jpp_schedule_validate(cfg, M, tasks) == brute(tasks, M, g), (kind, P, r, V, M, g)
    # the benchmark's schedule: groups of 8 = one run of backwards of a virtual stage
    cfg = cfg_for([0, 8])
    cfg.wgrad_group = 8
    assert B.jpp_schedule_validate(cfg, 32, B.jpp_schedule_make(inp.SCHED_INTERLEAVED, 8, 0, 2, 32)) == 32


def test_validator_rejects_rule_violations():
    cfg = cfg_for([0])
    good = B.jpp_schedule_make(inp.SCHED_GPIPE, 1, 0, 1, 2)
    bad_lists = {
        "incomplete": good[:-1],
        "bwd before fwd": [(0, 1, 0), (0, 0, 0)],
        "duplicate": good[:2] + [good[0]] + good[2:],
        "unknown stage": [(0, 0, 5), (0, 1, 5)],
        "microbatch range": [(0, 0, 0), (2, 0, 0), (0, 1, 0), (2, 1, 0)],
        "bad type": [(0, 0, 0), (0, 7, 0), (1, 0, 0), (1, 1, 0)],
    }
    for why, tasks in bad_lists.items():
        with pytest.raises(B.JppError) as e:
            B.jpp_schedule_validate(cfg, 2, tasks)
        assert e.value.status == B.JPP_ESCHED, why


def test_schedule_argument_errors():
    assert B.jpp_schedule_len(inp.SCHED_INTERLEAVED, 4, 0, 2, 6) == -1      # M % P != 0
    assert B.jpp_schedule_len(inp.SCHED_1F1B, 4, 4, 1, 8) == -1             # rank out of range
    assert B.jpp_schedule_len(inp.SCHED_GPIPE, 4, 0, 2, 8) == -1            # V > 1 only for interleaved
    assert B.jpp_schedule_len(inp.SCHED_INTERLEAVED, 8, 0, 2, 32) == 128
    with pytest.raises(B.JppError):
        B.jpp_schedule_make(9, 1, 0, 1, 1)


def test_arena_size_and_config_errors():
    for name, w in inp.CONFIGS.items():
        cfg = B.make_config(w)
        n = B.jpp_stage_arena_bytes(cfg, w.n_microbatches, 4)
        esz = 2 if w.dtype == inp.DT_BF16 else 4
        T = w.tokens
        f1 = 2 * w.d_ffn if w.act == inp.ACT_SWIGLU else w.d_ffn
        nqkv = (w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim
        stash = w.n_layers * T * esz * (5 * w.d_model + nqkv + w.n_q_heads * w.head_dim + f1 + w.d_ffn)
        assert n > 4 * stash, name
        assert n < 288e9, name                         # fits one MI355X
    bad = B.make_config(inp.C1)
    bad.n_kv_heads = 3
    with pytest.raises(B.JppError) as e:
        B.jpp_stage_arena_bytes(bad, 4, 4)
    assert e.value.status == B.JPP_EINVAL
    bad = B.make_config(inp.C2)
    bad.d_model = 2052                                  # not a multiple of 8 in bf16 mode
    with pytest.raises(B.JppError):
        B.jpp_stage_arena_bytes(bad, 8, 4)


def test_pipeline_merge_order_matches_the_oracle_and_reports_deadlocks():
    """The host-side merge of several actors' lists (Section 4.2: tasks are walked in a
    topological order of the task graph) against the oracle's, which uses the same round-robin
    rule; every task follows its producer; cyclic lists are refused."""
    from oracle import pipeline_oracle as po
    for P, V, M in [(2, 2, 4), (4, 2, 8), (3, 1, 5), (1, 2, 3)]:
        if V > 1 or P == 1:
            lists = [osch.interleaved_1f1b(P, r, V, M) for r in range(P)] if M % P == 0 else None
        if V == 1 and P > 1:
            lists = [osch.one_f_one_b(P, r, M) for r in range(P)]
        if lists is None:
            lists = [[(i, "fwd", v * P + r) for v in range(V) for i in range(M)] +
                     [(i, "bwd", v * P + r) for v in reversed(range(V)) for i in range(M)] for r in range(P)]
        got = B.jpp_pipeline_merge_order(P, V, M, lists)
        want = [r for (r, _) in po.global_order(lists, P * V)]
        assert got == want
    bad0 = [(0, "fwd", 2), (0, "fwd", 0), (0, "bwd", 2), (0, "bwd", 0)]
    good1 = [(0, "fwd", 1), (0, "fwd", 3), (0, "bwd", 3), (0, "bwd", 1)]
    with pytest.raises(B.JppError) as e:
        B.jpp_pipeline_merge_order(2, 2, 1, [bad0, good1])
    assert e.value.status == B.JPP_ESCHED and "deadlock" in str(e.value) and "actor 0" in str(e.value)
    with pytest.raises(B.JppError) as e:
        B.jpp_pipeline_merge_order(2, 2, 1, [[(0, "fwd", 1)], good1])      # stage 1 is not actor 0's
    assert e.value.status == B.JPP_ESCHED


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one stage on one GPU: --gpus above 1 ends with a message and a
    non-zero status before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_normal_tail_fit_reproduces_the_kernel_coefficients_and_error():
    """The coefficient list of normal_cdf_fit in device_utils.h is what normal_tail_fit.py
    computes, and the fp32 evaluation of that polynomial stays within 3e-7 of the cumulative
    normal (so within 5e-7 of the erf-form GeLU over [-8, 8]), far below bf16 rounding."""
    import importlib.util
    import re
    from scipy.special import erf
    here = os.path.dirname(os.path.abspath(__file__))
    csrc = os.path.join(here, "..", "paper_2412_14374_amd", "csrc")
    spec = importlib.util.spec_from_file_location("normal_tail_fit", os.path.join(csrc, "normal_tail_fit.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    coef = mod.fit()
    src = open(os.path.join(csrc, "device_utils.h")).read()
    body = src[src.index("inline float normal_cdf_fit"):src.index("inline float gelu_erf_fit")]
    in_kernel = [float(x) for x in re.findall(r"(-?\d\.\d+e[+-]\d+)f", body)]
    assert len(in_kernel) == len(coef) == 9
    for have, want in zip(in_kernel, coef[::-1]):       # Horner: highest power first
        assert np.float32(have) == np.float32(want), (have, want)
    h = np.linspace(-8, 8, 200001).astype(np.float32)
    exact = 0.5 * (1 + erf(h.astype(np.float64) / np.sqrt(2.0)))
    phi = mod.normal_cdf_f32(coef, h)
    assert np.abs(phi - exact).max() < 3e-7
    assert np.abs(h * phi - h * exact).max() < 5e-7
