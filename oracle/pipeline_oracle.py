"""CPU oracle for a whole pipeline: several actors, each with its own task list.

TEST INFRASTRUCTURE ONLY.  Plain float64 numpy; shares nothing with the HIP library.  Only
tests, the smoke check and the benchmark's CPU leg may import this module.

What it computes is a plain definition.  The model is the composition of S stages,
stage s placed on actor s mod P (the circular placement of Section 2.2.1); for every
microbatch i

    a_0 = x_i,  a_{s+1} = F_s(theta_s, a_s),  loss_i = CE(head(a_S), targets_i)
    (or, without a loss head, the cotangent of a_S is given),

and the result is the per-microbatch loss vector, the gradient of every stage summed over
the microbatches without 1/M (Section 3.1) and the cotangent of x_i.  The schedule (one
task list per actor, Section 4.2) only fixes the order: `global_order` merges the lists into
one order in which every task runs after the task that produces its operand, which is how
the paper places the send/receive pairs ("in their topological order", Section 4.2), and
reports a deadlock when the lists wait for each other in a cycle.

Every function here is pinned by tests/test_pipeline_oracle_pins.py: against the
single deep stage of oracle/stage_oracle.py, the example of Section 4.2, bitwise schedule
invariance and hand-made deadlocks.
"""
from dataclasses import replace

from . import stage_oracle as so


class Deadlock(Exception):
    """The actors' task lists wait for each other in a cycle (Section 4.2)."""


def actor_of(stage, P):
    return stage % P


def producer_of(task, S):
    """The task on another (or the same) actor whose result `task` consumes, or None.
    fwd(i, s) reads the output of fwd(i, s-1); bwd(i, s) reads the input cotangent produced by
    bwd(i, s+1); the first forward and the last backward read the pipeline's own inputs."""
    i, ty, s = task
    if ty == "fwd":
        return (i, "fwd", s - 1) if s > 0 else None
    return (i, "bwd", s + 1) if s < S - 1 else None


def global_order(task_lists, S):
    """Merge per-actor lists into one order: repeatedly, every actor in turn runs its next
    task if that task's producer has run (and, for a backward, its own forward, which
    validate() of the single-actor oracle already demands).  Returns [(actor, task)].
    Raises Deadlock naming the blocked tasks when no actor can move."""
    nxt = [0] * len(task_lists)
    done = set()
    order = []
    total = sum(len(l) for l in task_lists)
    while len(order) < total:
        moved = False
        for r, lst in enumerate(task_lists):
            if nxt[r] == len(lst):
                continue
            t = lst[nxt[r]]
            need = producer_of(t, S)
            own_fwd = (t[0], "fwd", t[2])
            if (need is None or need in done) and (t[1] == "fwd" or own_fwd in done):
                done.add(t)
                order.append((r, t))
                nxt[r] += 1
                moved = True
        if not moved:
            blocked = [(r, lst[nxt[r]]) for r, lst in enumerate(task_lists) if nxt[r] < len(lst)]
            raise Deadlock("no actor can run its next task: %r" % (blocked,))
    return order


def run_pipeline(spec, params_by_stage, task_lists, x0, targets=None, cot_last=None):
    """spec: StageSpec of one stage (n_layers = layers per stage); spec.loss_head says whether
    the LAST stage ends with the loss head, every other stage has none.
    params_by_stage: {s: params} for s = 0..S-1.  task_lists[r]: list of (i, ty, stage) of
    actor r, stage % P == r.  x0[i]: inputs of stage 0; targets[i] (loss head) or cot_last[i]
    (cotangent of the last stage's output).

    Returns dict: loss[i] or y[i]; dx[i] (cotangent of x0[i]); grads[s]; order (the global
    order used); peak_live[r] (stashes alive at once on actor r)."""
    S = len(params_by_stage)
    P = len(task_lists)
    M = len(x0)
    for r, lst in enumerate(task_lists):
        for (i, ty, s) in lst:
            assert 0 <= s < S and actor_of(s, P) == r and 0 <= i < M
    body = replace(spec, loss_head=False)
    order = global_order(task_lists, S)
    act, cot, stash = {}, {}, {}
    live, peak = [0] * P, [0] * P
    out = {"loss": [None] * M, "y": [None] * M, "dx": [None] * M,
           "grads": {s: None for s in range(S)}, "order": order}
    for r, (i, ty, s) in order:
        sp = spec if s == S - 1 else body
        if ty == "fwd":
            xin = x0[i] if s == 0 else act.pop((s - 1, i))
            res, cache = so.stage_forward(sp, params_by_stage[s], xin,
                                          targets[i] if sp.loss_head else None)
            if s == S - 1:
                out["loss" if sp.loss_head else "y"][i] = res
            else:
                act[(s, i)] = res
            stash[(s, i)] = cache
            live[r] += 1
            peak[r] = max(peak[r], live[r])
        else:
            if s == S - 1:
                c = None if sp.loss_head else cot_last[i]
            else:
                c = cot.pop((s, i))
            dx, g = so.stage_backward(sp, params_by_stage[s], stash.pop((s, i)), c)
            out["grads"][s] = so._tree_add(out["grads"][s], g)
            if s == 0:
                out["dx"][i] = dx
            else:
                cot[(s - 1, i)] = dx
            live[r] -= 1
    assert not stash and not act and not cot
    out["peak_live"] = peak
    return out
