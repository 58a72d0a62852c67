"""Oracle-side pipeline schedules (TEST INFRASTRUCTURE ONLY).

This file is part of the CPU oracle.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product library has its own,
independently written generators in C++.

A schedule for one actor is a list of (i, ty, stage) triples -- the Task(i, ty,
stage) records of the paper's Section 4.2 ("Task Scheduling"): i is the
gradient-accumulation iteration (microbatch), ty is 'fwd' or 'bwd', stage is the
global stage index.  Section 2.2.1 ("The Importance of Pipeline Schedules")
describes the three orders generated here:

* GPipe: every forward of every microbatch, then every backward.
* 1F1B: backward tasks are run eagerly, so that the number of live activation
  sets is bounded by the number of stages rather than microbatches.
* Interleaved 1F1B ("circular repeat"): each actor owns several stages.

The paper's figures are not available, so the exact block order of 1F1B and
interleaved 1F1B follows the published definitions of those schedules
(PipeDream-flush and Megatron's interleaved schedule); the interleaved order is
pinned by the two-actor, four-stage example printed in Section 4.2.

Every generator emits, for each owned stage, the backward tasks in ascending
microbatch order, so a running fp accumulation G <- G + g_i has one
association in every schedule.
"""

FWD = "fwd"
BWD = "bwd"


def gpipe(P, rank, M):
    """All forwards for i = 0..M-1, then all backwards for i = 0..M-1, on the
    single stage `rank` owned by this actor (Section 2.2.1, GPipe paragraph)."""
    assert 0 <= rank < P and M >= 1
    return [(i, FWD, rank) for i in range(M)] + [(i, BWD, rank) for i in range(M)]


def one_f_one_b(P, rank, M):
    """1F1B for actor `rank` of P (Section 2.2.1, 1F1B paragraph).

    The actor first runs enough forwards to fill the pipeline below it
    (P - rank - 1 of them, or M if there are fewer microbatches), then
    alternates one forward with one backward, then drains the remaining
    backwards.  Live activation sets never exceed min(P - rank, M)."""
    assert 0 <= rank < P and M >= 1
    warm = min(P - rank - 1, M)
    out = []
    f = b = 0
    for _ in range(warm):
        out.append((f, FWD, rank)); f += 1
    while f < M:
        out.append((f, FWD, rank)); f += 1
        out.append((b, BWD, rank)); b += 1
    while b < M:
        out.append((b, BWD, rank)); b += 1
    return out


def _interleaved_chunk(k, P, V, forward):
    """k-th forward (or backward) unit of work of an actor under the interleaved
    schedule -> (microbatch, local virtual-stage index).

    Units are taken in groups of P*V; inside a group the actor sweeps P
    consecutive microbatches through its first virtual stage, then the same P
    microbatches through its second one, and so on (backward: last virtual
    stage first)."""
    group, within = divmod(k, P * V)
    v = within // P
    if not forward:
        v = V - 1 - v
    i = group * P + within % P
    return i, v


def interleaved_1f1b(P, rank, V, M):
    """Interleaved 1F1B with circular repeat V for actor `rank` of P (Section
    2.2.1 last paragraph; example in Section 4.2).  Global stage index of local
    virtual stage v is v*P + rank.  Requires M to be a multiple of P."""
    assert 0 <= rank < P and V >= 1 and M >= 1
    if M % P != 0:
        raise ValueError("interleaved 1F1B needs M to be a multiple of P")
    total = M * V
    warm = min((P - rank - 1) * 2 + (V - 1) * P, total)
    out = []

    def emit(k, forward):
        i, v = _interleaved_chunk(k, P, V, forward)
        out.append((i, FWD if forward else BWD, v * P + rank))

    for k in range(warm):
        emit(k, True)
    for j in range(total - warm):
        emit(warm + j, True)
        emit(j, False)
    for j in range(total - warm, total):
        emit(j, False)
    return out


def validate(tasks, owned_stages, M):
    """Check a task list against the rules of Section 2.2.1 (forward and
    backward of a stage live on the same actor; data dependencies honoured):
    every (i, ty, stage) with stage owned and 0 <= i < M appears exactly once
    and bwd(i, s) comes after fwd(i, s).  Returns the peak number of
    (microbatch, stage) activation sets alive at once."""
    owned = set(owned_stages)
    seen = set()
    live = 0
    peak = 0
    for (i, ty, s) in tasks:
        if s not in owned:
            raise ValueError(f"stage {s} not owned")
        if not (0 <= i < M):
            raise ValueError(f"microbatch {i} out of range")
        if ty not in (FWD, BWD):
            raise ValueError(f"bad task type {ty}")
        if (i, ty, s) in seen:
            raise ValueError(f"duplicate task {(i, ty, s)}")
        if ty == BWD and (i, FWD, s) not in seen:
            raise ValueError(f"bwd before fwd for {(i, s)}")
        seen.add((i, ty, s))
        if ty == FWD:
            live += 1
            peak = max(peak, live)
        else:
            live -= 1
    if len(seen) != 2 * M * len(owned):
        raise ValueError("task list incomplete")
    return peak
