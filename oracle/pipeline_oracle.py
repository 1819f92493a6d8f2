"""CPU oracle for the multi-stage side of the DAPPLE schedule: who runs what when.

THIS IS TEST INFRASTRUCTURE, not a product path: only the tests, the smoke
check and the benchmark may call it.  It shares no code with the HIP library and
imports nothing from it.

Three things, each written from the paper's definitions in plain Python:

  * `stage_lists`   -- the task list of every stage of an S-stage pipeline: stage i
                       injects K_i micro-batches and then alternates one backward, one
                       forward (section V-C; K_i from policy A or B);
  * `simulate`      -- what those lists mean in time when every stage is its own device:
                       a task starts when its stage is free, the task before it in the
                       stage's list has finished (control edges, section V-C) and its data
                       has arrived (F_{i,m} needs F_{i-1,m}; B_{i,m} needs B_{i+1,m}, the
                       last stage's B_m its own F_m) -- the definition of the trapezoid of
                       section IV-A written out, no more;
  * `latency_model` -- the planner's estimate L = T_w + T_s + T_e (equations 1 and 2 of
                       section IV-A) with the AllReduce term at zero, and `pivot_stage`, the
                       rule of section IV-B-1 that picks Q.

Pins (tests/test_oracle_pipeline.py): a two-stage, three-micro-batch timeline worked by
hand from the control edges the paper's scheduling figure names; the closed form
(M + S - 1)(f + b) for equal stages; the paper's statement that the early-backward order
has the same bubble time as the all-forward-then-all-backward order; the model as a
lower bound of the simulated time (it follows one dependency path) that is met when the
last stage is the slowest; peak residency K_i per stage.
"""
from __future__ import annotations

from oracle.stage_oracle import EARLY_BACKWARD, GPIPE, schedule_ops, warmup_depth


def warmup_depths(S: int, M: int, policy: str, D: int | None = None):
    """K_i for every stage (section V-C): policy A or B, capped by the D micro-batches
    that fit in memory and by the M micro-batches there are."""
    D = M if D is None else D
    return [max(1, min(warmup_depth(policy, S, i, D), M)) for i in range(S)]


def stage_lists(S: int, M: int, K, order: int = EARLY_BACKWARD):
    """One task list per stage; K: the S warm-up depths (ignored for the GPipe order)."""
    return [schedule_ops(M, K[i] if order == EARLY_BACKWARD else M, order) for i in range(S)]


def simulate(F, B, M: int, lists, comm: float = 0.0):
    """Timeline of one iteration with every stage on a device of its own.

    F[i], B[i]: duration of one forward / backward task of stage i; comm: time a boundary
    tensor takes from one stage to the next (either direction).  Returns a dict with
    start / end times per (kind, stage, micro-batch), the makespan, and per stage the busy
    time, the idle time inside the iteration ("bubble") and the peak number of resident
    micro-batches.  Raises if the lists cannot all complete (a deadlock)."""
    S = len(lists)
    end, start = {}, {}
    pos = [0] * S
    free = [0.0] * S
    live = [0] * S
    peak = [0] * S
    remaining = sum(len(l) for l in lists)
    while remaining:
        progressed = False
        for i in range(S):
            while pos[i] < len(lists[i]):
                kind, m = lists[i][pos[i]]
                if kind == "F":
                    dep = None if i == 0 else ("F", i - 1, m)
                else:
                    dep = ("F", i, m) if i == S - 1 else ("B", i + 1, m)
                if dep is not None and dep not in end:
                    break
                ready = 0.0 if dep is None else end[dep] + (comm if dep[1] != i else 0.0)
                t0 = max(free[i], ready)
                t1 = t0 + (F[i] if kind == "F" else B[i])
                start[(kind, i, m)], end[(kind, i, m)] = t0, t1
                free[i] = t1
                live[i] += 1 if kind == "F" else -1
                peak[i] = max(peak[i], live[i])
                pos[i] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("the task lists deadlock: no stage can run its next task")
    makespan = max(end.values())
    busy = [M * (F[i] + B[i]) for i in range(S)]
    return {"start": start, "end": end, "makespan": makespan, "busy": busy,
            "bubble": [makespan - b for b in busy], "peak_live": peak}


def pivot_stage(F, B, M: int) -> int:
    """Q by the rule of section IV-B-1: start at the last stage, walk s towards stage 0 and
    move Q to s when the steady phase of s alone, (M-1)(F_s+B_s), is longer than the steady
    phase of the current Q plus the forward and backward work of the stages between them."""
    S = len(F)
    Q = S - 1
    for s in range(S - 2, -1, -1):
        between = sum(F[a] + B[a] for a in range(s + 1, Q))
        if (M - 1) * (F[s] + B[s]) > (M - 1) * (F[Q] + B[Q]) + between:
            Q = s
    return Q


def latency_model(F, B, M: int, Q: int | None = None) -> float:
    """L = T_w + T_s + T_e (equations 1 and 2, section IV-A) with AR = 0:
    T_w = sum_{s<=Q} F_s;  T_s = (M-1)(F_Q + B_Q);
    T_e = max over s of (sum_{a=s..Q} B_a for s <= Q;  -sum_{a=Q..s} B_a for s > Q).
    Reading: the printed case split puts s = Q on the negative side, which would end a
    one-stage pipeline before its last backward; T_s leaves out one forward and one backward
    of the pivot, so the pivot's last backward belongs to the ending phase and s = Q is
    taken with the positive side.  With AR = 0 the negative side never is the maximum."""
    S = len(F)
    if Q is None:
        Q = pivot_stage(F, B, M)
    T_w = sum(F[s] for s in range(Q + 1))
    T_s = (M - 1) * (F[Q] + B[Q])
    T_e = max((sum(B[a] for a in range(s, Q + 1)) if s <= Q else -sum(B[a] for a in range(Q, s + 1)))
              for s in range(S))
    return T_w + T_s + T_e
