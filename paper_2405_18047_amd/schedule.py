"""Host-side pipeline-schedule simulator for 2-stage backpropagation (no GPU involved).

Given the per-stage times of forward, backward-p1 and backward-p2 (for example the ones bench.py measures on
an MI355X) it plays the paper's four schedules (Section 3.2: naive, GPipe, 1F1B-1, 1F1B-2) with and without 2BP
on N pipeline stages and returns the makespan, the bubble ratio (idle time / total time, Section 3.2) and the
throughput gain of 2BP.  Under the paper's assumption of equal forward / p1 / p2 times it reproduces the closed
forms of Table 1 exactly; with measured times it predicts what 2BP would buy on this hardware.

Model: stage s runs forward(mb) after stage s-1 did, backward(mb) after stage s+1 did (the last stage right after
its own forward); transfers are free; an operation is never pre-empted.  Every stage walks a fixed order of
forwards and backwards given by the schedule.  Without 2BP a backward costs t_p1 + t_p2.  With 2BP a backward
costs t_p1 and leaves one p2 pending; whenever a stage would idle because its next operation is not ready yet it
runs a pending p2 instead (the gap filling of Section 3.2), and whatever is still pending at the end is run as one
concatenated p2 (same total time as one by one).
"""
from __future__ import annotations

import dataclasses
from fractions import Fraction

SCHEDULES = ("naive", "gpipe", "1f1b-1", "1f1b-2")


@dataclasses.dataclass
class Result:
    makespan: Fraction
    busy_per_stage: list
    bubble_ratio: Fraction       # idle / total, averaged over stages (all stages do the same work here)
    peak_pending_p2: list        # per stage: largest number of micro-batches whose p2 operands were held at once


def _orders(schedule: str, n: int):
    """Per stage: list of ('F', mb) / ('B', mb) in execution order, and the number of micro-batches."""
    if schedule == "naive":
        m = 1
    elif schedule in ("gpipe", "1f1b-1"):
        m = n
    elif schedule == "1f1b-2":
        m = 2 * n
    else:
        raise ValueError(f"unknown schedule {schedule!r}")
    orders = []
    for s in range(n):
        if schedule in ("naive", "gpipe"):
            order = [("F", mb) for mb in range(m)] + [("B", mb) for mb in range(m)]
        else:                                   # one-forward-one-backward with n - s - 1 warm-up forwards
            warm = min(n - s - 1, m)
            order = [("F", mb) for mb in range(warm)]
            f, b = warm, 0
            while f < m:
                order.append(("F", f)); f += 1
                order.append(("B", b)); b += 1
            while b < m:
                order.append(("B", b)); b += 1
        orders.append(order)
    return orders, m


def simulate(schedule: str, n_stages: int, t_fwd=1, t_p1=1, t_p2=1, two_bp: bool = True) -> Result:
    tf, t1, t2 = Fraction(t_fwd), Fraction(t_p1), Fraction(t_p2)
    orders, m = _orders(schedule, n_stages)
    n = n_stages
    done = {}                                    # (kind, mb, stage) -> finish time
    pos = [0] * n                                # next index into the stage's order
    free_at = [Fraction(0)] * n
    pending = [0] * n                            # p2 operations whose operands are held
    peak = [0] * n
    busy = [Fraction(0)] * n
    now = Fraction(0)
    while True:
        progressed = False
        for s in range(n):
            if free_at[s] > now:
                continue
            if pos[s] < len(orders[s]):
                kind, mb = orders[s][pos[s]]
                if kind == "F":
                    dep = done.get(("F", mb, s - 1)) if s > 0 else Fraction(0)
                else:
                    dep = done.get(("B", mb, s + 1)) if s < n - 1 else done.get(("F", mb, s))
                    own = done.get(("F", mb, s))
                    dep = None if (dep is None or own is None) else max(dep, own)
                if dep is not None and dep <= now:
                    dur = tf if kind == "F" else (t1 if two_bp else t1 + t2)
                    free_at[s] = now + dur
                    busy[s] += dur
                    done[(kind, mb, s)] = free_at[s]
                    pos[s] += 1
                    if kind == "B" and two_bp:
                        pending[s] += 1
                        peak[s] = max(peak[s], pending[s])
                    progressed = True
                    continue
                if two_bp and pending[s] > 0:    # fill the gap with one deferred weight-gradient computation
                    free_at[s] = now + t2
                    busy[s] += t2
                    pending[s] -= 1
                    progressed = True
                    continue
            elif two_bp and pending[s] > 0:      # everything else done: the rest as one concatenated p2
                free_at[s] = now + t2 * pending[s]
                busy[s] += t2 * pending[s]
                pending[s] = 0
                progressed = True
        if all(pos[s] == len(orders[s]) and pending[s] == 0 for s in range(n)):
            break
        future = [t for t in free_at if t > now] + [t for t in done.values() if t > now]
        if not future:
            if not progressed:
                raise RuntimeError("schedule deadlocked")
            continue
        now = min(future)
    total = max(free_at)
    idle = sum(total - b for b in busy)
    return Result(total, busy, idle / (total * n), peak)


def throughput_gain(schedule: str, n_stages: int, t_fwd=1, t_p1=1, t_p2=1) -> Fraction:
    """Makespan without 2BP / makespan with 2BP (= (1 - b) / (1 - a) of Section 3.2 when the work is equal)."""
    a = simulate(schedule, n_stages, t_fwd, t_p1, t_p2, two_bp=False)
    b = simulate(schedule, n_stages, t_fwd, t_p1, t_p2, two_bp=True)
    return a.makespan / b.makespan


def table1(n: int) -> dict:
    """The closed forms of Table 1 (bubble ratio without 2BP, with 2BP, throughput gain) as exact fractions."""
    F = Fraction
    return {
        "naive": (F(n - 1, n), F(2 * (n - 1), 2 * n + 1), F(3 * n, 2 * n + 1)),
        "gpipe": (F(n - 1, 2 * n - 1), F(2 * (n - 1), 2 * (n - 1) + 3 * n), F(3 * (2 * n - 1), 2 * (n - 1) + 3 * n)),
        "1f1b-1": (F(n - 1, 2 * n - 1), F(n - 1, n - 1 + 3 * n), F(3 * (2 * n - 1), n - 1 + 3 * n)),
        "1f1b-2": (F(n - 1, 3 * n - 1), F(n - 1, n - 1 + 6 * n), F(3 * (3 * n - 1), n - 1 + 6 * n)),
    }
