"""CPU oracle of eager-SGD with a clock, a step counter and a weight view per process
(the severe-imbalance case, last paragraph of Section 5 of the paper).

TEST INFRASTRUCTURE ONLY, like the rest of this package; shares no code with the GPU side.

The model, in the paper's terms.  Process p computes gradients one after the other; when its
k-th gradient is done it makes its k-th call of the partial allreduce, which belongs to the
k-th execution of the (persistent, Section 4.1.1) collective.
  * A call that reaches its execution before or when it is triggered is ACTIVE in it (the
    initiator and everybody who arrived no later, Section 7.1): the process contributes send
    buffer + fresh gradient, applies the result to ITS weights (Algorithm 2, lines 7-8) and
    starts its next gradient when the execution is over.
  * A call that comes after its execution was triggered is LATE (Fig. 7): the gradient is
    kept in the send buffer - added to a stale gradient that is still there - and the process
    goes on at once.  It finds only the latest result in the receive buffer (earlier ones were
    overwritten) and applies it if it has not done so yet; results it never saw make its
    weights differ from the others'.  Whatever a send buffer holds is contributed passively
    to the next execution, which empties it.
  * Execution k is triggered (solo) by the first call k to arrive, (majority) by call k of
    the designated initiator drawn from the shared seed (Section 4.2), (quorum q) by the q-th
    call k to arrive.  Every result is sum / P (Algorithm 2, line 6).
  * Every `sync_every` executions all weight (and momentum) views are replaced by their
    average over the processes (periodic model synchronisation).
Calls at the same instant: late ones first (by rank), then the others reach the open
execution together.  Synchronisation takes no time.

Shape of this oracle.  Since call k of a process can only arrive after execution k - 1, the
whole timetable follows from the compute times alone, execution by execution, in closed form
(`timetable`): arrival of every call, trigger time of every execution, who is active.  From
it `ledger` states for every gradient (process, call) in which execution it is delivered.
`simulate` then does the arithmetic by walking the timetable's events in order of time; it
never decides anything about participation itself, and it checks the send buffers against
the ledger as it goes.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Tuple

import numpy as np

from . import eager_oracle as eo


def timetable(P: int, mode: str, rounds: int, compute_ms: Callable[[int, int], float],
              quorum: int = 0, seed: int = 0):
    """arrive[p][k]: when process p makes call k (k = 0..rounds); trigger[k]: when execution k
    is triggered; active[p][k]: whether call k of p is active in execution k."""
    arrive = [[float(compute_ms(p, 0))] for p in range(P)]
    active: List[List[bool]] = [[] for _ in range(P)]
    trigger: List[float] = []
    for k in range(rounds):
        at = [arrive[p][k] for p in range(P)]
        if mode == "solo":
            fired = min(at)
        elif mode == "majority":
            fired = at[eo.initiator_hash(seed, k) % P]
        elif mode == "quorum":
            if not 1 <= quorum <= P:
                raise ValueError(quorum)
            fired = sorted(at)[quorum - 1]
        else:
            raise ValueError(mode)
        trigger.append(fired)
        for p in range(P):
            on_time = at[p] <= fired
            active[p].append(on_time)
            # an active process goes on when the execution is over, a late one at once
            arrive[p].append((fired if on_time else at[p]) + float(compute_ms(p, k + 1)))
    return arrive, trigger, active


def ledger(P: int, rounds: int, arrive, trigger, active) -> Dict[Tuple[int, int], Optional[int]]:
    """For every call (p, k) made before the last execution is over: the execution that
    delivers its gradient - k itself for an active call, else the first one triggered at or
    after the call (late calls go first at equal times), None if there is none yet."""
    end = trigger[-1]
    out: Dict[Tuple[int, int], Optional[int]] = {}
    for p in range(P):
        for k in range(rounds):
            if active[p][k]:
                out[(p, k)] = k
            elif arrive[p][k] <= end:
                later = [j for j in range(rounds) if trigger[j] >= arrive[p][k]]
                out[(p, k)] = later[0] if later else None
    return out


def simulate(P: int, n: int, w0: np.ndarray, lr: float, mu: float, mode: str, rounds: int,
             compute_ms: Callable[[int, int], float],
             gradient: Callable[[int, int, np.ndarray], np.ndarray],
             quorum: int = 0, seed: int = 0, sync_every: int = 0, keep_results: bool = False):
    """Run until `rounds` executions.  Returns a dict with the final weight and momentum
    views, send buffers and their validity, per-process counters (and which results each
    process applied), per round the NAP, the set of active processes and the time of
    execution, the ledger (process, call) -> delivering execution and, on request, every
    result that was put into the receive buffer."""
    arrive, trigger, active = timetable(P, mode, rounds, compute_ms, quorum, seed)
    delivery = ledger(P, rounds, arrive, trigger, active)
    # events in order of time; at equal times late calls (by rank), then arrivals at the open
    # execution (by rank), then the execution itself
    LATE, ARRIVAL, EXECUTION = 0, 1, 2
    events = [(trigger[k], EXECUTION, k, k) for k in range(rounds)]
    for (p, k) in delivery:
        events.append((arrive[p][k], ARRIVAL if active[p][k] else LATE, p, k))
    events.sort()

    w = [np.ascontiguousarray(w0, dtype=np.float32).copy() for _ in range(P)]
    v = [np.zeros(n, dtype=np.float32) for _ in range(P)]
    send = [np.zeros(n, dtype=np.float32) for _ in range(P)]
    in_send: List[List[Tuple[int, int]]] = [[] for _ in range(P)]    # calls whose gradient is there
    receive = np.zeros(n, dtype=np.float32)
    last_applied = [-1] * P
    fresh: Dict[int, np.ndarray] = {}
    log = {"nap": [], "late_calls": [0] * P, "missed": [0] * P, "results": [], "active": [],
           "round_time_ms": list(trigger), "applied": [[] for _ in range(P)]}

    def read_receive_buffer(p: int, latest: int) -> None:
        eo.sgd_f32(receive, w[p], v[p], lr, mu)
        log["missed"][p] += latest - last_applied[p] - 1
        log["applied"][p].append(latest)
        last_applied[p] = latest

    executed = 0
    for when, kind, p, k in events:
        if kind == LATE:
            eo.stash_f32(gradient(p, k, w[p]), send[p], bool(in_send[p]))
            in_send[p].append((p, k))
            log["late_calls"][p] += 1
            assert executed > k and delivery[(p, k)] in (executed, None)
            if last_applied[p] < executed - 1:
                read_receive_buffer(p, executed - 1)
        elif kind == ARRIVAL:
            assert executed == k
            fresh[p] = gradient(p, k, w[p])
        else:
            assert executed == k and sorted(fresh) == [q for q in range(P) if active[q][k]]
            for q in range(P):
                assert all(delivery[c] == k for c in in_send[q])
            mask = sum(1 << q for q in fresh)
            everyone = (1 << P) - 1
            stand_in = next(iter(fresh.values()))                 # absent processes: not read
            left = eo.round_f32([fresh.get(q, stand_in) for q in range(P)], send,
                                sum(1 << q for q in range(P) if in_send[q]), mask, None, None,
                                0.0, 0.0, recv=receive, absent=everyone & ~mask)
            assert left == 0
            in_send = [[] for _ in range(P)]
            if keep_results:
                log["results"].append(receive.copy())
            executed += 1
            log["nap"].append(len(fresh))
            log["active"].append(mask)
            for q in sorted(fresh):
                read_receive_buffer(q, k)
            fresh = {}
            if sync_every and executed % sync_every == 0:
                for views in (w, v):
                    mean = np.zeros(n, dtype=np.float32)
                    eo.round_f32(views, [np.zeros(n, dtype=np.float32) for _ in range(P)], 0,
                                 everyone, None, None, 0.0, 0.0, recv=mean)
                    for x in views:
                        x[:] = mean
    calls = [sum(1 for (q, _) in delivery if q == p) for p in range(P)]
    clock = [arrive[p][calls[p]] for p in range(P)]
    return {"w": w, "v": v, "send": send, "has_stale": [bool(x) for x in in_send], "calls": calls,
            "clock": clock, "held": {}, "time_ms": trigger[-1], "ledger": delivery,
            "pending": [list(x) for x in in_send], **log}
