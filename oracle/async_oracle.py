"""CPU oracle of eager-SGD with a clock, a step counter and a weight view per process
(the severe-imbalance case, last paragraph of Section 5 of the paper).

TEST INFRASTRUCTURE ONLY, like the rest of this package; shares no code with the GPU side.

The model, in the paper's terms.  Process p computes gradients one after the other; when its
k-th gradient is done it makes its k-th call of the partial allreduce, which belongs to the
k-th execution of the (persistent, Section 4.1.1) collective.  Let r be the number of
executions so far.
  * k == r: p waits at the open collective.  It executes when it is triggered (solo: by the
    first process to get there; majority: by the designated initiator drawn from the shared
    seed, Section 4.2; quorum q: by the q-th arrival).  The processes waiting at that moment
    are the active ones (initiator and everybody who arrived before it, Section 7.1): they
    contribute send buffer + fresh gradient.  All others contribute their send buffer
    passively.  Send buffers become G_null.  The result (sum / P, Algorithm 2 line 6) is put
    into the receive buffer; every active process applies the update rule to ITS weights
    (lines 7-8) and starts the next gradient.
  * k < r: the collective ran without p's gradient (Fig. 7): the gradient is stale and is
    kept in the send buffer - added to a stale gradient that is still there.  p finds only
    the latest result in the receive buffer (earlier ones were overwritten), applies it if
    it has not done so yet, and goes on with call k + 1.  Results it never saw make its
    weights differ from the others'.
  * every `sync_every` executions all weight (and momentum) views are replaced by their
    average over the processes (periodic model synchronisation).
Simultaneous arrivals: late calls first (by rank), then all others join the waiting set
together.  Synchronisation takes no time.
"""
from __future__ import annotations

from typing import Callable, List, Optional

import numpy as np

from . import eager_oracle as eo


def simulate(P: int, n: int, w0: np.ndarray, lr: float, mu: float, mode: str, rounds: int,
             compute_ms: Callable[[int, int], float],
             gradient: Callable[[int, int, np.ndarray], np.ndarray],
             quorum: int = 0, seed: int = 0, sync_every: int = 0, keep_results: bool = False):
    """Run until `rounds` executions.  Returns a dict with the final weight and momentum
    views, send buffers and their validity, per-process counters (and which results each process applied),
    per round the NAP, the set of active processes and the time of execution, the gradients of processes still waiting
    at the open collective ("held") and, on request, every result that was put into the
    receive buffer."""
    w = [np.ascontiguousarray(w0, dtype=np.float32).copy() for _ in range(P)]
    v = [np.zeros(n, dtype=np.float32) for _ in range(P)]
    send = [np.zeros(n, dtype=np.float32) for _ in range(P)]
    has_stale = [False] * P
    receive = np.zeros(n, dtype=np.float32)
    calls_done = [0] * P
    last_applied = [-1] * P
    clock = [float(compute_ms(p, 0)) for p in range(P)]
    blocked: List[int] = []
    fresh = {}
    executed = 0
    log = {"nap": [], "late_calls": [0] * P, "missed": [0] * P, "time_ms": 0.0, "results": [],
           "active": [], "round_time_ms": [], "applied": [[] for _ in range(P)]}

    def read_receive_buffer(p: int) -> None:
        eo.sgd_f32(receive, w[p], v[p], lr, mu)
        log["missed"][p] += (executed - 1) - last_applied[p] - 1
        log["applied"][p].append(executed - 1)
        last_applied[p] = executed - 1

    while executed < rounds:
        t = min(clock[p] for p in range(P) if p not in blocked)
        here = [p for p in range(P) if p not in blocked and clock[p] == t]
        newcomers = []
        for p in here:
            if calls_done[p] < executed:
                # too late for its collective: the gradient goes to the send buffer
                g = gradient(p, calls_done[p], w[p])
                eo.stash_f32(g, send[p], has_stale[p])
                has_stale[p] = True
                if last_applied[p] < executed - 1:
                    read_receive_buffer(p)
                log["late_calls"][p] += 1
                calls_done[p] += 1
                clock[p] = t + float(compute_ms(p, calls_done[p]))
        for p in here:
            if calls_done[p] == executed and p not in blocked and clock[p] == t:
                fresh[p] = gradient(p, calls_done[p], w[p])
                blocked.append(p)
                newcomers.append(p)
        if not newcomers:
            continue
        if mode == "solo":
            fire = True
        elif mode == "majority":
            fire = eo.initiator_hash(seed, executed) % P in blocked
        elif mode == "quorum":
            fire = len(blocked) >= quorum
        else:
            raise ValueError(mode)
        if not fire:
            continue
        active = sum(1 << p for p in blocked)
        everyone = (1 << P) - 1
        stand_in = next(iter(fresh.values()))                 # absent processes: not read
        G = [fresh.get(p, stand_in) for p in range(P)]
        valid = sum(1 << p for p in range(P) if has_stale[p])
        left = eo.round_f32(G, send, valid, active, None, None, 0.0, 0.0, recv=receive,
                            absent=everyone & ~active)
        assert left == 0
        if keep_results:
            log["results"].append(receive.copy())
        has_stale = [False] * P
        executed += 1
        log["nap"].append(len(blocked))
        log["active"].append(active)
        log["round_time_ms"].append(t)
        for p in blocked:
            read_receive_buffer(p)
            calls_done[p] += 1
            clock[p] = t + float(compute_ms(p, calls_done[p]))
        blocked, fresh = [], {}
        if sync_every and executed % sync_every == 0:
            for views in (w, v):
                mean = np.zeros(n, dtype=np.float32)
                eo.round_f32(views, [np.zeros(n, dtype=np.float32) for _ in range(P)], 0, everyone,
                             None, None, 0.0, 0.0, recv=mean)
                for x in views:
                    x[:] = mean
        log["time_ms"] = t
    return {"w": w, "v": v, "send": send, "has_stale": has_stale, "calls": calls_done,
            "clock": clock, "held": fresh, **log}
