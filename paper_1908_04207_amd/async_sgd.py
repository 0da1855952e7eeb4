"""Eager-SGD with its own clock per process: the severe-imbalance behaviour the paper describes
at the end of Section 5.

The rounds of `eager_partial_allreduce_solo/majority/quorum` start every process from a common
origin, so nobody is ever more than one round behind.  Here every process p keeps its own time,
its own weights w_p and momentum v_p, and makes its k-th call of the partial allreduce when its
k-th gradient is done; the k-th call of a process belongs to the k-th execution ("round") of the
collective (persistent schedules, Section 4.1.1).  What happens at a call (process p, call k,
rounds executed so far r):

  k == r   p has reached the round that is open.  It joins the processes waiting at it; the
           round executes when its trigger condition holds - solo: at once (p is the
           initiator); majority: when the designated initiator of round r (shared seed,
           Section 4.2) is among the waiting; quorum q: when q processes wait.  The waiting
           processes are the active ones (they arrived no later than the initiator) and
           contribute send buffer + fresh gradient; everybody else contributes what its send
           buffer holds, passively.  Every active process applies the result U_r to its own
           weights and starts its next gradient.
  k <  r   round k was executed without p's gradient.  The gradient becomes stale and goes
           into the send buffer (added to what is there, if the buffer was not emptied by a
           round in between).  p looks into the receive buffer, which holds only the LATEST
           result U_{r-1}: it applies that one (once) and has missed the results in between,
           so its weights drift away from the others'.  Its next call is k + 1.

Every `sync_every` rounds the models are synchronised: every w_p and v_p is replaced by the
average over the processes (the periodic model synchronisation that Section 5 prescribes).

Whether the open round executes, and its plan, is decided by the library
(`eager_plan_open_round`), and all arithmetic runs there: the round
(`eager_partial_allreduce_lagging`, receive buffer only), the update rule on the weight views of the processes that see a result
(`eager_sgd_step_views`, one kernel), the stash (`eager_stash`) and the model average
(`eager_average_views`).  This module is the event loop and the bookkeeping.

Readings taken here (the paper gives no detail): simultaneous arrivals are handled together
(late calls first, by rank; the others all count as arrived); a model synchronisation takes
no time and does not wait for anybody; the momentum is averaged along with the weights.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

from . import binding as eb


@dataclass
class AsyncResult:
    rounds: int = 0
    time_ms: float = 0.0                      # time of the last round
    calls: List[int] = field(default_factory=list)        # calls made per process
    late_calls: List[int] = field(default_factory=list)   # of which: gradient went to the send buffer
    missed: List[int] = field(default_factory=list)       # results a process never applied
    nap: List[int] = field(default_factory=list)          # active processes per round
    divergence: List[float] = field(default_factory=list)  # max_p |w_p - mean w|_inf after each round


class AsyncEagerSGD:
    """State of P processes with separate clocks and weight views over one bucketed arena."""

    def __init__(self, P: int, bucket_offset: Sequence[int], bucket_numel: Sequence[int],
                 arena_numel: int, w0, lr: float, mu: float, mode: str = "solo",
                 quorum: int = 0, seed: int = 0, sync_every: int = 0,
                 grad_dtype: int = eb.F32, track_divergence: bool = True):
        import torch
        self.torch = torch
        self.P, self.n, self.lr, self.mu = P, arena_numel, lr, mu
        self.mode, self.quorum, self.seed, self.sync_every = mode, quorum, seed, sync_every
        dev = torch.device("cuda:0")
        self.ctx = eb.Context(P, bucket_offset, bucket_numel, grad_dtype, eb.ORDER_FIXED)
        self.w = [w0.to(dev).clone() for _ in range(P)]
        self.v = [torch.zeros(arena_numel, device=dev) for _ in range(P)]
        self.R = [torch.zeros(arena_numel, device=dev) for _ in range(P)]
        self.recv = torch.zeros(arena_numel, device=dev)
        self.r = 0                              # rounds executed
        self.k = [0] * P                        # calls made
        self.T = [0.0] * P                      # time of the next call
        self.seen = [-1] * P                    # last result applied
        self.waiting: List[int] = []
        self.held = {}                          # gradients of the waiting processes
        self.track_divergence = track_divergence
        self.res = AsyncResult(calls=[0] * P, late_calls=[0] * P, missed=[0] * P)

    def _apply(self, procs: Sequence[int]) -> None:
        """The listed processes apply the result in the receive buffer (the latest round's)
        to their own weights: one kernel, one read of the result."""
        self.ctx.eager_sgd_step_views(self.recv, [self.w[p] for p in procs],
                                      [self.v[p] for p in procs], self.lr, self.mu)
        for p in procs:
            self.res.missed[p] += self.r - 1 - self.seen[p] - 1
            self.seen[p] = self.r - 1

    def _synchronise(self) -> None:
        self.ctx.eager_average_views(self.w)
        self.ctx.eager_average_views(self.v)

    def run(self, rounds: int, compute_ms: Callable[[int, int], float],
            gradient: Callable[[int, int, object], object]) -> AsyncResult:
        """Advance until `rounds` more rounds have executed.  compute_ms(p, k): duration of
        process p's k-th gradient; gradient(p, k, w_p): that gradient as a device tensor
        (arena layout, the context's gradient type)."""
        torch, P = self.torch, self.P
        if not any(self.k) and not any(self.T):
            self.T = [compute_ms(p, 0) for p in range(P)]
        target = self.r + rounds
        while self.r < target:
            free = [p for p in range(P) if p not in self.waiting]
            now = min(self.T[p] for p in free)
            arrived = [p for p in free if self.T[p] == now]
            for p in [q for q in arrived if self.k[q] < self.r]:           # late calls
                self.ctx.eager_stash(p, gradient(p, self.k[p], self.w[p]), self.R[p])
                if self.seen[p] < self.r - 1:
                    self._apply([p])
                self.res.calls[p] += 1
                self.res.late_calls[p] += 1
                self.k[p] += 1
                self.T[p] = now + compute_ms(p, self.k[p])
            # (a process that has just made a late call is computing again: its time moved on)
            for p in [q for q in arrived if self.k[q] == self.r and self.T[q] == now]:
                self.held[p] = gradient(p, self.k[p], self.w[p])
                self.waiting.append(p)
                self.res.calls[p] += 1
            if not any(p in self.waiting for p in arrived):
                continue
            # whether the open execution is triggered, and its plan, is the library's decision
            mask = sum(1 << p for p in self.waiting)
            mode = {"solo": eb.SOLO, "majority": eb.MAJORITY, "quorum": eb.QUORUM}[self.mode]
            plan = eb.eager_plan_open_round(mode, P, mask, self.waiting[-1], self.r, self.quorum,
                                            self.seed)
            if plan is None:
                continue
            absent = ((1 << P) - 1) & ~mask
            grads = [self.held.get(p) for p in range(P)]
            self.ctx.eager_partial_allreduce_lagging(plan, absent, grads, self.R, recv=self.recv)
            self.r += 1
            self.res.nap.append(len(self.waiting))
            self._apply(self.waiting)
            for p in self.waiting:
                self.k[p] += 1
                self.T[p] = now + compute_ms(p, self.k[p])
            self.waiting, self.held = [], {}
            if self.sync_every and self.r % self.sync_every == 0:
                self._synchronise()
            if self.track_divergence:
                stack = torch.stack(self.w)
                self.res.divergence.append(float((stack - stack.mean(0)).abs().max()))
            self.res.rounds, self.res.time_ms = self.r, now
        return self.res

    def close(self) -> None:
        self.ctx.close()
