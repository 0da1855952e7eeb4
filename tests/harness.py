"""Side-by-side driver for parity tests: the same seeded rounds go through the GPU library
(via the ctypes binding, i.e. through the C ABI) and through the CPU oracle.

The two sides share only the inputs produced by `workloads`; expected values always come
from the oracle.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from oracle import eager_oracle as eo
from workloads import grads as wg
from workloads import times as wt

NT_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def paper_values() -> dict:
    """tests/golden/paper_reported_values.txt as {key: float}."""
    import os
    out = {}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden",
                        "paper_reported_values.txt")
    for line in open(path):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def as_oracle_grad(t: torch.Tensor) -> np.ndarray:
    """CPU tensor -> what the oracle takes (float32, or uint16 bit patterns for bf16)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def normwise(a: np.ndarray, b: np.ndarray) -> float:
    """max |a - b| / max |b|  (per array; the tolerance metric of the fast mode)."""
    if a.size == 0:
        return 0.0
    return float(np.max(np.abs(a.astype(np.float64) - b.astype(np.float64)))
                 / max(float(np.max(np.abs(b))), 1e-30))


class Pair:
    """GPU state + oracle state over one bucketed arena, stepped in lock-step."""

    def __init__(self, eb, P: int, offset: Sequence[int], numel: Sequence[int],
                 arena_numel: int, grad_dtype: str = "f32", order: int = 0,
                 lr: float = 0.1, mu: float = 0.9, seed: int = 1,
                 grad_sigma: float = 1e-3, param_sigma: float = 0.02, poison: bool = True,
                 wd: float = 0.0, nesterov: bool = False):
        self.eb, self.P, self.seed = eb, P, seed
        self.offset, self.numel, self.arena = list(offset), list(numel), arena_numel
        self.dtype = NT_DTYPE[grad_dtype]
        self.lr, self.mu, self.gs = lr, mu, grad_sigma
        dev = torch.device("cuda:0")
        self.ctx = eb.Context(P, self.offset, self.numel,
                              eb.BF16 if grad_dtype == "bf16" else eb.F32, order)
        w0 = wg.fill(torch.empty(arena_numel), seed, 0, wg.PARAM_RANK, param_sigma)
        self.w = w0.to(dev)
        self.v = torch.zeros(arena_numel, device=dev)
        # empty send buffers are poisoned: reading one shows up as NaN in w
        self.R = [torch.full((arena_numel,), float("nan") if poison else 0.0, device=dev)
                  for _ in range(P)]
        self.G = [torch.empty(arena_numel, dtype=self.dtype, device=dev) for _ in range(P)]
        self.recv = torch.empty(arena_numel, device=dev)
        if wd or nesterov:
            self.ctx.eager_set_update_rule(wd, nesterov)
        self.oracle = eo.OracleState(P, self.offset, self.numel, arena_numel, w0.numpy(), lr, mu,
                                     wd, nesterov)
        self.oracle_recv = np.zeros(arena_numel, dtype=np.float32)
        self.step_no = 0

    # -- inputs --------------------------------------------------------------------------
    def fresh_grads(self, step: int) -> List[np.ndarray]:
        out = []
        for p in range(self.P):
            g = wg.fill(torch.empty(self.arena, dtype=self.dtype), self.seed, step, p, self.gs)
            self.G[p].copy_(g)
            out.append(as_oracle_grad(g))
        return out

    def set_grads(self, arrays: Sequence[torch.Tensor]) -> List[np.ndarray]:
        out = []
        for p, g in enumerate(arrays):
            self.G[p].copy_(g)
            out.append(as_oracle_grad(g))
        return out

    # -- one round on both sides ---------------------------------------------------------
    def round(self, plan, G_host: List[np.ndarray], b0: int = 0, b1: Optional[int] = None,
              fused: bool = True, want_recv: bool = False, absent: Optional[int] = None) -> None:
        opt = (self.w, self.v, self.lr, self.mu) if fused else None
        recv = self.recv if (want_recv or not fused) else None
        if absent is None:
            self.ctx.eager_partial_allreduce(plan, self.G, self.R, recv=recv, opt=opt, b0=b0, b1=b1)
        else:       # processes that lag by more than a round: no gradient handed over for them
            G = [None if (absent >> p) & 1 else g for p, g in enumerate(self.G)]
            self.ctx.eager_partial_allreduce_lagging(plan, absent, G, self.R, recv=recv, opt=opt,
                                                     b0=b0, b1=b1)
        self.oracle.round(plan.mask, G_host, b0, b1,
                          recv=self.oracle_recv if recv is not None else None, fused=fused,
                          absent=absent or 0)

    def round_exchange(self, plan, G_host: List[np.ndarray], fused: bool = True,
                       want_recv: bool = False) -> None:
        """The same round, but the library makes the gradient buffer of every late process its
        send buffer by exchanging the two pointers (self.G and self.R are permuted to match);
        the oracle runs its ordinary round."""
        opt = (self.w, self.v, self.lr, self.mu) if fused else None
        recv = self.recv if (want_recv or not fused) else None
        self.ctx.eager_partial_allreduce_exchange(plan, self.G, self.R, recv=recv, opt=opt)
        self.oracle.round(plan.mask, G_host, recv=self.oracle_recv if recv is not None else None,
                          fused=fused)

    def flush(self, b0: int = 0, b1: Optional[int] = None, fused: bool = True) -> None:
        """The round in which nobody hands over a gradient: pending send buffers delivered."""
        opt = (self.w, self.v, self.lr, self.mu) if fused else None
        self.ctx.eager_flush(self.R, recv=self.recv, opt=opt, b0=b0, b1=b1)
        everyone = (1 << self.P) - 1
        none = [np.zeros(self.arena, dtype=np.uint16 if self.dtype == torch.bfloat16 else np.float32)
                for _ in range(self.P)]
        self.oracle.round(0, none, b0, b1, recv=self.oracle_recv, fused=fused, absent=everyone)

    def stash(self, p: int, g: torch.Tensor, b0: int = 0, b1: Optional[int] = None) -> None:
        """A gradient of process p finished between two rounds (tensor on the host)."""
        dev = g.to(self.G[p].device)
        self.ctx.eager_stash(p, dev, self.R[p], b0, b1)
        self.oracle.stash(p, as_oracle_grad(g), b0, b1)

    def sgd(self, b0: int = 0, b1: Optional[int] = None) -> None:
        self.ctx.eager_sgd_step(self.recv, (self.w, self.v, self.lr, self.mu), b0, b1)
        self.oracle.sgd(self.oracle_recv, b0, b1)

    # -- comparison ----------------------------------------------------------------------
    def _bucket_slices(self, b0=0, b1=None):
        b1 = len(self.numel) if b1 is None else b1
        return [(b, slice(self.offset[b], self.offset[b] + self.numel[b])) for b in range(b0, b1)]

    def compare(self, exact: bool, tol: float = 1e-6, check_recv: bool = False,
                b0: int = 0, b1: Optional[int] = None, what: str = "") -> None:
        torch.cuda.synchronize()
        w, v = self.w.cpu().numpy(), self.v.cpu().numpy()
        recv = self.recv.cpu().numpy() if check_recv else None
        R = None
        for b, sl in self._bucket_slices(b0, b1):
            valid = self.ctx.eager_get_valid(b)
            assert valid == self.oracle.valid[b], (what, b, hex(valid), hex(self.oracle.valid[b]))
            pairs = [("w", w[sl], self.oracle.w[sl]), ("v", v[sl], self.oracle.v[sl])]
            if check_recv:
                pairs.append(("recv", recv[sl], self.oracle_recv[sl]))
            if valid:
                if R is None:
                    R = [r.cpu().numpy() for r in self.R]
                for p in range(self.P):
                    if (valid >> p) & 1:
                        pairs.append((f"R{p}", R[p][sl], self.oracle.R[p][sl]))
            for name, got, want in pairs:
                if exact:
                    # equal bits wherever the oracle's value is a number (so +0.0 and -0.0 are
                    # told apart); where it is NaN the payload may differ, NaN-ness may not
                    nan = np.isnan(want)
                    same = np.array_equal(bits(got)[~nan], bits(want)[~nan]) and \
                        bool(np.all(np.isnan(got[nan])))
                    assert same, f"{what}: bucket {b} {name} differs bitwise " \
                                 f"({int(np.sum(bits(got) != bits(want)))} of {got.size})"
                else:
                    err = normwise(got, want)
                    assert err <= tol, f"{what}: bucket {b} {name} normwise error {err:.3g} > {tol}"


def plan_for(eb, cfg, step: int, library: bool = True):
    """Participation plan of a configuration's step, from its seeded compute times; the
    library's and the oracle's planners must agree, which is asserted here."""
    t = wt.compute_times(cfg.times, cfg.P, cfg.seed, step)
    mode = eb.SOLO if cfg.mode == "solo" else eb.MAJORITY
    lp = eb.eager_plan_participation(mode, t, cfg.seed, step)
    op = eo.plan_participation(eo.SOLO if cfg.mode == "solo" else eo.MAJORITY, cfg.P, t,
                               cfg.seed, step)
    assert (lp.mask, lp.initiator, lp.nap) == (op.mask, op.initiator, op.nap)
    return lp
