"""Hyperplane regression trained with eager-SGD through the library (the paper's one fully
synthetic experiment: Section 7.2, the hyperplane regression under light load imbalance, Fig. 10).

    y = a_0 x_0 + ... + a_{d-1} x_{d-1} + noise,   d = 8192,
    model = one linear layer (d weights + bias = 8,193 parameters, Table 1),
    P = 8 processes, total batch 2,048, one random process per step delayed by 200/300/400 ms.

What runs where: the MODEL (forward and gradient of the mean squared error, two matrix-vector
products per process) is application code and uses torch on the GPU, as the paper's model
runs in TensorFlow.  Everything eager-SGD does with the P gradients - participation plan,
partial allreduce with stale-gradient carry, 1/P average, momentum-SGD update (Algorithm 2,
lines 6-8) - runs in the library's kernels through the C ABI.

Time is simulated (there is one GPU and no network): every process needs `base_ms` per step,
with a small seeded jitter, and one seeded random rank per step gets `delay_ms` on top.  A round
lasts until its initiator arrives (solo: the first arrival; majority: the designated rank;
quorum k: the k-th arrival; synchronous SGD = quorum P: the last arrival), each round measured
from a common origin (the reading of the arrival clock this repository takes).  The paper's three
speedups over synchronous SGD (1.50x, 1.75x, 2.01x for 200, 300, 400 ms) fix base_ms at about
400 ms, which is the default here; they are a property of that time model, reproduced for
context, not a measurement of this machine.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional

from . import binding as eb

_M64 = (1 << 64) - 1


def _hash(seed: int, step: int, tag: int) -> int:
    """Counter-based 64-bit hash (SplitMix64 output function) for the delayed rank and jitter."""
    z = (seed + (step + 1) * 0x9E3779B97F4A7C15 + tag * 0xD1B54A32D192ED03) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def arrival_times(P: int, seed: int, step: int, base_ms: float, delay_ms: float,
                  jitter: float = 0.01, delayed_ranks: int = 1) -> List[float]:
    """Arrival of each process at the collective of `step`, ms from the round's origin.
    `delayed_ranks` seeded random ranks (the paper delays 1 of 8, or 4 of 64) get delay_ms on
    top; draws may coincide, then fewer ranks are delayed."""
    t = [base_ms * (1.0 + jitter * ((_hash(seed, step, 1 + p) >> 11) / 2.0 ** 53 - 0.5))
         for p in range(P)]
    # tag 0 would reproduce the library's draw of the majority initiator for the same seed
    for d in {_hash(seed, step, 1000 + i) % P for i in range(delayed_ranks)}:
        t[d] += delay_ms
    return t


@dataclass
class Result:
    mode: str
    steps: int
    sim_ms: float = 0.0                     # simulated training time
    nap_mean: float = 0.0                   # mean number of active processes
    val_loss: List[float] = field(default_factory=list)   # validation MSE, every `eval_every`
    final_w: Optional[object] = None        # device tensor, d + 1 parameters (padded arena)


def train(mode: str = "solo", steps: int = 200, P: int = 8, dim: int = 8192,
          total_batch: int = 2048, delay_ms: float = 300.0, base_ms: float = 400.0,
          lr: float = 0.01, mu: float = 0.9, noise: float = 2.0, seed: int = 20190804,
          quorum: int = 0, eval_every: int = 10, order: int = eb.ORDER_FIXED,
          on_round: Optional[Callable] = None, delayed_ranks: int = 1) -> Result:
    """Train the hyperplane model for `steps` rounds.  mode: "solo", "majority", "quorum"
    (with `quorum` = k) or "sync" (= quorum P, ordinary synchronous SGD).

    on_round(step, plan, grads, w, v), if given, is called after every round with the device
    tensors (tests use it to run the CPU oracle in lock-step)."""
    import torch
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n = dim + 1                                   # weights and bias
    arena = (n + 3) // 4 * 4
    a_true = torch.randn(dim, device=dev, generator=gen)
    Xv = torch.randn(4096, dim, device=dev, generator=gen)
    yv = Xv @ a_true + noise * torch.randn(4096, device=dev, generator=gen)
    bs = total_batch // P

    ctx = eb.Context(P, [0], [n], eb.F32, order)
    w = torch.zeros(arena, device=dev)
    v = torch.zeros(arena, device=dev)
    G = [torch.zeros(arena, device=dev) for _ in range(P)]
    R = [torch.zeros(arena, device=dev) for _ in range(P)]
    res = Result(mode, steps)
    nap_sum = 0
    for t in range(steps):
        # the model: each process draws its share of the batch and computes its gradient
        for p in range(P):
            X = torch.randn(bs, dim, device=dev, generator=gen)
            y = X @ a_true + noise * torch.randn(bs, device=dev, generator=gen)
            err = X @ w[:dim] + w[dim] - y
            G[p][:dim] = (2.0 / bs) * (X.t() @ err)
            G[p][dim] = 2.0 * err.mean()
        # eager-SGD: who is on time, then one fused round in the library
        arr = arrival_times(P, seed, t, base_ms, delay_ms, delayed_ranks=delayed_ranks)
        if mode == "solo":
            plan = eb.eager_plan_participation(eb.SOLO, arr, seed, t)
        elif mode == "majority":
            plan = eb.eager_plan_participation(eb.MAJORITY, arr, seed, t)
        elif mode in ("quorum", "sync"):
            plan = eb.eager_plan_quorum(arr, P if mode == "sync" else quorum, t)
        else:
            raise ValueError(f"unknown mode {mode!r}")
        ctx.eager_partial_allreduce(plan, G, R, opt=(w, v, lr, mu))
        res.sim_ms += arr[plan.initiator]
        nap_sum += plan.nap
        if on_round is not None:
            on_round(t, plan, G, w, v)
        if (t + 1) % eval_every == 0 or t + 1 == steps:
            res.val_loss.append(float(((Xv @ w[:dim] + w[dim] - yv) ** 2).mean()))
    torch.cuda.synchronize()
    res.nap_mean = nap_sum / steps
    res.final_w = w
    ctx.close()
    return res


def train_async(mode: str = "solo", rounds: int = 1200, sync_every: int = 0, P: int = 8,
                dim: int = 8192, total_batch: int = 2048, lr: float = 0.001, mu: float = 0.9,
                noise: float = 2.0, seed: int = 20190804, quorum: int = 0,
                recipe: str = "lognormal_0.3_straggler2x"):
    """The same problem with a clock and a weight view per process (async_sgd.AsyncEagerSGD):
    compute times from a heavy-tailed recipe carry over from call to call, so processes lag
    by several rounds, miss results and drift apart; every `sync_every` rounds the models
    are averaged (Section 5, last paragraph).  Each process computes its gradients from ITS
    weights.  Returns (AsyncResult, validation MSE of the averaged model, largest distance of
    a weight view from the average).  The learning rate is smaller than in `train`: gradients
    that arrive several rounds late and weight views that drift apart make the larger one
    unstable without synchronisation (with it, 0.01 works as well)."""
    import torch
    from workloads import times as wt
    from .async_sgd import AsyncEagerSGD
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n = dim + 1
    arena = (n + 3) // 4 * 4
    a_true = torch.randn(dim, device=dev, generator=gen)
    Xv = torch.randn(4096, dim, device=dev, generator=gen)
    yv = Xv @ a_true + noise * torch.randn(4096, device=dev, generator=gen)
    bs = total_batch // P

    def gradient(p, k, w):
        X = torch.randn(bs, dim, device=dev, generator=gen)
        y = X @ a_true + noise * torch.randn(bs, device=dev, generator=gen)
        err = X @ w[:dim] + w[dim] - y
        g = torch.zeros(arena, device=dev)
        g[:dim] = (2.0 / bs) * (X.t() @ err)
        g[dim] = 2.0 * err.mean()
        return g

    sim = AsyncEagerSGD(P, [0], [n], arena, torch.zeros(arena), lr, mu, mode, quorum, seed,
                        sync_every)
    res = sim.run(rounds, lambda p, k: 400.0 * wt.compute_times(recipe, P, seed, k)[p], gradient)
    stack = torch.stack(sim.w)
    mean = stack.mean(0)
    loss = float(((Xv @ mean[:dim] + mean[dim] - yv) ** 2).mean())
    spread = float((stack - mean).abs().max())
    sim.close()
    return res, loss, spread


def main() -> None:
    import argparse
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--delay-ms", type=float, nargs="*", default=[200.0, 300.0, 400.0])
    ap.add_argument("--quorum-sweep", action="store_true",
                    help="the spectrum between solo (k = 1) and synchronous SGD (k = P) that the "
                         "paper's conclusions propose: k-of-P rounds for every k, 300 ms delay on "
                         "two random ranks per step")
    ap.add_argument("--lagging", action="store_true",
                    help="a clock and a weight view per process, heavy-tailed compute times: "
                         "lag of several rounds, with and without periodic model synchronisation")
    a = ap.parse_args()
    if a.lagging:
        for mode, kw in (("solo", {}), ("majority", {}), ("quorum", {"quorum": 4})):
            for sync in (0, 10):
                r, loss, spread = train_async(mode, max(a.steps, 1200), sync, **kw)
                print(f"{mode:9s} sync every {sync:2d}: {r.rounds} rounds in {r.time_ms / 1e3:6.1f} s, "
                      f"NAP {sum(r.nap) / len(r.nap):4.2f}, late calls {sum(r.late_calls)}, results "
                      f"missed {sum(r.missed)}, views differ by {spread:.2e}, validation MSE of the "
                      f"mean model {loss:.3f}")
        return
    if a.quorum_sweep:
        P = 8
        runs = [train("quorum", a.steps, P=P, quorum=k, delay_ms=300.0, delayed_ranks=2)
                for k in range(1, P + 1)]
        for k, r in enumerate(runs, 1):
            print(f"quorum {k} of {P}  NAP {r.nap_mean:4.2f}  simulated {r.sim_ms / 1e3:7.1f} s "
                  f"({runs[-1].sim_ms / r.sim_ms:.2f}x synchronous)  validation MSE {r.val_loss[-1]:.3f}")
        return
    for d in a.delay_ms:
        runs = {m: train(m, a.steps, delay_ms=d) for m in ("sync", "majority", "solo")}
        for m, r in runs.items():
            print(f"delay {d:.0f} ms  {m:9s} NAP {r.nap_mean:4.2f}  simulated {r.sim_ms / 1e3:7.1f} s "
                  f"({r.steps / (r.sim_ms / 1e3):.2f} steps/s, {runs['sync'].sim_ms / r.sim_ms:.2f}x "
                  f"synchronous)  validation MSE {r.val_loss[0]:.2f} -> {r.val_loss[-1]:.3f}")


if __name__ == "__main__":
    main()
