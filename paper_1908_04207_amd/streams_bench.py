"""Bandwidth of the library's auxiliary kernels, each on its own (the round itself is timed by
bench.py at the repository root): the send-buffer stash, the update rule on a receive buffer
(plain, with a layer-wise rate, on several weight views) and the model average.

    python -m paper_1908_04207_amd.streams_bench [--log2-elements 26] [--reps 20]

One line per kernel: milliseconds per call (HIP events on the launch stream) and the
algorithmic bytes of the call divided by that time.  Under `rocprofv3 --kernel-trace --stats`
the same run gives the per-kernel durations.
"""
from __future__ import annotations

import argparse

from . import binding as eb


def _time(fn, reps: int) -> float:
    import torch
    fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / reps


def main() -> None:
    import torch
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--log2-elements", type=int, default=26)
    ap.add_argument("--views", type=int, default=8)
    ap.add_argument("--buckets", type=int, default=64, help="equal buckets the arena is cut into")
    ap.add_argument("--reps", type=int, default=20)
    a = ap.parse_args()
    n = 1 << a.log2_elements
    per = n // a.buckets // 8 * 8
    offset = [b * per for b in range(a.buckets)]
    numel = [per] * (a.buckets - 1) + [n - per * (a.buckets - 1)]
    dev = torch.device("cuda:0")
    rows = []

    def report(name: str, nbytes: int, fn) -> None:
        ms = _time(fn, a.reps)
        rows.append((name, ms, nbytes / (ms * 1e-3) / 1e9))
        print(f"{name:44s} {ms:9.4f} ms  {rows[-1][2]:7.0f} GB/s", flush=True)

    for dt, tdt, gb in ((eb.F32, torch.float32, 4), (eb.BF16, torch.bfloat16, 2)):
        ctx = eb.Context(2, [0], [n], dt, eb.ORDER_FIXED)      # one bucket: one flag to set per call
        g = torch.zeros(n, dtype=tdt, device=dev)
        r = torch.zeros(n, device=dev)
        for accumulate in (0, 1):
            def stash():
                ctx.eager_set_valid(0, accumulate)
                ctx.eager_stash(0, g, r)
            report(f"eager_stash {'bf16' if gb == 2 else 'f32'} {'R += G' if accumulate else 'R = G'}",
                   (gb + 4 + 4 * accumulate) * n, stash)
        ctx.close()
        del g, r

    ctx = eb.Context(2, offset, numel, eb.F32, eb.ORDER_FIXED)
    u = torch.randn(n, device=dev) * 1e-3
    w = [torch.randn(n, device=dev) * 0.02 for _ in range(a.views)]
    v = [torch.zeros(n, device=dev) for _ in range(a.views)]
    report("eager_sgd_step", 20 * n, lambda: ctx.eager_sgd_step(u, (w[0], v[0], 0.1, 0.9)))
    stats = torch.zeros(a.buckets * 4, dtype=torch.float64, device=dev)
    nbytes = ctx.eager_stats_workspace_bytes()
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ctx.eager_stats_attach(stats, ws, nbytes)
    report("eager_sgd_step_lars (norms, rate, update)", 28 * n,
           lambda: ctx.eager_sgd_step_lars(u, (w[0], v[0], 0.1, 0.9), 0.02, 1e-9))
    ctx.eager_stats_attach(None, None)
    report(f"eager_sgd_step x {a.views} views, one call each", 20 * a.views * n,
           lambda: [ctx.eager_sgd_step(u, (w[i], v[i], 0.1, 0.9)) for i in range(a.views)])
    report(f"eager_sgd_step_views, {a.views} views", (4 + 16 * a.views) * n,
           lambda: ctx.eager_sgd_step_views(u, w, v, 0.1, 0.9))
    report(f"eager_average_views, {a.views} views", 8 * a.views * n,
           lambda: ctx.eager_average_views(w))
    ctx.close()


if __name__ == "__main__":
    main()
