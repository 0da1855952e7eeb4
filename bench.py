#!/usr/bin/env python3
"""Throughput of the fused eager-SGD round (partial allreduce + carry + momentum SGD) on
one MI355X, on synthetic gradients shaped like the paper's workloads.

A step = plan participation from that step's seeded compute times (host) + one fused
round over every bucket of the model (device).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line: throughput of the timed steps, the roofline fraction of
the round kernels, and the CPU oracle's rate on the host cores for comparison.

  python bench.py [--steps K] [--warmup W] [--config 2] [--order fixed|fast]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
PAPER_CONTEXT = ("paper (Piz Daint, Xeon E5-2690 + P100 per node, Cray Aries, fp32): eager-SGD "
                 "1.29x over Deep500 / 1.27x over Horovod (ResNet-50, 64 proc), 1.27x over "
                 "Horovod (LSTM/UCF101, majority), 2.64x over async PS; end-to-end training "
                 "throughput on a cluster, not this kernel: context only")


# HBM bytes per launch of the round kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE runs (the
# summaries and the commands are under profiles/); counters cannot be read from inside a
# timed run, so the figure of the committed profile is quoted here.
MEASURED_TRAFFIC = {
    "cfg2_resnet50_P8_majority": {
        "bytes_per_launch": 1966000000,
        "note": "rocprofv3 --pmc FETCH_SIZE (x2.0000) + WRITE_SIZE (x1.0000), scale factors from "
                "a 1 GiB copy kernel in the same process; mean of rounds 0..21, whose algorithmic "
                "mean is 1965700000 B: ratio 1.0001"},
    "cfg3_lstm_P16_solo": {
        "bytes_per_launch": 13131100000,
        "note": "same method; slot_kernel + carry_kernel of a round together, mean of rounds "
                "0..11, whose algorithmic mean is 13129800000 B: ratio 1.0001"},
    "cfg4_transformer350M_P32_majority": {
        "bytes_per_launch": 107871900000,
        "note": "same method, inputs set up with --light-setup (the profiler's counter mode does "
                "not survive the generator's tens of thousands of dispatches); slot_kernel + "
                "carry_kernel of a round together, mean of rounds 0..7, whose algorithmic mean is "
                "107866200000 B: ratio 1.0001"},
    "cfg5_gpt2xl_P16_solo_bf16": {
        "bytes_per_launch": 261679500000,
        "note": "same method, inputs set up with --light-setup; rounds 1..5 (15 processes late, 15 "
                "send buffers pending), algorithmic 261678700000 B: ratio 1.0000"},
    "cfg5_gpt2xl_P16_solo_bf16_clip262144": {
        "bytes_per_launch": 8401100000,
        "note": "same method, on the configuration clipped to 262144 elements per tensor (the "
                "profiler's counter mode fails at the full size); mean of rounds 0..9, whose "
                "algorithmic mean is 8400900000 B: ratio 1.0000"},
}


def alg_bytes_per_element(P: int, gbytes: int, q_prev: int, q_now: int) -> int:
    """Algorithmic HBM bytes per element of one round: every fresh gradient read once,
    non-empty send buffers read, send buffers of late processes written, w and v read and
    written.  Empty send buffers and the reset of on-time ones cost nothing."""
    return gbytes * P + 4 * q_prev + 4 * q_now + 16


def popcount(x: int) -> int:
    return bin(x).count("1")


class Workload:
    """Device state of one configuration, inputs generated on the GPU by the seeded
    generator (outside any timed region)."""

    def __init__(self, k: int, order: str, launch: dict | None = None, stagger: int = 0,
                 clip: int = 0, stats: bool = False, unfused: bool = False, lars: float = 0.0,
                 light_setup: bool = False, views: bool = False):
        import torch
        from paper_1908_04207_amd import binding as eb
        from workloads import grads as wg
        from workloads import shapes
        self.torch, self.eb = torch, eb
        self.cfg = cfg = shapes.scaled(shapes.config(k), clip) if clip else shapes.config(k)
        bt = cfg.buckets
        dev = torch.device("cuda:0")
        self.gdtype = torch.bfloat16 if cfg.grad_dtype == "bf16" else torch.float32
        self.gbytes = 2 if cfg.grad_dtype == "bf16" else 4
        self.ctx = eb.Context(cfg.P, bt.offset, bt.numel,
                              eb.BF16 if cfg.grad_dtype == "bf16" else eb.F32,
                              eb.ORDER_FIXED if order == "fixed" else eb.ORDER_FAST)
        for key, val in (launch or {}).items():
            self.ctx.eager_set_launch(key, val)
        n = bt.arena_numel

        def arena(dtype, i):
            # optional stagger: shifts each stream's base by i*stagger bytes so that the
            # P same-offset streams do not start on the same HBM channel
            pad = (i * stagger) // (2 if dtype == torch.bfloat16 else 4)
            return torch.empty(n + pad, dtype=dtype, device=dev)[pad:]
        self.G = [arena(self.gdtype, p) for p in range(cfg.P)]
        self.R = [arena(torch.float32, cfg.P + p) for p in range(cfg.P)]
        for p in range(cfg.P):
            if light_setup and p > 0:
                # few dispatches before the timed region (the profiler's counter mode does not
                # survive the tens of thousands of small generator kernels of the largest
                # configurations): every process gets a copy of process 0's gradient
                self.G[p].copy_(self.G[0])
            else:
                wg.fill(self.G[p], cfg.seed, 0, p, cfg.grad_sigma,
                        chunk=1 << 26 if light_setup else 1 << 24)
            self.R[p].zero_()
        self.w = wg.fill(torch.empty(n, device=dev), cfg.seed, 0, wg.PARAM_RANK, cfg.param_sigma,
                         chunk=1 << 26 if light_setup else 1 << 24)
        self.v = torch.zeros(n, device=dev)
        self.lars = lars
        if lars > 0.0:  # layer-wise rate: needs the receive buffer and the statistics workspace
            if not stats:   # ... but not the rounds' own by-products: the step forms its norms
                self.ctx.eager_set_launch("round_stats", 0)
            stats = unfused = True
        if stats:      # optional per-bucket by-products (norms), computed in the same pass
            nbytes = self.ctx.eager_stats_workspace_bytes()
            self.stats = torch.zeros(bt.n_buckets * 4, dtype=torch.float64, device=dev)
            self.stats_ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            self.ctx.eager_stats_attach(self.stats, self.stats_ws, nbytes)
        self.views = views
        if views:      # a weight view per process (Section 5, last paragraph): the round goes to
            unfused = True   # the receive buffer, every process applies it to its own w_p, v_p
            self.wp = [self.w] + [self.w.clone() for _ in range(cfg.P - 1)]
            self.vp = [self.v] + [torch.zeros(n, device=dev) for _ in range(cfg.P - 1)]
            self.wpp, self.vpp = self.ctx.pointers(self.wp), self.ctx.pointers(self.vp)
        self.unfused = unfused
        if unfused:    # A/B: receive buffer first, update rule as a second pass
            self.recv = torch.empty(n, device=dev)
        self.step_no = 0
        self.q_prev = 0
        # argument marshalling done once: pointer tables, the stream handle
        self.Gp, self.Rp = self.ctx.pointers(self.G), self.ctx.pointers(self.R)
        self.stream = torch.cuda.current_stream().cuda_stream
        self.mode = eb.SOLO if cfg.mode == "solo" else eb.MAJORITY
        self.arrivals = {}
        torch.cuda.synchronize()

    def prepare(self, first: int, count: int) -> None:
        """The seeded compute times of steps first .. first+count-1.  They are inputs of the
        workload, like the gradients, and are produced before the timed region; deciding
        who is on time from them (eager_plan_participation) is part of every step."""
        from workloads import times
        cfg = self.cfg
        for s in range(first, first + count):
            if s not in self.arrivals:
                self.arrivals[s] = times.compute_times(cfg.times, cfg.P, cfg.seed, s)

    def plan(self, step: int):
        if step not in self.arrivals:
            self.prepare(step, 1)
        return self.eb.eager_plan_participation(self.mode, self.arrivals[step], self.cfg.seed, step)

    def step(self) -> int:
        """One step; returns its algorithmic bytes."""
        cfg = self.cfg
        plan = self.last_plan = self.plan(self.step_no)
        if self.unfused:
            self.ctx.eager_partial_allreduce(plan, self.Gp, self.Rp, recv=self.recv, opt=None,
                                             stream=self.stream)
            if self.views:
                self.ctx.eager_sgd_step_views(self.recv, self.wpp, self.vpp, cfg.lr, cfg.mu,
                                              stream=self.stream)
            elif self.lars > 0.0:
                self.ctx.eager_sgd_step_lars(self.recv, (self.w, self.v, cfg.lr, cfg.mu), self.lars,
                                             1e-9, stream=self.stream)
            else:
                self.ctx.eager_sgd_step(self.recv, (self.w, self.v, cfg.lr, cfg.mu),
                                        stream=self.stream)
        else:
            self.ctx.eager_partial_allreduce(plan, self.Gp, self.Rp, recv=None,
                                             opt=(self.w, self.v, cfg.lr, cfg.mu),
                                             stream=self.stream)
        q_now = cfg.P - plan.nap
        b = alg_bytes_per_element(cfg.P, self.gbytes, self.q_prev, q_now) * cfg.numel
        self.q_prev = q_now
        self.step_no += 1
        return b


def run_gpu(k: int, steps: int, warmup: int, order: str, launch=None, stagger=0, clip=0,
            stats=False, unfused=False, lars=0.0, light_setup=False, views=False):
    """W untimed steps, then K timed steps.  Returns the workload, the wall-clock seconds
    of the K steps (synchronised on both sides), their algorithmic bytes, and the GPU time
    of the same K steps between two HIP events recorded on the launch stream (torch's
    current stream, which is the one the binding launches on)."""
    import torch
    wl = Workload(k, order, launch, stagger, clip, stats, unfused, lars, light_setup, views)
    wl.prepare(0, warmup + steps)
    for _ in range(warmup):
        wl.step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    nbytes = []
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        nbytes.append(wl.step())
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wl, wall, nbytes, e0.elapsed_time(e1) * 1e-3


def trace_steps(wl: "Workload", steps: int, path: str) -> None:
    """Per-step log (JSON lines) of a separate, untimed pass: participation of the round,
    algorithmic bytes, GPU time of the step between two HIP events, GB/s."""
    import torch
    with open(path, "w") as f:
        for _ in range(steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            b = wl.step()
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            pl = wl.last_plan
            f.write(json.dumps({"step": wl.step_no - 1, "nap": pl.nap, "initiator": pl.initiator,
                                "mask": f"{pl.mask:#x}", "alg_bytes": b,
                                "gpu_us": round(ms * 1e3, 2),
                                "GBps": round(b / (ms * 1e-3) / 1e9, 1)}) + "\n")


def copy_ceiling_gbs() -> dict:
    """Device-to-device copy and read-only stream rates of plain kernels, for context."""
    import torch
    from paper_1908_04207_amd import binding as eb
    n = 1 << 30
    # gradient-like data, not zeros: what the buffers hold changes the rate by 1-2 %
    a = (torch.randn(n // 4, device="cuda") * 1e-3).view(torch.uint8)
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, device="cuda")
    out = {}
    for name, fn, traffic in (("copy", lambda: eb.eager_calib_copy(b, a, n), 2 * n),
                              ("read", lambda: eb.eager_calib_read(a, n, sink), n)):
        for _ in range(3):
            fn()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(10):
            fn()
        e.record()
        torch.cuda.synchronize()
        out[name] = traffic * 10 / (s.elapsed_time(e) * 1e-3) / 1e9
    return out


def cpu_baseline(wl: Workload, budget_s: float = 20.0) -> dict:
    """The CPU oracle, as it stands, on this host's cores, on a bounded sample of the
    same workload: the first rounds of the configuration on a leading slice of the arena
    (whole buckets), same gradients and plans as the GPU run."""
    import numpy as np
    from oracle import eager_oracle as eo
    cfg = wl.cfg
    bt = cfg.buckets
    cores = len(os.sched_getaffinity(0))
    # whole buckets from the front of the arena, at most 2^25 elements per process (the
    # whole model where it is smaller); the round loop below stops at the time budget
    cap = 1 << 25
    nb, tot = 0, 0
    while nb < bt.n_buckets and (nb == 0 or tot + bt.numel[nb] <= cap):
        tot += bt.numel[nb]
        nb += 1
    hi = bt.offset[nb - 1] + bt.numel[nb - 1]
    if bt.numel[0] > cap:                    # a single huge first bucket: take a slice of it
        hi, tot = cap, cap
        offs, nums = [0], [hi]
    else:
        offs, nums = list(bt.offset[:nb]), list(bt.numel[:nb])

    def host(t):
        t = t[:hi].cpu()
        if t.dtype == wl.torch.bfloat16:
            return t.view(wl.torch.int16).numpy().view(np.uint16)
        return t.numpy()
    import torch
    from workloads import grads as wg
    G = [host(g) for g in wl.G]
    w0 = wg.fill(torch.empty(hi), cfg.seed, 0, wg.PARAM_RANK, cfg.param_sigma).numpy()
    res = {}
    for label, nthreads in (("threaded", cores), ("scalar", 1)):   # 12 s + 8 s of oracle work
        st = eo.OracleState(cfg.P, offs, nums, hi, w0, cfg.lr, cfg.mu)
        q_prev, nbytes, secs, rounds = 0, 0, 0.0, 0
        limit = budget_s * (0.6 if nthreads > 1 else 0.4)
        step = 0
        while True:                      # rounds continue past cfg.steps until the budget
            mask = wl.plan(step).mask
            t0 = time.perf_counter()
            st.round(mask, G, nthreads=nthreads)
            secs += time.perf_counter() - t0
            q_now = cfg.P - popcount(mask)
            nbytes += alg_bytes_per_element(cfg.P, wl.gbytes, q_prev, q_now) * tot
            q_prev = q_now
            rounds += 1
            step += 1
            if secs > limit:
                break
        res[label] = (nbytes / secs / 1e9, rounds, secs)
    gbs, rounds, secs = res["threaded"]
    return {"value": round(gbs, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{rounds} rounds of {cfg.name} on its first {tot} elements per process "
                      f"({len(nums)} buckets), element-parallel oracle, {secs:.1f} s",
            "scalar_1core_GBs": round(res["scalar"][0], 3)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--order", choices=("fixed", "fast"), default="fixed")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true")
    ap.add_argument("--launch", default="", help="key=value,... passed to eager_set_launch")
    ap.add_argument("--stagger", type=int, default=0, help="bytes of base offset per stream")
    ap.add_argument("--clip", type=int, default=0,
                    help="clip every tensor to this many elements (a reduced layout of the same "
                         "configuration, for counter runs the profiler cannot take at full size)")
    ap.add_argument("--trace", default="", metavar="FILE",
                    help="after the timed run, log this many more steps one by one to FILE "
                         "(JSON lines: NAP, initiator, mask, bytes, GPU microseconds)")
    ap.add_argument("--unfused", action="store_true",
                    help="A/B: partial allreduce into a receive buffer, then eager_sgd_step (same "
                         "algorithmic bytes in the numerator, 8 B/element more traffic)")
    ap.add_argument("--stats", action="store_true",
                    help="also compute the per-bucket norms in every round (eager_stats_attach)")
    ap.add_argument("--views", action="store_true",
                    help="a weight view per process: the round goes to the receive buffer and "
                         "eager_sgd_step_views applies it to all P views (P x (w, v) more memory; the "
                         "numerator stays the single-view path's algorithmic bytes)")
    ap.add_argument("--light-setup", action="store_true",
                    help="inputs with few kernel dispatches (every process's gradient arena is a copy "
                         "of process 0's): for `rocprofv3 --pmc` runs on the largest configurations")
    ap.add_argument("--lars", type=float, default=0.0, metavar="TRUST",
                    help="update rule with a layer-wise rate per bucket (eager_sgd_step_lars with this "
                         "trust coefficient) on the receive buffer of an unfused round; the numerator "
                         "stays the fused path's algorithmic bytes")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (P simulated processes share its HBM); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    from paper_1908_04207_amd import build as hip_build
    hip_build.ensure_built()             # compiles only if no library has been built
    launch = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in a.launch.split(",") if kv}
    wl, wall, nbytes, kern_s = run_gpu(a.config, a.steps, a.warmup, a.order, launch, a.stagger,
                                       a.clip, a.stats, a.unfused, a.lars, a.light_setup, a.views)
    cfg = wl.cfg
    total_b = sum(nbytes)
    traffic = MEASURED_TRAFFIC.get(cfg.name)
    achieved = total_b / kern_s / 1e9
    out = {
        "metric": "effective reduce+update GB/s (fused partial allreduce + momentum SGD)",
        "value": round(total_b / wall / 1e9, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(wall / a.steps * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",          # the arithmetic type (sums, average, update rule); gradients
                                 # may be stored as bf16, see config.grad_dtype
        "data": "synthetic",
        "config": {"workload": cfg.name, "P": cfg.P, "mode": cfg.mode, "grad_dtype": cfg.grad_dtype,
                   "elements_per_process": cfg.numel, "buckets": cfg.buckets.n_buckets,
                   "order": a.order, "launch": launch, "stagger": a.stagger,
                   "bucket_stats": a.stats or a.lars > 0, "unfused": a.unfused or a.lars > 0,
                   "lars_trust": a.lars, "weight_views": cfg.P if a.views else 1},
        "steps_per_s": round(a.steps / wall, 2),
        "pct_hbm_peak": round(100.0 * total_b / wall / 1e9 / HBM_PEAK_GBS, 2),
        "alg_bytes_per_step": round(total_b / a.steps),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic["bytes_per_launch"] if traffic else None,
                     "traffic_note": traffic["note"] if traffic else None,
                     "kernel": ("slot_kernel<bf16> (fused round)" if cfg.grad_dtype == "bf16" else
                                "slot_kernel (+ carry_kernel when the round is split)"),
                     "avg_kernel_ms": round(kern_s / a.steps * 1e3, 5)},
        "paper_context": PAPER_CONTEXT,
    }
    if a.trace:
        trace_steps(wl, min(a.steps, 64), a.trace)
    if not a.no_ceiling:
        c = copy_ceiling_gbs()
        out["measured_ceiling_GBs"] = {"copy_read_plus_write": round(c["copy"], 1),
                                       "read_only": round(c["read"], 1)}
        out["pct_of_measured_copy"] = round(100.0 * achieved / c["copy"], 1)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
