#!/usr/bin/env python3
"""Throughput of the fused eager-SGD round (partial allreduce + carry + momentum SGD) on
one MI355X, on synthetic gradients shaped like the paper's workloads.

A step = plan participation from that step's seeded compute times (host) + one fused
round over every bucket of the model (device).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.  Without --config it times all five configurations
one after the other: the headline fields (value, ms_per_step, roofline, cpu_baseline) are
those of the largest all-fp32 configuration (cfg4, timed with exactly --steps steps) and
`per_config` holds one entry per configuration.  With --config K only that configuration
runs (for sweeps, traces and profiler runs).

  python bench.py [--steps K] [--warmup W]
  python bench.py --config 3 [--order fixed|fast] [--launch key=value,...] [--unfused] ...
  python bench.py --aux                    # the auxiliary kernels, one line each
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
LLC_BYTES = 256 << 20      # last-level cache: w and v up to this size are left to it
HEADLINE = 4               # largest configuration whose buffers are all fp32
# timed steps per configuration as a multiple of --steps (the headline uses --steps itself):
# enough for some tens of milliseconds of timed work on the small ones
STEP_FACTOR = {1: 200, 2: 10, 3: 2, 4: 1, 5: 1}
TRAFFIC_FILE = os.path.join(ROOT, "bench_traffic.json")
PAPER_CONTEXT = ("paper (Piz Daint, Xeon E5-2690 + P100 per node, Cray Aries, fp32): eager-SGD "
                 "1.29x over Deep500 / 1.27x over Horovod (ResNet-50, 64 proc), 1.27x over "
                 "Horovod (LSTM/UCF101, majority), 2.64x over async PS; end-to-end training "
                 "throughput on a cluster, not this kernel: context only")


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
        self.k = k
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
        self.rounds = []       # (nap, q_prev, q_now) of every step taken
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

    def step(self, exchange: bool = False) -> int:
        """One step; returns its algorithmic bytes.  exchange: the round in which the gradient
        buffer of a late process becomes its send buffer (fp32 gradients only); it moves, and
        is credited with, fewer bytes."""
        cfg = self.cfg
        plan = self.last_plan = self.plan(self.step_no)
        if exchange:
            self.ctx.eager_partial_allreduce_exchange(plan, self.Gp, self.Rp, recv=None,
                                                      opt=(self.w, self.v, cfg.lr, cfg.mu),
                                                      stream=self.stream)
            q_now = cfg.P - plan.nap
            b = (4 * (plan.nap + self.q_prev) + 16) * cfg.numel
            self.rounds.append((plan.nap, self.q_prev, q_now))
            self.q_prev = q_now
            self.step_no += 1
            return b
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
        self.rounds.append((plan.nap, self.q_prev, q_now))
        self.q_prev = q_now
        self.step_no += 1
        return b

    def release(self) -> None:
        """Give the device memory back before the next configuration is set up."""
        for name in ("G", "R", "w", "v", "recv", "wp", "vp", "stats", "stats_ws", "Gp", "Rp"):
            if hasattr(self, name):
                delattr(self, name)
        self.ctx.close()
        self.torch.cuda.empty_cache()


def time_steps(wl: "Workload", steps: int, warmup: int, exchange: bool = False):
    """W untimed steps, then K timed ones: wall-clock seconds (synchronised on both sides),
    algorithmic bytes per step, GPU seconds between two HIP events on the launch stream."""
    import torch
    wl.prepare(wl.step_no, warmup + steps)
    for _ in range(warmup):
        wl.step(exchange)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    nbytes = []
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        nbytes.append(wl.step(exchange))
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, nbytes, e0.elapsed_time(e1) * 1e-3


def run_gpu(k: int, steps: int, warmup: int, order: str, launch=None, stagger=0, clip=0,
            stats=False, unfused=False, lars=0.0, light_setup=False, views=False):
    """W untimed steps, then K timed steps.  Returns the workload, the wall-clock seconds
    of the K steps (synchronised on both sides), their algorithmic bytes, and the GPU time
    of the same K steps between two HIP events recorded on the launch stream (torch's
    current stream, which is the one the binding launches on)."""
    wl = Workload(k, order, launch, stagger, clip, stats, unfused, lars, light_setup, views)
    wall, nbytes, kern_s = time_steps(wl, steps, warmup)
    return wl, wall, nbytes, kern_s


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


def _gpu_ms(fn, reps: int) -> float:
    import torch
    fn()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(reps):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / reps


class Calibration:
    """Plain kernels of known traffic on buffers of gradient-like data, for context: a copy,
    a read-only stream, and a kernel with the same mix of read and write streams as a
    configuration's rounds (eager_calib_mix)."""

    VEC = 1 << 22          # 16-byte lane-vectors per stream: 64 MiB, beyond every cache

    def __init__(self):
        import torch
        self.torch = torch
        self.pool = []
        self.seed = (torch.randn(self.VEC * 4, device="cuda") * 1e-3)
        self.sink = torch.zeros(4, device="cuda")

    def streams(self, n: int):
        # what the buffers hold changes the rate by 1-2 %: random data, not zeros
        while len(self.pool) < n:
            self.pool.append(self.seed.clone())
        return self.pool[:n]

    def copy_and_read(self) -> dict:
        from paper_1908_04207_amd import binding as eb
        n = 1 << 30
        a = (self.torch.randn(n // 4, device="cuda") * 1e-3).view(self.torch.uint8)
        b = self.torch.empty(n, dtype=self.torch.uint8, device="cuda")
        out = {"copy_read_plus_write": round(2 * n / (_gpu_ms(lambda: eb.eager_calib_copy(b, a, n), 10) * 1e-3) / 1e9, 1),
               "read_only": round(n / (_gpu_ms(lambda: eb.eager_calib_read(a, n, self.sink), 10) * 1e-3) / 1e9, 1)}
        del a, b
        self.torch.cuda.empty_cache()
        return out

    def stream_mix(self, P: int, gbytes: int, nap: int, q_prev: int, q_now: int) -> dict:
        """Best rate of plain kernels that move one round's streams (nap on-time gradients,
        q_prev pending send buffers, q_now late gradients stored, w and v) - as one pass, or
        as the reduction's streams followed by the copies of the late gradients - over
        occupancy caps of 3..24 wavefronts per CU and none.  The numerator is the round's algorithmic
        bytes, as for the rounds themselves."""
        from paper_1908_04207_amd import binding as eb
        half = gbytes == 2
        nv = self.VEC
        alg = alg_bytes_per_element(P, gbytes, q_prev, q_now) * nv * 4
        caps = (3, 4, 5, 6, 8, 10, 12, 16, 24, 0)       # 0: no cap

        def best(n_read, n_half, n_write):
            n_read, n_write = min(n_read, 80), min(n_write, 80)
            bufs = self.streams(n_read + n_write)
            rd, wr = eb.Context.pointers(bufs[:n_read]), eb.Context.pointers(bufs[n_read:])
            mask = (1 << min(n_half, 64)) - 1
            return min(_gpu_ms(lambda: eb.eager_calib_mix(rd, wr, nv, mask, c, self.sink), 3)
                       for c in caps)
        # one pass: every gradient and every pending send buffer read, late gradients and w, v written
        fused = best(P + q_prev + 2, P if half else 0, q_now + 2)
        out = {"one_pass": round(alg / (fused * 1e-3) / 1e9, 1)}
        if q_now:
            # reduction's streams (only the on-time gradients), then q_now copies G -> R
            reduce_ms = best(nap + q_prev + 2, nap if half else 0, 2)
            copy_ms = q_now * best(1, 1 if half else 0, 1)
            out["reduction_then_copies"] = round(alg / ((reduce_ms + copy_ms) * 1e-3) / 1e9, 1)
        out["best"] = max(out.values())
        out["round"] = {"on_time": nap, "pending_send_buffers": q_prev, "late": q_now}
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


def committed_traffic(cfg_name: str, default_launch: bool):
    """L2 <-> fabric bytes per round from the committed rocprofv3 counter runs
    (bench_traffic.json, written by `bench.py --record-traffic`), or None when the library
    has changed since they were taken or this run is not the default launch."""
    from paper_1908_04207_amd import binding as eb
    if not default_launch or not os.path.exists(TRAFFIC_FILE):
        return None
    with open(TRAFFIC_FILE) as f:
        rec = json.load(f)
    if rec.get("source_hash") != eb.source_hash():
        return None
    return rec.get("configs", {}).get(cfg_name)


def llc_resident_bytes(wl: Workload, step_bytes: float) -> int:
    """Algorithmic bytes of a step that the 256 MiB last-level cache can serve instead of
    HBM: w and v (read and written every step, 16 B/element) when they fit it - the library
    then leaves them cached on purpose; everything when the whole working set fits."""
    cfg = wl.cfg
    n = cfg.numel
    working_set = n * (cfg.P * (wl.gbytes + 4) + 8)
    if working_set <= LLC_BYTES:
        return int(step_bytes)
    return 16 * n if 8 * n <= LLC_BYTES else 0


def measure(k: int, steps: int, warmup: int, order: str, calib: Calibration | None, **kw):
    """Times one configuration and returns (workload, its per_config entry)."""
    no_exchange = kw.pop("no_exchange", False)
    wl, wall, nbytes, kern_s = run_gpu(k, steps, warmup, order, **kw)
    kw["no_exchange"] = no_exchange
    cfg = wl.cfg
    total_b = sum(nbytes)
    step_b = total_b / steps
    achieved = total_b / kern_s / 1e9
    resident = llc_resident_bytes(wl, step_b)
    entry = {
        "workload": cfg.name, "P": cfg.P, "mode": cfg.mode, "grad_dtype": cfg.grad_dtype,
        "elements_per_process": cfg.numel, "buckets": cfg.buckets.n_buckets,
        "steps": steps, "warmup": warmup,
        "ms_per_step": round(wall / steps * 1e3, 5),
        "steps_per_s": round(steps / wall, 2),
        "alg_bytes_per_step": round(step_b),
        "value_GBs": round(total_b / wall / 1e9, 2),
        "achieved_GBs": round(achieved, 2),
        "avg_kernel_ms_per_step": round(kern_s / steps * 1e3, 5),
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "llc_resident_bytes_per_step": resident,
        "hbm_frac": round((total_b - resident * steps) / kern_s / 1e9 / HBM_PEAK_GBS, 4),
        "cache_resident": resident >= step_b,
        "kernels_per_round": ("slot_kernel (one fused pass)" if cfg.grad_dtype == "bf16" else
                              "slot_kernel; in rounds the library splits, slot_kernel (reduction + "
                              "update) then carry_kernel (late gradients into the send buffers)"),
    }
    plain = not (kw.pop("no_exchange", False) or kw.get("stats") or kw.get("unfused") or
                 kw.get("lars") or kw.get("views"))
    if cfg.grad_dtype == "f32" and plain and not entry["cache_resident"]:
        # the same workload with eager_partial_allreduce_exchange: a late gradient's buffer
        # becomes the send buffer, nothing is copied; fewer bytes moved AND credited
        timed = wl.rounds[warmup:]
        xwall, xbytes, xkern = time_steps(wl, steps, warmup, exchange=True)
        entry["exchange_round"] = {
            "ms_per_step": round(xwall / steps * 1e3, 5), "steps_per_s": round(steps / xwall, 2),
            "alg_bytes_per_step": round(sum(xbytes) / steps),
            "achieved_GBs": round(sum(xbytes) / xkern / 1e9, 2),
            "frac": round(sum(xbytes) / xkern / 1e9 / HBM_PEAK_GBS, 4),
            "speedup_in_steps_per_s": round((wall / steps) / (xwall / steps), 3),
            "note": "4*(on time + pending) + 16 bytes per element; w, v up to 256 MiB may be served "
                    "by the last-level cache"}
        wl.rounds = wl.rounds[:warmup] + timed
    if calib is not None:
        mid = sorted(wl.rounds[warmup:], key=lambda r: r[2])[len(wl.rounds[warmup:]) // 2]
        mix = calib.stream_mix(cfg.P, wl.gbytes, *mid)
        entry["stream_mix_ceiling_GBs"] = mix
        entry["pct_of_stream_mix_ceiling"] = round(100.0 * achieved / mix["best"], 1)
    return wl, entry


def aux_lines(log2_elements: int, views: int, buckets: int, reps: int) -> None:
    """Bandwidth of the auxiliary kernels, each on its own: the send-buffer stash, the update
    rule on a receive buffer (plain, with a layer-wise rate, on several weight views) and the
    model average.  One line per kernel: milliseconds per call (HIP events on the launch
    stream) and the algorithmic bytes of the call divided by that time."""
    import torch
    from paper_1908_04207_amd import binding as eb
    n = 1 << log2_elements
    per = n // buckets // 8 * 8
    offset = [b * per for b in range(buckets)]
    numel = [per] * (buckets - 1) + [n - per * (buckets - 1)]
    dev = torch.device("cuda:0")

    def report(name: str, nbytes: int, fn) -> None:
        ms = _gpu_ms(fn, reps)
        print(f"{name:44s} {ms:9.4f} ms  {nbytes / (ms * 1e-3) / 1e9:7.0f} GB/s", flush=True)

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
    w = [torch.randn(n, device=dev) * 0.02 for _ in range(views)]
    v = [torch.zeros(n, device=dev) for _ in range(views)]
    report("eager_sgd_step", 20 * n, lambda: ctx.eager_sgd_step(u, (w[0], v[0], 0.1, 0.9)))
    stats = torch.zeros(buckets * 4, dtype=torch.float64, device=dev)
    nbytes = ctx.eager_stats_workspace_bytes()
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ctx.eager_stats_attach(stats, ws, nbytes)
    report("eager_sgd_step_lars (norms, rate, update)", 28 * n,
           lambda: ctx.eager_sgd_step_lars(u, (w[0], v[0], 0.1, 0.9), 0.02, 1e-9))
    ctx.eager_stats_attach(None, None)
    report(f"eager_sgd_step x {views} views, one call each", 20 * views * n,
           lambda: [ctx.eager_sgd_step(u, (w[i], v[i], 0.1, 0.9)) for i in range(views)])
    report(f"eager_sgd_step_views, {views} views", (4 + 16 * views) * n,
           lambda: ctx.eager_sgd_step_views(u, w, v, 0.1, 0.9))
    report(f"eager_average_views, {views} views", 8 * views * n,
           lambda: ctx.eager_average_views(w))
    ctx.close()


def record_traffic(spec: str) -> int:
    """--record-traffic K:FETCH.csv:WRITE.csv[,...]: turn rocprofv3 --pmc FETCH_SIZE and
    WRITE_SIZE runs of `bench.py --config K --light-setup` (counter_collection csv files) into
    bench_traffic.json: L2 <-> fabric bytes per round, scaled by what the same counter reads
    for the library's plain copy kernel on 1 GiB in the same run, stamped with the digest of
    the library's sources."""
    import csv
    from paper_1908_04207_amd import build as hip_build
    from workloads import shapes
    rec = {"source_hash": hip_build.source_hash(),
           "what": "L2 <-> fabric bytes per round (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, KiB "
                   "per dispatch, each scaled by the same counter's reading for the 1 GiB copy "
                   "kernel of the same run); reads and writes that the last-level cache serves "
                   "are included, so this is an upper bound on HBM bytes",
           "configs": {}}
    if os.path.exists(TRAFFIC_FILE):
        with open(TRAFFIC_FILE) as f:
            old = json.load(f)
        if old.get("source_hash") == rec["source_hash"]:
            rec["configs"] = old.get("configs", {})

    def per_kernel(path, counter):
        agg = {}
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] == counter and "eager::" in r["Kernel_Name"]:
                for tag in ("slot_kernel", "carry_kernel", "copy_kernel"):
                    if tag in r["Kernel_Name"]:
                        agg.setdefault(tag, []).append(float(r["Counter_Value"]))
        return agg
    for item in spec.split(","):
        k, fetch_csv, write_csv = item.split(":")
        cfg = shapes.config(int(k))
        f, w = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
        gib_kib = float(1 << 20)
        fs = gib_kib / (sum(f["copy_kernel"]) / len(f["copy_kernel"]))
        ws = gib_kib / (sum(w["copy_kernel"]) / len(w["copy_kernel"]))
        rounds = len(f["slot_kernel"])
        total = 0.0
        for tag in ("slot_kernel", "carry_kernel"):
            total += sum(f.get(tag, [])) * fs * 1024 + sum(w.get(tag, [])) * ws * 1024
        # algorithmic bytes of the same rounds (0 .. rounds-1 of the configuration)
        from paper_1908_04207_amd import binding as eb
        from workloads import times
        g = 2 if cfg.grad_dtype == "bf16" else 4
        q_prev, alg = 0, 0
        for t in range(rounds):
            plan = eb.eager_plan_participation(eb.SOLO if cfg.mode == "solo" else eb.MAJORITY,
                                               times.compute_times(cfg.times, cfg.P, cfg.seed, t),
                                               cfg.seed, t)
            alg += alg_bytes_per_element(cfg.P, g, q_prev, cfg.P - plan.nap) * cfg.numel
            q_prev = cfg.P - plan.nap
        rec["configs"][cfg.name] = {"bytes_per_round": round(total / rounds), "rounds": rounds,
                                    "algorithmic_bytes_per_round_same_rounds": round(alg / rounds),
                                    "over_algorithmic": round(total / alg, 4),
                                    "fetch_scale": round(fs, 4), "write_scale": round(ws, 4)}
    with open(TRAFFIC_FILE, "w") as fh:
        json.dump(rec, fh, indent=1)
        fh.write("\n")
    print(json.dumps(rec))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=0,
                    help="time only this configuration (default: all five, headline cfg4)")
    ap.add_argument("--order", choices=("fixed", "fast"), default="fixed")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true")
    ap.add_argument("--no-exchange", action="store_true",
                    help="skip the extra timing of eager_partial_allreduce_exchange (profiler runs: "
                         "only the rounds of the headline path are launched)")
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
    ap.add_argument("--aux", action="store_true",
                    help="time the auxiliary kernels (stash, update rule alone, weight views) instead")
    ap.add_argument("--log2-elements", type=int, default=26, help="--aux: elements per buffer")
    ap.add_argument("--aux-views", type=int, default=8, help="--aux: weight views")
    ap.add_argument("--record-traffic", default="", metavar="K:FETCH.csv:WRITE.csv,...",
                    help="no GPU work: write bench_traffic.json from rocprofv3 counter csv files")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (P simulated processes share its HBM); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        return 2
    if a.record_traffic:
        return record_traffic(a.record_traffic)
    # before anything touches the GPU: a compile, if one is needed, starts child processes
    from paper_1908_04207_amd import build as hip_build
    hip_build.ensure_built()
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if a.aux:
        aux_lines(a.log2_elements, a.aux_views, 64, 20)
        return 0
    launch = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in a.launch.split(",") if kv}
    variant = dict(launch=launch, stagger=a.stagger, clip=a.clip, stats=a.stats, unfused=a.unfused,
                   lars=a.lars, light_setup=a.light_setup, views=a.views)
    default_launch = not (launch or a.stagger or a.clip or a.stats or a.unfused or a.lars or a.views
                          or a.order != "fixed")
    calib = None if a.no_ceiling else Calibration()
    ceilings = calib.copy_and_read() if calib else None
    headline = a.config or HEADLINE
    per_config, head, cpu = [], None, None
    # the headline first, on a device whose memory nothing has been carved out of yet; its CPU
    # leg runs while its inputs are still there, then the memory goes back before the next one
    for k in ([a.config] if a.config else [headline] + [c for c in (1, 2, 3, 5, 4) if c != headline]):
        steps = a.steps if k == headline else a.steps * STEP_FACTOR[k]
        wl, entry = measure(k, steps, a.warmup, a.order, calib if k != 1 else None,
                            no_exchange=a.no_exchange, **variant)
        per_config.append(entry)
        if k == headline:
            head, cfg = entry, wl.cfg
            if a.trace:
                trace_steps(wl, min(a.steps, 64), a.trace)
            if not a.no_cpu_baseline:
                cpu = cpu_baseline(wl)
        wl.release()
        del wl
    per_config.sort(key=lambda e: e["workload"])
    traffic = committed_traffic(cfg.name, default_launch)
    out = {
        "metric": "effective reduce+update GB/s (fused partial allreduce + momentum SGD)",
        "value": head["value_GBs"], "unit": "GB/s",
        "n_gpus": 1, "steps": head["steps"], "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",          # the arithmetic type (sums, average, update rule); gradients
                                 # may be stored as bf16, see config.grad_dtype
        "data": "synthetic",
        "config": {"workload": cfg.name, "P": cfg.P, "mode": cfg.mode, "grad_dtype": cfg.grad_dtype,
                   "elements_per_process": cfg.numel, "buckets": cfg.buckets.n_buckets,
                   "order": a.order, "launch": launch, "stagger": a.stagger,
                   "bucket_stats": a.stats or a.lars > 0, "unfused": a.unfused or a.lars > 0,
                   "lars_trust": a.lars, "weight_views": cfg.P if a.views else 1},
        "steps_per_s": head["steps_per_s"],
        "pct_hbm_peak": round(100.0 * head["value_GBs"] / HBM_PEAK_GBS, 2),
        "alg_bytes_per_step": head["alg_bytes_per_step"],
        "roofline": {"bound": "hbm", "achieved": head["achieved_GBs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": head["frac"],
                     "hbm_frac": head["hbm_frac"],
                     "llc_resident_bytes_per_step": head["llc_resident_bytes_per_step"],
                     "traffic": traffic["bytes_per_round"] if traffic else None,
                     "traffic_kind": ("L2 <-> fabric bytes per round (FETCH_SIZE + WRITE_SIZE, scaled "
                                      "by a copy kernel of known size); includes what the last-level "
                                      "cache serves, so an upper bound on HBM bytes") if traffic else None,
                     "traffic_source": ("bench_traffic.json, taken with the library whose source digest "
                                        "matches the one loaded now, on rounds 0..%d of the configuration, whose "
                                        "algorithmic bytes are %d per round: ratio %.4f" %
                                        (traffic["rounds"] - 1, traffic["algorithmic_bytes_per_round_same_rounds"],
                                         traffic["over_algorithmic"])) if traffic else None,
                     "kernel": head["kernels_per_round"],
                     "avg_kernel_ms": head["avg_kernel_ms_per_step"]},
        "per_config": per_config,
        "paper_context": PAPER_CONTEXT,
    }
    if ceilings:
        out["measured_ceiling_GBs"] = dict(ceilings)
        if "stream_mix_ceiling_GBs" in head:
            out["measured_ceiling_GBs"]["stream_mix"] = head["stream_mix_ceiling_GBs"]["best"]
        out["pct_of_measured_copy"] = round(100.0 * head["achieved_GBs"] / ceilings["copy_read_plus_write"], 1)
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
