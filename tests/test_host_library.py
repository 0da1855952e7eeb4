"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, plans participation exactly like the oracle, and rejects bad
arguments before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import eager_oracle as eo
from paper_1908_04207_amd import binding as eb
from workloads import shapes, times

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read()
                     for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(eager_[a-z_]+)\s*\(", header))
    assert declared == set(eb.EXPORTS)
    lib = ctypes.CDLL(eb.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_header_is_plain_c_and_host_calls_run_from_c(tmp_path):
    """include/eager.h in a C99 translation unit (gcc, pedantic), every entry point with its
    declared type, structure layouts; the program links against the library and runs the
    host-only planning calls (no GPU needed)."""
    import subprocess
    exe = tmp_path / "header_is_plain_c"
    lib_dir = os.path.dirname(eb.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                           "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c", "header_is_plain_c.c"),
                           "-o", str(exe), "-L", lib_dir, "-leager", "-Wl,-rpath," + lib_dir])
    assert subprocess.run([str(exe)]).returncode == 0


def test_plan_matches_oracle_on_all_configs():
    for k in range(1, 6):
        cfg = shapes.config(k)
        lm = eb.SOLO if cfg.mode == "solo" else eb.MAJORITY
        om = eo.SOLO if cfg.mode == "solo" else eo.MAJORITY
        for step in range(cfg.steps):
            t = times.compute_times(cfg.times, cfg.P, cfg.seed, step)
            a = eb.eager_plan_participation(lm, t, cfg.seed, step)
            b = eo.plan_participation(om, cfg.P, t, cfg.seed, step)
            assert (a.mode, a.P, a.step, a.mask, a.initiator, a.nap) == \
                   (lm, cfg.P, step, b.mask, b.initiator, b.nap)


def test_designated_initiator_is_the_published_splitmix64_sequence():
    """The shared-seed draw of the majority initiator (Section 4.2) against the published
    SplitMix64 outputs for seed 0: the residues of a 64-bit value modulo every P in 1..64
    determine it (their least common multiple exceeds 2^64), so this pins the library's and the
    oracle's generator completely through the planner alone."""
    path = os.path.join(ROOT, "tests", "golden", "splitmix64_seed0.txt")
    published = [int(l, 16) for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(published) == 3
    for step, value in enumerate(published):
        for P in range(1, 65):
            times_ = [float(p) for p in range(P)]
            assert eb.eager_plan_participation(eb.MAJORITY, times_, 0, step).initiator == value % P
            assert eo.plan_participation(eo.MAJORITY, P, times_, 0, step).initiator == value % P


def test_open_round_trigger_rule():
    """eager_plan_open_round (processes with their own clocks, Section 5 last paragraph): solo
    triggers as soon as anybody waits, majority when the designated initiator waits, quorum q at
    q waiting processes; the plan's active set is the waiting set."""
    rng = np.random.default_rng(5)
    for it in range(3000):
        P = int(rng.integers(1, 65))
        waiting = 0
        while waiting == 0:
            waiting = int(rng.integers(0, 2 ** 62)) & ((1 << P) - 1) if P < 62 else \
                int(rng.integers(0, 2 ** 62)) | (1 << (P - 1))
        members = [p for p in range(P) if (waiting >> p) & 1]
        newest = int(rng.choice(members))
        seed, rnd = int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 1000))
        designated = eo.initiator_hash(seed, rnd) % P
        assert eb.eager_designated_initiator(seed, rnd, P) == designated
        solo = eb.eager_plan_open_round(eb.SOLO, P, waiting, newest, rnd)
        assert solo is not None and (solo.mask, solo.initiator, solo.nap, solo.step, solo.mode) == \
            (waiting, members[0], len(members), rnd, eb.SOLO)
        maj = eb.eager_plan_open_round(eb.MAJORITY, P, waiting, newest, rnd, seed=seed)
        assert (maj is not None) == (designated in members)
        if maj is not None:
            assert (maj.mask, maj.initiator, maj.nap) == (waiting, designated, len(members))
        q = int(rng.integers(1, P + 1))
        quo = eb.eager_plan_open_round(eb.QUORUM, P, waiting, newest, rnd, quorum=q)
        assert (quo is not None) == (len(members) >= q)
        if quo is not None:
            assert (quo.mask, quo.initiator, quo.mode) == (waiting, newest, eb.QUORUM)
    for bad in (dict(waiting=0, newest=0), dict(waiting=0b10000, newest=4), dict(waiting=0b0011, newest=2)):
        with pytest.raises(eb.EagerError):
            eb.eager_plan_open_round(eb.SOLO, 4, bad["waiting"], bad["newest"], 0)
    with pytest.raises(eb.EagerError):
        eb.eager_plan_open_round(eb.QUORUM, 4, 0b0011, 1, 0, quorum=5)


def test_strict_quorum_is_enforced_where_the_round_is_entered():
    """Majority as "at least half of the processes" (Section 4.2, first paragraph): the planner
    records the flag in the plan and eager_partial_allreduce_majority refuses such a plan with
    fewer than ceil(P/2) active processes before anything is launched."""
    P = 5
    c = eb.Context(P, [0], [64])
    ptrs = [0x10000 * (p + 1) for p in range(P)]
    opt = (0x900000, 0xA00000, 0.1, 0.9)
    plan = eb.eager_plan_participation(eb.MAJORITY, [5.0, 1.0, 4.0, 2.0, 3.0], 3, 0, 0.0,
                                       eb.FLAG_STRICT_QUORUM)
    assert plan.flags == eb.FLAG_STRICT_QUORUM and plan.nap >= 3
    assert eb.eager_plan_participation(eb.MAJORITY, [5.0, 1.0, 4.0, 2.0, 3.0], 3, 0).flags == 0
    for nap_mask, ok in ((0b00011, False), (0b00111, True)):
        forged = eb.make_plan(eb.MAJORITY, P, 9, nap_mask, flags=eb.FLAG_STRICT_QUORUM)
        if ok:
            continue                                   # would launch: covered on the GPU
        with pytest.raises(eb.EagerError) as err:
            c.eager_partial_allreduce_majority(forged, ptrs, ptrs, opt=opt, stream=0)
        assert err.value.status == eb.ESTATE and "strict majority" in str(err.value)
    # without the flag the same participation set is accepted by the checks (a plan built by hand
    # promises nothing): it fails later, on purpose, with a NULL gradient pointer instead
    with pytest.raises(eb.EagerError) as err:
        c.eager_partial_allreduce_majority(eb.make_plan(eb.MAJORITY, P, 9, 0b00011),
                                           [0] * P, ptrs, opt=opt, stream=0)
    assert err.value.status == eb.EINVAL
    with pytest.raises(eb.EagerError) as err:                      # unknown flag bits
        c.eager_partial_allreduce_majority(eb.make_plan(eb.MAJORITY, P, 9, 0b00111, flags=8), ptrs, ptrs,
                                           opt=opt, stream=0)
    assert err.value.status == eb.ESTATE
    c.close()


def test_plan_matches_oracle_random_with_ties_window_and_strict_quorum():
    rng = np.random.default_rng(0)
    for it in range(2000):
        P = int(rng.integers(1, 65))
        t = rng.integers(0, 6, P).astype(float).tolist() if it % 2 else rng.random(P).tolist()
        seed = int(rng.integers(0, 2 ** 63))
        window = float(rng.choice([0.0, 0.5, 2.0]))
        for lm, om in ((eb.SOLO, eo.SOLO), (eb.MAJORITY, eo.MAJORITY)):
            for flags in (0, eb.FLAG_STRICT_QUORUM):
                a = eb.eager_plan_participation(lm, t, seed, it, window, flags)
                b = eo.plan_participation(om, P, t, seed, it, window, flags)
                assert (a.mask, a.initiator, a.nap) == (b.mask, b.initiator, b.nap)


def test_quorum_plan_matches_oracle_and_spans_solo_to_full():
    """k-of-P participation (Section 9): same sets as the oracle; k = 1 is the solo set,
    k = P everybody; the set grows with k."""
    rng = np.random.default_rng(1)
    for it in range(500):
        P = int(rng.integers(1, 65))
        t = rng.integers(0, 6, P).astype(float).tolist() if it % 2 else rng.random(P).tolist()
        window = float(rng.choice([0.0, 0.5]))
        prev = 0
        for k in range(1, P + 1):
            a = eb.eager_plan_quorum(t, k, it, window)
            b = eo.plan_participation(eo.QUORUM, P, t, 0, it, window, quorum=k)
            assert (a.mode, a.mask, a.initiator, a.nap) == (eb.QUORUM, b.mask, b.initiator, b.nap)
            assert a.nap >= k and a.mask & prev == prev
            prev = a.mask
        assert eb.eager_plan_quorum(t, 1, it, window).mask == \
            eb.eager_plan_participation(eb.SOLO, t, 0, it, window).mask
        assert eb.eager_plan_quorum(t, P, it).mask == (1 << P) - 1
    for bad in (lambda: eb.eager_plan_quorum([1.0, 2.0], 0, 0),
                lambda: eb.eager_plan_quorum([1.0, 2.0], 3, 0),
                lambda: eb.eager_plan_quorum([1.0, float("nan")], 1, 0),
                lambda: eb.eager_plan_quorum([1.0], 1, 0, window_ms=-1.0)):
        with pytest.raises(eb.EagerError) as e:
            bad()
        assert e.value.status == eb.EINVAL


def test_microbenchmark_latency_shape_and_nap():
    """The paper's microbenchmark (Section 7.1, Fig. 9): 32 processes skewed linearly from 1
    to 32 ms, 64 iterations.  With the library's planner and the simplest latency model - a
    process waits from its arrival until the initiator triggers the round, then the
    collective itself takes t_c - the waits have closed forms, and the reported ratios
    (53.32x for solo, 2.46x for majority over the full allreduce) fall where those forms put
    them for a collective of a few hundred microseconds.  NAP: exactly 1 for solo, rank of
    the initiator + 1 for majority, about half the processes on average."""
    from harness import paper_values
    pv = paper_values()
    P, iters = int(pv["microbench_processes"]), int(pv["microbench_iterations"])
    arrival = [float(p) for p in range(int(pv["microbench_skew_first_ms"]),
                                       int(pv["microbench_skew_last_ms"]) + 1)]
    assert len(arrival) == P

    def mean_wait(plans):
        return sum(sum(max(0.0, arrival[pl.initiator] - a) for a in arrival) / P
                   for pl in plans) / len(plans)

    solo = [eb.eager_plan_participation(eb.SOLO, arrival, 3, t) for t in range(iters)]
    full = [eb.eager_plan_quorum(arrival, P, t) for t in range(iters)]
    assert all(pl.nap == pv["microbench_solo_nap"] and pl.initiator == 0 for pl in solo)
    assert all(pl.nap == P and pl.initiator == P - 1 for pl in full)
    assert mean_wait(solo) == 0.0
    assert mean_wait(full) == (P - 1) / 2.0                       # mean of 31, 30, ..., 0 ms
    naps, waits = [], []
    for seed in range(200):
        maj = [eb.eager_plan_participation(eb.MAJORITY, arrival, seed, t) for t in range(iters)]
        assert all(pl.nap == pl.initiator + 1 for pl in maj)
        naps.append(sum(pl.nap for pl in maj) / iters)
        waits.append(mean_wait(maj))
    # initiator uniform over the ranks: E[NAP] = (P+1)/2, E[wait] = (P^2 - 1) / (6 P) ms
    assert abs(np.mean(naps) - (P + 1) / 2.0) < 0.15
    assert abs(np.mean(naps) - pv["microbench_majority_nap"]) < 1.0
    assert abs(np.mean(waits) - (P * P - 1) / (6.0 * P)) < 0.1
    t_c = 0.3                                                     # ms, a small-message allreduce
    lat_full, lat_solo, lat_maj = (P - 1) / 2.0 + t_c, t_c, float(np.mean(waits)) + t_c
    assert 0.75 < (lat_full / lat_solo) / pv["microbench_solo_latency_ratio"] < 1.3
    assert 0.8 < (lat_full / lat_maj) / pv["microbench_majority_latency_ratio"] < 1.4
    assert lat_solo < lat_maj < lat_full


def test_plan_rejects_bad_arguments():
    for bad in (lambda: eb.eager_plan_participation(7, [1.0], 0, 0),
                lambda: eb.eager_plan_participation(eb.SOLO, [], 0, 0),
                lambda: eb.eager_plan_participation(eb.SOLO, [1.0] * 65, 0, 0),
                lambda: eb.eager_plan_participation(eb.SOLO, [float("nan")], 0, 0),
                lambda: eb.eager_plan_participation(eb.SOLO, [1.0], 0, 0, window_ms=-1.0)):
        with pytest.raises(eb.EagerError) as e:
            bad()
        assert e.value.status == eb.EINVAL


def test_create_rejects_bad_bucket_tables():
    for P, off, num, dt, status in (
            (0, [0], [4], eb.F32, eb.EINVAL), (65, [0], [4], eb.F32, eb.EINVAL),
            (2, [], [], eb.F32, eb.EINVAL), (2, [0], [4], 9, eb.EINVAL),
            (2, [0, 2], [2, 4], eb.F32, eb.ESHAPE),      # start not 16-byte aligned
            (2, [0, 4], [2, 4], eb.BF16, eb.ESHAPE),     # bf16 needs multiples of 8
            (2, [0, 4], [8, 4], eb.F32, eb.ESHAPE),      # overlap
            (2, [0], [-1], eb.F32, eb.ESHAPE)):
        with pytest.raises(eb.EagerError) as e:
            eb.Context(P, off, num, dt)
        assert e.value.status == status
    c = eb.Context(64, [0, 8, 16], [5, 0, 3], eb.BF16, eb.ORDER_FAST)
    assert c.eager_get_valid(2) == 0
    c.close()


def test_allreduce_validation_happens_before_any_launch():
    """Every case below must be refused on the host; fake device addresses are never
    dereferenced, so this runs without a GPU."""
    P = 4
    c = eb.Context(P, [0, 8], [8, 8])
    fake = [0x10000 + 0x1000 * p for p in range(P)]
    opt = (0x90000, 0xA0000, 0.1, 0.9)
    ok = eb.make_plan(eb.SOLO, P, 0, 0b0011)

    def expect(status, plan, **kw):
        args = dict(grads=fake, resid=fake, recv=None, opt=opt, b0=0, b1=2, stream=0)
        args.update(kw)
        with pytest.raises(eb.EagerError) as e:
            c.eager_partial_allreduce_solo(plan, args["grads"], args["resid"], args["recv"],
                                           args["opt"], args["b0"], args["b1"], args["stream"])
        assert e.value.status == status, str(e.value)

    expect(eb.ESTATE, eb.make_plan(eb.MAJORITY, P, 0, 0b0011))          # wrong entry point
    expect(eb.ESTATE, eb.make_plan(eb.QUORUM, P, 0, 0b0011))
    expect(eb.ESTATE, eb.make_plan(eb.SOLO, 5, 0, 0b0011))              # P mismatch
    expect(eb.ESTATE, eb.make_plan(eb.SOLO, P, 0, 0b10011))             # mask beyond P
    expect(eb.ESTATE, eb.make_plan(eb.SOLO, P, 0, 0b0011, initiator=3))  # initiator not active
    expect(eb.ESTATE, eb.Plan(eb.SOLO, P, 0, 0b0011, 0, 3))             # nap wrong
    expect(eb.ESTATE, eb.Plan(eb.SOLO, P, 0, 0, 0, 0))                  # nobody active
    expect(eb.EINVAL, ok, b0=1, b1=1)
    expect(eb.EINVAL, ok, b1=3)
    expect(eb.EINVAL, ok, opt=None)                                     # nothing to produce
    expect(eb.EINVAL, ok, grads=[0x10004] + fake[1:])                   # misaligned
    expect(eb.EINVAL, ok, resid=[0] + fake[1:])                         # NULL
    expect(eb.EINVAL, ok, opt=(0x90008, 0xA0000, 0.1, 0.9))
    expect(eb.EINVAL, ok, recv=0x90004)
    with pytest.raises(eb.EagerError) as e:
        c.eager_sgd_step(0, opt, stream=0)
    assert e.value.status == eb.EINVAL
    with pytest.raises(eb.EagerError):
        c.eager_set_launch("block", 100)
    with pytest.raises(eb.EagerError):
        c.eager_set_launch("nonsense", 1)
    with pytest.raises(eb.EagerError):
        c.eager_set_valid(0, 1 << P)
    c.eager_set_valid(1, 0b1010)
    assert c.eager_get_valid(1) == 0b1010 and c.eager_get_valid(0) == 0
    c.close()


def test_other_entry_points_validate_on_the_host():
    """Stash, rounds with absent processes, weight views, the layer-wise rule, statistics and
    launch keys: every bad call is refused before anything is launched (fake addresses)."""
    P = 4
    c = eb.Context(P, [0, 8], [8, 8])
    fake = [0x10000 + 0x1000 * p for p in range(P)]
    opt = (0x90000, 0xA0000, 0.1, 0.9)

    def refused(status, fn):
        with pytest.raises(eb.EagerError) as e:
            fn()
        assert e.value.status == status, str(e.value)

    refused(eb.EINVAL, lambda: c.eager_stash(P, 0x10000, 0x20000, stream=0))         # no such process
    refused(eb.EINVAL, lambda: c.eager_stash(-1, 0x10000, 0x20000, stream=0))
    refused(eb.EINVAL, lambda: c.eager_stash(0, 0, 0x20000, stream=0))               # NULL
    refused(eb.EINVAL, lambda: c.eager_stash(0, 0x10000, 0x20004, stream=0))         # misaligned
    refused(eb.EINVAL, lambda: c.eager_stash(0, 0x10000, 0x20000, 1, 1, stream=0))   # empty range
    plan = eb.make_plan(eb.SOLO, P, 0, 0b0011)
    refused(eb.ESTATE, lambda: c.eager_partial_allreduce_lagging(plan, 0b0001, fake, fake, opt=opt,
                                                                 stream=0))          # absent and active
    refused(eb.ESTATE, lambda: c.eager_partial_allreduce_lagging(plan, 0b10000, fake, fake, opt=opt,
                                                                 stream=0))          # beyond P
    refused(eb.EINVAL, lambda: c.eager_partial_allreduce_lagging(plan, 0b0100, [fake[0], fake[1], None, None],
                                                                 fake, opt=opt, stream=0))  # late, no gradient
    views = [0x100000, 0x200000, 0x300000]
    refused(eb.EINVAL, lambda: c.eager_sgd_step_views(0x90000, [], [], 0.1, 0.9, stream=0))
    refused(eb.EINVAL, lambda: c.eager_sgd_step_views(0x90000, [0x100000] * 65, [0x200000] * 65, 0.1, 0.9,
                                                      stream=0))
    refused(eb.EINVAL, lambda: c.eager_sgd_step_views(0x90000, [views[0], views[0]], views[1:], 0.1, 0.9,
                                                      stream=0))                     # one buffer twice
    refused(eb.EINVAL, lambda: c.eager_sgd_step_views(0x90004, views[:1], views[1:2], 0.1, 0.9, stream=0))
    refused(eb.EINVAL, lambda: c.eager_average_views([views[0], 0], stream=0))
    refused(eb.EINVAL, lambda: c.eager_average_views([views[0], views[0]], stream=0))
    refused(eb.ESTATE, lambda: c.eager_sgd_step_lars(0x90000, opt, 0.01, stream=0))  # nothing attached
    refused(eb.EINVAL, lambda: c.eager_sgd_step_lars(0x90000, opt, 0.0, stream=0))
    refused(eb.EINVAL, lambda: c.eager_sgd_step_lars(0x90000, opt, 0.01, -1.0, stream=0))
    refused(eb.EINVAL, lambda: c.eager_sgd_step_lars(0, opt, 0.01, stream=0))
    need = c.eager_stats_workspace_bytes()
    assert need >= 2 * 16 + 32 * (8 + 3 * 64)          # table, records, lane records at least
    refused(eb.EINVAL, lambda: c.eager_stats_attach(0x400000, 0x500000, need - 1, stream=0))
    refused(eb.EINVAL, lambda: c.eager_stats_attach(0x400008, 0x500000, need, stream=0))
    refused(eb.EINVAL, lambda: c.eager_stats_attach(0x400000, 0, need, stream=0))
    c.eager_stats_attach(None, None, stream=0)         # detaching what is not attached is fine
    for key, bad in (("round_stats", 2), ("split", 3), ("nt_state", 2), ("xcd_map", -1), ("chunk", 5),
                     ("blocks_per_cu", 33), ("carry_vec", 3), ("compact", 1)):
        refused(eb.EINVAL, lambda: c.eager_set_launch(key, bad))
    refused(eb.EINVAL, lambda: c.eager_set_update_rule(float("nan"), False))
    c.close()


def test_host_side_under_address_and_ub_sanitizers(tmp_path):
    """eager_api.cpp compiled without the kernels (the launchers and the one runtime call it
    uses are recorders in tests/c/api_host_sanitized.cpp) and driven on the CPU under
    AddressSanitizer and UndefinedBehaviorSanitizer: how a bucket range is cut into launches,
    the fused and the split form, absent processes, stash runs, views, statistics and the
    layer-wise rule, state after every call, error paths, a 2^31-element bucket."""
    import subprocess
    exe = tmp_path / "api_host_sanitized"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra", "-Werror",
                           "-D__HIP_PLATFORM_AMD__", "-isystem", "/opt/rocm/include",
                           os.path.join(ROOT, "tests", "c", "api_host_sanitized.cpp"),
                           os.path.join(ROOT, "paper_1908_04207_amd", "csrc", "eager_api.cpp"),
                           "-o", str(exe)])
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.stdout[-500:], r.stderr[-2000:])


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """Without the built HIP library the binding refuses to load: there is no CPU path."""
    monkeypatch.setattr(eb, "LIB_PATH", str(tmp_path / "libeager.so"))
    with pytest.raises(ImportError, match="no fallback"):
        eb._load()
    import inspect
    from paper_1908_04207_amd import async_sgd, hyperplane
    for mod in (eb, async_sgd, hyperplane):
        src = inspect.getsource(mod)
        assert "import oracle" not in src and "from oracle" not in src, mod.__name__
