"""Eager-SGD with a clock, a call counter and a weight view per process (Section 5, last
paragraph): processes that lag by more than one round, stale gradients that accumulate in the
send buffer, results missed in the receive buffer, diverging weights, periodic model
synchronisation.

The CPU tests pin the oracle (a closed-form timetable, a ledger of deliveries, an arithmetic walk)
against what the paper and arithmetic fix and against a tick-by-tick brute force; the GPU
tests run the library-driven loop (all arithmetic in the kernels) and the oracle's,
independently, on the same seeded compute times and gradients and compare every state bit
for bit.
"""
import numpy as np
import pytest
import torch

from harness import as_oracle_grad, bits
from oracle import async_oracle as ao
from oracle import eager_oracle as eo
from workloads import grads as wg
from workloads import times as wt


# ------------------------------------------------------------------ CPU: the oracle's loop
def _int_gradient(n):
    def g(p, k, w):
        return np.array([((p * 3 + k * 5 + i) % 7) - 3 for i in range(n)], dtype=np.float32)
    return g


def test_equal_compute_times_are_synchronous_sgd():
    """Everybody always arrives together: every round is a full allreduce, nobody is ever
    late, all weight views stay identical and equal ordinary synchronous momentum SGD."""
    P, n, T = 4, 9, 12
    rng = np.random.default_rng(0)
    w0 = rng.standard_normal(n).astype(np.float32)
    grads = {}

    def g(p, k, w):
        return grads.setdefault((p, k), rng.standard_normal(n).astype(np.float32))
    out = ao.simulate(P, n, w0, 0.05, 0.9, "solo", T, lambda p, k: 2.0, g)
    assert out["nap"] == [P] * T and out["late_calls"] == [0] * P and out["missed"] == [0] * P
    ref = eo.OracleState(P, [0], [n], n, w0, 0.05, 0.9)
    for t in range(T):
        ref.round((1 << P) - 1, [grads[(p, t)] for p in range(P)])
    for p in range(P):
        assert np.array_equal(bits(out["w"][p]), bits(ref.w))
        assert np.array_equal(bits(out["v"][p]), bits(ref.v))
    assert out["time_ms"] == 2.0 * T


@pytest.mark.parametrize("mode,kw", [("solo", {}), ("majority", {"seed": 5}), ("quorum", {"quorum": 2})])
def test_every_gradient_is_delivered_exactly_once(mode, kw):
    """Conservation under arbitrary lag (Section 6.1: a rejected update is added later,
    once): P * sum of all results + what is still in send buffers + the gradients of the
    processes waiting at the open collective = sum of all gradients computed.  Integer data,
    P a power of two: exact.  A process that never missed a result holds w = -sum of the
    results (lr = 1, mu = 0)."""
    P, n, T = 4, 6, 40
    g = _int_gradient(n)
    produced = np.zeros(n)
    made = []

    def counted(p, k, w):
        x = g(p, k, w)
        made.append((p, k))
        produced[:] += x
        return x

    def ms(p, k):                                   # heavy tail: some calls take many rounds
        return [1.0, 1.3, 0.7, 9.5, 2.2, 0.9, 14.0][(p * 5 + k * 3) % 7]
    out = ao.simulate(P, n, np.zeros(n, np.float32), 1.0, 0.0, mode, T, ms, counted,
                      keep_results=True, **kw)
    assert len(set(made)) == len(made)              # each (process, call) computed once
    assert max(out["late_calls"]) > 0 and max(out["missed"]) > 0
    assert len(out["results"]) == T
    delivered = P * sum(u.astype(np.float64) for u in out["results"])
    pending = sum((out["send"][p].astype(np.float64) for p in range(P) if out["has_stale"][p]),
                  np.zeros(n))
    held = sum((x.astype(np.float64) for x in out["held"].values()), np.zeros(n))
    assert np.array_equal(delivered + pending + held, produced)
    for p in range(P):
        if out["missed"][p] == 0 and out["late_calls"][p] == 0:
            assert np.array_equal(-out["w"][p].astype(np.float64) * P, delivered)
        # every process holds exactly the results it read, each once, in order (lr = 1, mu = 0)
        seen = out["applied"][p]
        assert seen == sorted(set(seen)) and len(seen) + out["missed"][p] <= T
        assert np.array_equal(-out["w"][p].astype(np.float64),
                              sum((out["results"][r].astype(np.float64) for r in seen), np.zeros(n)))


def test_missed_results_make_weights_differ_and_synchronisation_repairs_it():
    P, n, T = 4, 8, 30
    rng = np.random.default_rng(1)
    w0 = rng.standard_normal(n).astype(np.float32)

    def g(p, k, w):
        return (0.1 * w + 0.01 * ((p + k) % 3 - 1)).astype(np.float32)

    def ms(p, k):
        return 7.3 if (p == 3 and k % 2 == 0) else 1.0 + 0.1 * p
    free = ao.simulate(P, n, w0, 0.1, 0.9, "solo", T, ms, g)
    sync = ao.simulate(P, n, w0, 0.1, 0.9, "solo", T, ms, g, sync_every=T)
    assert free["missed"][3] > 0
    spread = lambda ws: max(float(np.max(np.abs(x - np.mean(ws, axis=0)))) for x in ws)  # noqa: E731
    assert spread(free["w"]) > 1e-4
    assert spread(sync["w"]) == 0.0 and spread(sync["v"]) == 0.0
    assert np.allclose(sync["w"][0], np.mean(free["w"], axis=0), atol=1e-6)


def _distinct_ms(p, k):
    """Compute times whose partial sums do not tie (a mixing hash of (p, k): no linear
    structure that sums could cancel), some of them long."""
    u = eo.initiator_hash(p * 1000003 + 17, k) / float(1 << 64)
    return 1.0 + u * (6.0 if (p + k) % 5 == 0 else 1.0)


def test_what_triggers_a_round():
    """Section 4: solo - the first process to reach the open collective triggers it alone
    (NAP = 1 when no two arrive together); majority - it waits for the designated initiator
    of the shared seed, who is therefore always among the active; quorum q - exactly q
    processes are active; quorum P - everybody, every round, nobody is ever late, and the
    round ends with the slowest process: T_r = T_{r-1} + max_p c_p(r)."""
    P, n, T = 8, 4, 60
    g = _int_gradient(n)
    w0 = np.zeros(n, np.float32)
    solo = ao.simulate(P, n, w0, 0.1, 0.0, "solo", T, _distinct_ms, g)
    assert solo["nap"] == [1] * T and all(bin(m).count("1") == 1 for m in solo["active"])
    assert solo["round_time_ms"] == sorted(solo["round_time_ms"])
    assert solo["round_time_ms"][0] == min(_distinct_ms(p, 0) for p in range(P))
    for seed in (1, 2, 3):
        maj = ao.simulate(P, n, w0, 0.1, 0.0, "majority", T, _distinct_ms, g, seed=seed)
        for r, mask in enumerate(maj["active"]):
            assert (mask >> (eo.initiator_hash(seed, r) % P)) & 1, (seed, r)
        assert 1 <= min(maj["nap"]) and max(maj["nap"]) <= P and len(set(maj["nap"])) > 1
        assert maj["time_ms"] >= solo["time_ms"]
    for q in (2, 5):
        out = ao.simulate(P, n, w0, 0.1, 0.0, "quorum", T, _distinct_ms, g, quorum=q)
        assert out["nap"] == [q] * T
    full = ao.simulate(P, n, w0, 0.1, 0.0, "quorum", T, _distinct_ms, g, quorum=P)
    assert full["nap"] == [P] * T and full["late_calls"] == [0] * P and full["missed"] == [0] * P
    t = 0.0
    for r in range(T):
        t += max(_distinct_ms(p, r) for p in range(P))
        assert abs(full["round_time_ms"][r] - t) < 1e-9
    assert full["time_ms"] > maj["time_ms"] > 0


def _tick_schedule(P, mode, rounds, ms, quorum=0, seed=0):
    """The rules of the model written out tick by tick, for compute times that are whole
    numbers (no arithmetic, no closed form): at every tick, the processes whose gradient is
    done make their call - those whose execution is already over are late (by rank) and start
    their next gradient at once, the others wait at the open execution - and then the
    execution runs if its trigger condition holds.  Returns per execution (tick, active set)
    and per gradient (process, call) the execution that delivers it (None: still in a send
    buffer)."""
    done_at = [ms(p, 0) for p in range(P)]           # tick at which the current gradient is done
    call = [0] * P
    waiting, pending = [], [[] for _ in range(P)]
    executed, log, delivered = 0, [], {}
    tick = 0
    while executed < rounds:
        tick += 1
        assert tick < 10_000
        for p in range(P):
            if p not in waiting and done_at[p] == tick and call[p] < executed:
                pending[p].append((p, call[p]))
                delivered[(p, call[p])] = None
                call[p] += 1
                done_at[p] = tick + ms(p, call[p])
        for p in range(P):
            if p not in waiting and done_at[p] == tick and call[p] == executed:
                waiting.append(p)
        if not waiting:
            continue
        if mode == "solo":
            go = True
        elif mode == "majority":
            go = eo.initiator_hash(seed, executed) % P in waiting
        else:
            go = len(waiting) >= quorum
        if not go:
            continue
        for p in range(P):
            for c in pending[p]:
                delivered[c] = executed
            pending[p] = []
        for p in waiting:
            delivered[(p, call[p])] = executed
            call[p] += 1
            done_at[p] = tick + ms(p, call[p])
        log.append((tick, sum(1 << p for p in waiting)))
        waiting = []
        executed += 1
    return log, delivered


def test_timetable_and_ledger_against_the_rules_tick_by_tick():
    """Brute force over EVERY table of whole-number compute times (1..3 ticks, so ties of every
    kind occur; two values where three would take minutes) for up to 3 processes and 4 calls, in
    every mode: the oracle's closed-form timetable and its ledger of deliveries equal a
    tick-by-tick walk through the rules."""
    import itertools
    checked = 0
    for P, rounds, ticks in ((1, 3, (1, 2, 3)), (2, 4, (1, 2, 3)), (3, 2, (1, 2, 3)), (3, 3, (1, 2)),
                             (3, 4, (1, 3))):
        cells = P * (rounds + 1)
        for table in itertools.product(ticks, repeat=cells):
            ms = lambda p, k, t=table, r=rounds: t[p * (r + 1) + k]      # noqa: E731
            modes = [("solo", {}), ("majority", {"seed": 1}), ("majority", {"seed": 6})]
            modes += [("quorum", {"quorum": q}) for q in range(1, P + 1)]
            for mode, kw in modes:
                arrive, trigger, active = ao.timetable(P, mode, rounds, ms, **kw)
                want_log, want_delivery = _tick_schedule(P, mode, rounds, ms, **kw)
                got_log = [(trigger[k], sum(1 << p for p in range(P) if active[p][k]))
                           for k in range(rounds)]
                assert got_log == [(float(t), m) for t, m in want_log], (table, mode, kw)
                assert ao.ledger(P, rounds, arrive, trigger, active) == want_delivery, (table, mode, kw)
                checked += 1
    assert checked > 400_000


@pytest.mark.parametrize("mode,kw", [("solo", {}), ("majority", {"seed": 3}), ("quorum", {"quorum": 2})])
def test_every_result_holds_exactly_the_gradients_the_ledger_names(mode, kw):
    """Gradient (p, k) is a distinct power of two in every element, P = 4, lr = 1, mu = 0: all
    sums are exact, so each result, times P, spells out which gradients it delivered, and each
    weight view which results its process read.  Both must be what the ledger and the rules
    say - for the arithmetic walk of the oracle this is an end-to-end check that does not rest
    on the oracle's round routine."""
    P, n, T = 4, 3, 5

    def ms(p, k):
        return [2.0, 3.0, 1.0, 7.0, 2.0, 11.0, 1.0][(p * 3 + k * 2) % 7]
    out = ao.simulate(P, n, np.zeros(n, np.float32), 1.0, 0.0, mode, T, ms,
                      lambda p, k, w: np.full(n, 2.0 ** (p * (T + 1) + k), np.float32),
                      keep_results=True, **kw)
    assert any(v is not None and v != c[1] for c, v in out["ledger"].items())     # somebody was late
    for r, u in enumerate(out["results"]):
        code = int(u[0] * P)
        assert float(code) == float(u[0]) * P and np.all(u == u[0])
        named = {c for c, v in out["ledger"].items() if v == r}
        assert code == sum(1 << (p * (T + 1) + k) for p, k in named), (r, named)
    for p in range(P):
        code = int(out["send"][p][0]) if out["has_stale"][p] else 0
        assert code == sum(1 << (q * (T + 1) + k) for (q, k), v in out["ledger"].items()
                           if v is None and q == p)
        read = sum(float(out["results"][r][0]) for r in out["applied"][p])
        assert float(-out["w"][p][0]) == read


ASYNC_MUTATIONS = {
    "a late gradient overwrites a pending one":
        ("eo.stash_f32(gradient(p, k, w[p]), send[p], bool(in_send[p]))",
         "eo.stash_f32(gradient(p, k, w[p]), send[p], False)"),
    "the latest result is applied again":
        ("if last_applied[p] < executed - 1:", "if executed > 0:"),
    "majority does not wait for its initiator":
        ("fired = at[eo.initiator_hash(seed, k) % P]", "fired = min(at)"),
    "quorum waits for one process too many":
        ("fired = sorted(at)[quorum - 1]", "fired = sorted(at)[min(quorum, P - 1)]"),
    "processes that are still computing are treated as late":
        ("absent=everyone & ~mask)", "absent=0)"),
    "send buffers are not emptied by a round":
        ("            in_send = [[] for _ in range(P)]\n            if keep_results:", "            if keep_results:"),
    "an active process does not read the result":
        ("            for q in sorted(fresh):\n                read_receive_buffer(q, k)\n", ""),
    "a tie with the initiator counts as late":
        ("on_time = at[p] <= fired", "on_time = at[p] < fired or at[p] == min(at)"),
    "an active process does not wait for the execution to be over":
        ("arrive[p].append((fired if on_time else at[p]) +", "arrive[p].append(at[p] +"),
    "a gradient that comes with the trigger is delivered one execution later":
        ("if trigger[j] >= arrive[p][k]]", "if trigger[j] > arrive[p][k]]"),
}


@pytest.mark.parametrize("name", list(ASYNC_MUTATIONS))
def test_a_planted_mistake_in_the_loop_fails_a_pin(name, monkeypatch):
    """The pins above bite: each mistake planted in a copy of the oracle's module makes one of
    them fail (on the CPU; the GPU path is not involved)."""
    import inspect
    old, new = ASYNC_MUTATIONS[name]
    src = inspect.getsource(ao)
    assert src.count(old) == 1, f"mutation site not unique: {old!r}"
    scope = {"__name__": ao.__name__, "__package__": ao.__package__}
    exec(compile(src.replace(old, new), "<mutant>", "exec"), scope)
    for fn in ("timetable", "ledger", "simulate"):
        monkeypatch.setattr(ao, fn, scope[fn])
    caught = False
    for pin in (test_equal_compute_times_are_synchronous_sgd, test_what_triggers_a_round,
                lambda: test_every_gradient_is_delivered_exactly_once("solo", {}),
                lambda: test_every_gradient_is_delivered_exactly_once("majority", {"seed": 5}),
                lambda: test_every_gradient_is_delivered_exactly_once("quorum", {"quorum": 2}),
                lambda: test_every_result_holds_exactly_the_gradients_the_ledger_names("solo", {}),
                lambda: test_every_result_holds_exactly_the_gradients_the_ledger_names("quorum", {"quorum": 2}),
                _small_tick_check):
        try:
            pin()
        except (AssertionError, ValueError, IndexError, KeyError):
            caught = True
            break
    assert caught, f"no pin noticed: {name}"


def _small_tick_check():
    """A slice of the tick-by-tick brute force (two processes, three calls), for the mutants."""
    import itertools
    for table in itertools.product((1, 2, 3), repeat=8):
        ms = lambda p, k, t=table: t[p * 4 + k]                          # noqa: E731
        for mode, kw in (("solo", {}), ("majority", {"seed": 1}), ("quorum", {"quorum": 2})):
            arrive, trigger, active = ao.timetable(2, mode, 3, ms, **kw)
            want_log, want_delivery = _tick_schedule(2, mode, 3, ms, **kw)
            assert [(trigger[k], sum(1 << p for p in range(2) if active[p][k])) for k in range(3)] == \
                [(float(t), m) for t, m in want_log]
            assert ao.ledger(2, 3, arrive, trigger, active) == want_delivery


# ------------------------------------------------------------------ GPU: library loop == oracle loop
@pytest.fixture(scope="module")
def asgd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1908_04207_amd import async_sgd
    return async_sgd


@pytest.mark.gpu
@pytest.mark.parametrize("mode,kw,dtype,sync", [
    ("solo", {}, "f32", 0), ("solo", {}, "bf16", 9), ("majority", {"seed": 77}, "f32", 7),
    ("quorum", {"quorum": 5}, "f32", 0), ("quorum", {"quorum": 3}, "bf16", 11)])
def test_library_loop_is_bit_identical_to_the_oracle_loop(asgd, mode, kw, dtype, sync):
    from paper_1908_04207_amd import binding as eb
    P, rounds, seed = 8, 60, 4242
    align = 8 if dtype == "bf16" else 4
    numel = [301, 7, 0, 2050, 64, 1283]
    off, cur = [], 0
    for m in numel:
        off.append(cur)
        cur = (cur + m + align - 1) // align * align
    arena = cur
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    w0 = wg.fill(torch.empty(arena), seed, 0, wg.PARAM_RANK, 0.02)

    def ms(p, k):                                   # Pareto(1.5): long tail, lags of many rounds
        return wt.compute_times("pareto_1.5", P, seed, k)[p]

    def grad_cpu(p, k):
        return wg.fill(torch.empty(arena, dtype=tdt), seed, k, p, 1e-3)

    sim = asgd.AsyncEagerSGD(P, off, numel, arena, w0, 0.1, 0.9, mode, kw.get("quorum", 0),
                             kw.get("seed", 0), sync, eb.BF16 if dtype == "bf16" else eb.F32)
    res = sim.run(rounds, ms, lambda p, k, w: grad_cpu(p, k).cuda())
    torch.cuda.synchronize()

    # the oracle works on the concatenation of the buckets (padding carries no data)
    inside = np.concatenate([np.arange(o, o + m) for o, m in zip(off, numel)])
    out = ao.simulate(P, len(inside), w0.numpy()[inside], 0.1, 0.9, mode, rounds, ms,
                      lambda p, k, w: np.ascontiguousarray(as_oracle_grad(grad_cpu(p, k))[inside]),
                      sync_every=sync, **kw)
    assert res.nap == out["nap"] and res.late_calls == out["late_calls"]
    assert res.missed == out["missed"] and res.time_ms == out["time_ms"]
    assert max(res.late_calls) > 0 and max(res.missed) > 0      # the run did lag
    assert [sim.k[p] for p in range(P)] == out["calls"]
    valid = sim.ctx.eager_get_valid(0)
    assert all(sim.ctx.eager_get_valid(b) == valid for b in range(len(numel)))
    assert valid == sum(1 << p for p in range(P) if out["has_stale"][p])
    for p in range(P):
        assert np.array_equal(bits(sim.w[p].cpu().numpy()[inside]), bits(out["w"][p])), (p, "w")
        assert np.array_equal(bits(sim.v[p].cpu().numpy()[inside]), bits(out["v"][p])), (p, "v")
        if (valid >> p) & 1:
            assert np.array_equal(bits(sim.R[p].cpu().numpy()[inside]), bits(out["send"][p])), (p, "R")
    if sync:
        assert len(res.divergence) == rounds and min(res.divergence) == 0.0
    sim.close()
