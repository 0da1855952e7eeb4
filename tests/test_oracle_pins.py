"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pin is chosen so that a plausible
mistake in the oracle (a dropped stale term, dividing by the number of contributors,
a send buffer that is not emptied or not overwritten, a sign or an index slip in the
update rule) makes at least one of them fail.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import eager_oracle as eo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _empty_R(P, n):
    return [np.zeros(n, dtype=np.float32) for _ in range(P)]


# ------------------------------------------------------------------ brute-force ledger
def _ledger(P, T, masks, G, w0, lr, mu):
    """Closed form of the carry, exact rationals: gradient (t, p) is delivered in round
    t when p is on time, otherwise in round t + 1 (Section 6.1: a rejected update is
    added in the next round).  Independent of the oracle's recurrence: no send buffers,
    only delivery times."""
    n = len(w0)
    w = [Fraction(int(x)) for x in w0]
    v = [Fraction(0)] * n
    us = []
    for t in range(T):
        tot = [Fraction(0)] * n
        for tt in range(T):
            for p in range(P):
                delivered = tt if (masks[tt] >> p) & 1 else tt + 1
                if delivered == t:
                    tot = [a + int(b) for a, b in zip(tot, G[tt][p])]
        u = [x / P for x in tot]
        v = [mu * a + b for a, b in zip(v, u)]
        w = [a - lr * b for a, b in zip(w, v)]
        us.append(u)
    pending = {p: G[T - 1][p] for p in range(P) if not (masks[T - 1] >> p) & 1}
    return us, w, v, pending


@pytest.mark.parametrize("P,T", [(1, 3), (2, 3), (4, 3), (3, 2)])
def test_brute_force_every_mask_sequence(P, T):
    """Every sequence of participation masks (empty masks included) on a tiny problem.
    Integer gradients, dyadic lr and mu and power-of-two P make fp32 exact, so the
    comparison with the rational ledger is bitwise; P = 3 is compared to 1e-6."""
    n = 3
    rng = np.random.default_rng(100 + P)
    G = rng.integers(-8, 9, size=(T, P, n)).astype(np.float32)
    w0 = rng.integers(-4, 5, size=n).astype(np.float32)
    lr, mu = Fraction(1, 4), Fraction(1, 2)
    exact = P in (1, 2, 4)
    for masks in itertools.product(range(1 << P), repeat=T):
        R = _empty_R(P, n)
        valid = 0
        w, v = w0.copy(), np.zeros(n, dtype=np.float32)
        us = []
        for t in range(T):
            recv = np.empty(n, dtype=np.float32)
            valid = eo.round_f32([G[t, p].copy() for p in range(P)], R, valid, masks[t],
                                 w, v, float(lr), float(mu), recv)
            us.append(recv)
        lus, lw, lv, pending = _ledger(P, T, masks, G, w0, lr, mu)
        got = np.concatenate(us + [w, v]).astype(np.float64)
        want = np.array([float(x) for u in lus for x in u] + [float(x) for x in lw]
                        + [float(x) for x in lv])
        if exact:
            assert np.array_equal(got, want), (masks, got, want)
        else:
            assert np.allclose(got, want, rtol=1e-6, atol=1e-6), masks
        assert valid == sum(1 << p for p in pending)
        for p, g in pending.items():
            assert np.array_equal(R[p], g)


# ------------------------------------------------------------------ worked example
def _parse_cases(path):
    cases, cur = {}, None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = cases.setdefault(tok[1], [])
        elif tok[0] == "round":
            cur.append({"t": int(tok[1]), "active": [int(x) for x in tok[3:]], "expect": {}})
        elif tok[0] == "expect":
            name, expr = line[len("expect"):].split("=", 1)
            cur[-1]["expect"][name.strip()] = expr.strip()
    return cases


@pytest.mark.parametrize("case", ["catches_up", "late_again"])
def test_fig7_walkthrough(case):
    """Section 5, Fig. 7: the two-process example, both branches, on random vectors."""
    rounds = _parse_cases(os.path.join(GOLDEN, "fig7_walkthrough.txt"))[case]
    rng = np.random.default_rng(7)
    n = 5
    G = {f"G{p}_{k}": rng.integers(-50, 50, n).astype(np.float32)
         for p in range(2) for k in range(2)}
    R, valid = _empty_R(2, n), 0
    R64 = [None, None]
    for r in rounds:
        mask = sum(1 << p for p in r["active"])
        recv = np.empty(n, dtype=np.float32)
        g = [G[f"G{p}_{r['t']}"] for p in range(2)]
        valid = eo.round_f32(g, R, valid, mask, None, None, 0.0, 0.0, recv)
        u64, R64, _, _ = eo.round_f64(g, R64, mask, np.zeros(n), np.zeros(n), 0.0, 0.0)
        for name, expr in r["expect"].items():
            if name == "U":
                want = eval(expr, {}, dict(G))
                assert np.array_equal(recv, want.astype(np.float32))
                assert np.array_equal(u64, want)
            else:
                p = int(name[len("send"):])
                if expr == "null":
                    assert not (valid >> p) & 1 and R64[p] is None
                else:
                    assert (valid >> p) & 1
                    assert np.array_equal(R[p], G[expr]) and np.array_equal(R64[p], G[expr])


# ------------------------------------------------------------------ full participation
def test_full_participation_is_allreduce_mean_with_torch_sgd():
    """Algorithm 2 with everybody on time is Algorithm 1: the mean of the gradients fed
    to the update rule.  Checked against torch's own SGD with momentum (a library
    routine) over several rounds; the send buffers stay empty throughout."""
    P, n, T, lr, mu = 8, 1000, 6, 0.1, 0.9
    rng = np.random.default_rng(11)
    w0 = rng.normal(0, 0.02, n).astype(np.float32)
    w, v = w0.copy(), np.zeros(n, dtype=np.float32)
    R, valid = _empty_R(P, n), 0
    for r in R:
        r[:] = np.nan          # must never be read
    tw = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.SGD([tw], lr=lr, momentum=mu)
    for t in range(T):
        G = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(P)]
        valid = eo.round_f32(G, R, valid, (1 << P) - 1, w, v, lr, mu)
        assert valid == 0
        tw.grad = torch.from_numpy(np.stack(G)).to(torch.float64).mean(0).to(torch.float32)
        opt.step()
        assert np.allclose(w, tw.detach().numpy(), rtol=0, atol=2e-7 * np.abs(w).max())
    assert not np.array_equal(w, w0)


# ------------------------------------------------------------------ conservation
@pytest.mark.parametrize("P", [2, 4, 8])
def test_conservation_every_gradient_applied_exactly_once(P):
    """P * sum_t u(t) + (what is still pending) = sum of all gradients; after a final
    round in which everybody is on time with a zero gradient nothing is pending.
    Integer data and power-of-two P make this exact in fp32."""
    n, T = 64, 12
    rng = np.random.default_rng(P)
    R, valid = _empty_R(P, n), 0
    total_G = np.zeros(n)
    total_u = np.zeros(n)
    for t in range(T):
        G = [rng.integers(-20, 21, n).astype(np.float32) for _ in range(P)]
        mask = int(rng.integers(0, 1 << P))
        recv = np.empty(n, dtype=np.float32)
        valid = eo.round_f32(G, R, valid, mask, None, None, 0, 0, recv)
        total_G += np.sum(G, axis=0)
        total_u += recv.astype(np.float64)
        pending = sum(R[p].astype(np.float64) for p in range(P) if (valid >> p) & 1)
        assert np.array_equal(P * total_u + pending, total_G)
    zeros = [np.zeros(n, dtype=np.float32) for _ in range(P)]
    recv = np.empty(n, dtype=np.float32)
    valid = eo.round_f32(zeros, R, valid, (1 << P) - 1, None, None, 0, 0, recv)
    total_u += recv
    assert valid == 0 and np.array_equal(P * total_u, total_G)


# ------------------------------------------------------------------ Lemma 2
def test_lemma2_distance_to_clean_iterate():
    """Section 6.2: Lambda follows the clean iteration with every gradient of every
    round.  With plain SGD (mu = 0) the eager iterate differs from it by exactly alpha/P
    times the gradients not yet delivered, i.e. the valid send buffers; each gradient
    waits at most one round (staleness bound tau = 1 in this per-round model).  The
    norm is checked against the triangle-inequality form of the lemma's bound."""
    P, n, T, lr = 4, 32, 20, 0.25
    rng = np.random.default_rng(3)
    w0 = rng.integers(-3, 4, n).astype(np.float32)
    w, v = w0.copy(), np.zeros(n, dtype=np.float32)
    lam = w0.astype(np.float64)
    R, valid = _empty_R(P, n), 0
    for t in range(T):
        G = [rng.integers(-9, 10, n).astype(np.float32) for _ in range(P)]
        mask = int(rng.integers(1, 1 << P))
        valid = eo.round_f32(G, R, valid, mask, w, v, lr, 0.0)
        lam = lam - lr / P * np.sum(G, axis=0, dtype=np.float64)
        pend = [R[p].astype(np.float64) for p in range(P) if (valid >> p) & 1]
        diff = w.astype(np.float64) - lam
        assert np.array_equal(diff, lr / P * sum(pend, np.zeros(n)))
        M2 = max(float(np.dot(g, g)) for g in G)
        late = P - bin(mask).count("1")
        assert float(np.dot(diff, diff)) <= lr ** 2 * late ** 2 * M2 / P ** 2 + 1e-12


# ------------------------------------------------------------------ lag of more than one round
def test_late_is_absent_plus_stash():
    """A process that is late in a round is one that stores nothing during the round and
    puts its gradient into the (now empty) send buffer afterwards: the two descriptions of
    Section 5 give the same bits.  Links the new operations to the pinned round."""
    rng = np.random.default_rng(11)
    for P, bf16 in ((2, False), (5, False), (8, True)):
        n = 37
        G = [rng.standard_normal(n).astype(np.float32) for _ in range(P)]
        if bf16:
            G = [(g.view(np.uint32) >> 16).astype(np.uint16) for g in G]
        for trial in range(20):
            mask = int(rng.integers(1, 1 << P))
            valid = int(rng.integers(0, 1 << P))
            late = ~mask & ((1 << P) - 1)
            R0 = [rng.standard_normal(n).astype(np.float32) for _ in range(P)]
            w0, v0 = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
            Ra, wa, va = [r.copy() for r in R0], w0.copy(), v0.copy()
            Rb, wb, vb = [r.copy() for r in R0], w0.copy(), v0.copy()
            val_a = eo.round_f32(G, Ra, valid, mask, wa, va, 0.1, 0.9)
            val_b = eo.round_f32(G, Rb, valid, mask, wb, vb, 0.1, 0.9, absent=late)
            assert val_b == 0 and val_a == late
            for p in range(P):
                if (late >> p) & 1:
                    eo.stash_f32(G[p], Rb[p], False)
                    assert np.array_equal(Ra[p].view(np.uint32), Rb[p].view(np.uint32))
            assert np.array_equal(wa.view(np.uint32), wb.view(np.uint32))
            assert np.array_equal(va.view(np.uint32), vb.view(np.uint32))


@pytest.mark.parametrize("P,T", [(2, 3), (4, 2), (3, 2)])
def test_brute_force_with_absent_processes_and_stashes(P, T):
    """Every sequence of per-process states (on time / late / absent) over T rounds, with
    extra gradients stashed between rounds (a send buffer then holds a sum): the delivered
    averages must be exactly what a ledger of delivery times says - a gradient contributed
    on time is delivered in its round, one finished late or stashed afterwards in the next
    round - and after a final round with everybody on time every send buffer is empty and
    every produced gradient has been delivered exactly once (Section 6.1)."""
    import itertools
    from fractions import Fraction
    n = 3
    states = list(itertools.product((0, 1, 2), repeat=P))          # 0 on time, 1 late, 2 absent
    states = [s for s in states if 0 in s]                          # somebody triggers the round
    exact = P in (1, 2, 4)

    def grad(t, p, k):                                              # small integers: exact in fp32
        return np.array([((t * 5 + p * 3 + k * 7 + i) % 7) - 3 for i in range(n)], dtype=np.float32)

    for seq in itertools.product(states, repeat=T):
        R, valid = _empty_R(P, n), 0
        pending = [np.zeros(n) for _ in range(P)]                   # ledger of the send buffers
        produced = np.zeros(n)
        delivered = np.zeros(n)
        for t in range(T + 1):
            st = seq[t] if t < T else (0,) * P                      # last round: everybody on time
            if t == T:
                # the flush (nobody active, everybody absent) on a copy of the state: exactly what
                # the ledger holds as pending, and every send buffer empty afterwards
                Rf = [r.copy() for r in R]
                flushed = np.empty(n, dtype=np.float32)
                none = [np.full(n, np.nan, dtype=np.float32) for _ in range(P)]     # never read
                assert eo.round_f32(none, Rf, valid, 0, None, None, 0, 0, flushed,
                                    absent=(1 << P) - 1) == 0
                owed = sum(pending, np.zeros(n))
                if exact:
                    assert np.array_equal(flushed.astype(np.float64) * P, owed), (seq, "flush")
                else:
                    assert np.allclose(flushed.astype(np.float64) * P, owed, rtol=0, atol=1e-5)
            mask = sum(1 << p for p in range(P) if st[p] == 0)
            absent = sum(1 << p for p in range(P) if st[p] == 2)
            G = [grad(t, p, 0) if t < T else np.zeros(n, dtype=np.float32) for p in range(P)]
            recv = np.empty(n, dtype=np.float32)
            valid = eo.round_f32(G, R, valid, mask, None, None, 0, 0, recv, absent=absent)
            want = np.zeros(n)
            for p in range(P):
                want += pending[p]
                pending[p] = np.zeros(n)
                if st[p] == 0:
                    want += G[p]
                    produced += G[p]
                elif st[p] == 1:
                    pending[p] = G[p].astype(np.float64)
                    produced += G[p]
            if exact:
                assert np.array_equal(recv.astype(np.float64) * P, want), (seq, t)
            else:
                assert np.allclose(recv.astype(np.float64) * P, want, rtol=0, atol=1e-5), (seq, t)
            delivered += want
            if t < T:                                               # extra gradients between rounds
                for p in range(P):
                    for k in range(1, 1 + (t + p) % 3 if st[p] != 0 else 1):
                        g = grad(t, p, k)
                        eo.stash_f32(g, R[p], bool((valid >> p) & 1))
                        valid |= 1 << p
                        pending[p] = pending[p] + g
                        produced += g
        assert valid == 0
        assert np.array_equal(delivered, produced)


# ------------------------------------------------------------------ update rule
def test_momentum_closed_form_and_plain_sgd():
    """Constant averaged gradient g: v_t = g (1 - mu^t) / (1 - mu) and w_t = w_0 - lr *
    sum of v; mu = 0 reduces to plain SGD."""
    n, T, lr, mu, g = 4, 25, 0.1, 0.9, 0.37
    w, v = np.ones(n, dtype=np.float32), np.zeros(n, dtype=np.float32)
    G = [np.full(n, g, dtype=np.float32)]
    R, valid = _empty_R(1, n), 0
    acc = 0.0
    for t in range(1, T + 1):
        valid = eo.round_f32(G, R, valid, 1, w, v, lr, mu)
        vt = np.float32(g) * (1 - mu ** t) / (1 - mu)
        acc += vt
        assert np.allclose(v, vt, rtol=1e-6)
        assert np.allclose(w, 1.0 - lr * acc, rtol=0, atol=2e-6)
    w, v = np.ones(n, dtype=np.float32), np.zeros(n, dtype=np.float32)
    for t in range(1, 4):
        eo.round_f32(G, R, 0, 1, w, v, 0.5, 0.0)
        assert np.allclose(w, 1.0 - 0.5 * g * t, rtol=1e-6)
    u = np.full(n, g, dtype=np.float32)
    w2, v2 = np.ones(n, dtype=np.float32), np.zeros(n, dtype=np.float32)
    w3, v3 = w2.copy(), v2.copy()
    for t in range(5):
        eo.sgd_f32(u, w2, v2, lr, mu)
        eo.round_f32(G, R, 0, 1, w3, v3, lr, mu)
    assert np.array_equal(w2, w3) and np.array_equal(v2, v3)


@pytest.mark.parametrize("wd,nesterov", [(0.0, True), (0.05, False), (0.01, True)])
def test_update_rule_variants_against_torch_sgd(wd, nesterov):
    """Weight decay and Nesterov momentum (variants of the generic U of Algorithm 2 line 7)
    follow torch.optim.SGD (library routine) over several steps with everybody on time;
    the variants change nothing of the carry (send buffers stay empty)."""
    import torch
    P, n, T, lr, mu = 4, 257, 6, 0.05, 0.9
    rng = np.random.default_rng(5)
    w0 = rng.standard_normal(n).astype(np.float32)
    w, v = w0.copy(), np.zeros(n, dtype=np.float32)
    tw = torch.tensor(w0.copy(), requires_grad=True)
    opt = torch.optim.SGD([tw], lr=lr, momentum=mu, weight_decay=wd, nesterov=nesterov)
    R, valid = _empty_R(P, n), 0
    for t in range(T):
        G = [rng.standard_normal(n).astype(np.float32) for _ in range(P)]
        valid = eo.round_f32(G, R, valid, (1 << P) - 1, w, v, lr, mu, wd=wd, nesterov=nesterov)
        assert valid == 0
        tw.grad = torch.tensor(np.mean(np.stack(G).astype(np.float64), axis=0).astype(np.float32))
        opt.step()
        assert np.allclose(w, tw.detach().numpy(), rtol=0, atol=2e-6), t
    # closed form, one step from v = 0:  g = u + wd w ;  v = g ;  w' = w - lr (1 + mu) g  (Nesterov)
    w1, v1 = w0.copy(), np.zeros(n, dtype=np.float32)
    u = rng.standard_normal(n).astype(np.float32)
    eo.sgd_f32(u, w1, v1, lr, mu, wd=wd, nesterov=nesterov)
    g = u.astype(np.float64) + wd * w0
    want = w0 - lr * ((1 + mu) * g if nesterov else g)
    assert np.allclose(v1, g, rtol=1e-6, atol=1e-7) and np.allclose(w1, want, rtol=1e-6, atol=1e-6)
    # the variants switched off are the plain rule, bit for bit
    w2, v2, w3, v3 = w0.copy(), v1.copy(), w0.copy(), v1.copy()
    eo.sgd_f32(u, w2, v2, lr, mu)
    eo.sgd_f32(u, w3, v3, lr, mu, wd=0.0, nesterov=False)
    assert np.array_equal(w2, w3) and np.array_equal(v2, v3)


def test_layerwise_rate_closed_forms():
    """The layer-wise rate (You, Gitman, Ginsburg 2017) on vectors whose norms are known:
    w = c everywhere, u = d everywhere, so ||w|| / ||u|| = |c| / |d| whatever n.  Power-of-two
    values keep every fp32 operation exact."""
    n = 64
    for c, d, wd, trust in [(0.5, 0.25, 0.0, 0.5), (2.0, -0.5, 0.25, 1.0), (-1.0, 4.0, 0.0, 0.125)]:
        u = np.full(n, d, dtype=np.float32)
        w, v = np.full(n, c, dtype=np.float32), np.zeros(n, dtype=np.float32)
        (rate,) = eo.sgd_lars_f32(u, w, v, [0], [n], lr=0.5, mu=0.5, trust=trust, wd=wd)
        want = trust * abs(c) / (abs(d) + wd * abs(c))
        assert rate == np.float32(want)
        g = want * (d + wd * c)
        assert np.all(v == np.float32(g)) and np.all(w == np.float32(c - 0.5 * g))
    # a layer at zero (fresh biases) or a zero update: rate 1, the plain rule bit for bit
    rng = np.random.default_rng(3)
    for u, w0 in [(rng.standard_normal(n).astype(np.float32), np.zeros(n, np.float32)),
                  (np.zeros(n, np.float32), rng.standard_normal(n).astype(np.float32))]:
        w, v, w1, v1 = w0.copy(), np.ones(n, np.float32), w0.copy(), np.ones(n, np.float32)
        assert eo.sgd_lars_f32(u, w, v, [0], [n], 0.1, 0.9, trust=0.001, wd=0.01) == [1.0]
        eo.sgd_f32(u, w1, v1, 0.1, 0.9, wd=0.01)
        assert np.array_equal(w, w1) and np.array_equal(v, v1)


def test_layerwise_rate_properties_and_torch():
    """What defines the rule: (1) without weight decay the step does not depend on the scale
    of the gradient - u and 1024 u give the same new weights (powers of two: exactly);
    (2) the scaled gradient has norm trust * ||w||; (3) every bucket gets its own rate and
    the padding between buckets is left alone; (4) over several steps it equals torch's SGD
    (library routine, momentum and Nesterov) fed with gradients scaled by rates computed
    with torch.linalg.norm in fp64."""
    import torch
    rng = np.random.default_rng(11)
    offset, numel = [0, 40, 48, 120], [37, 5, 70, 9]
    arena = 132
    u = (1e-3 * rng.standard_normal(arena)).astype(np.float32)
    w0 = (0.02 * rng.standard_normal(arena)).astype(np.float32)
    v0 = (1e-3 * rng.standard_normal(arena)).astype(np.float32)
    wa, va, wb, vb = w0.copy(), v0.copy(), w0.copy(), v0.copy()
    ra = eo.sgd_lars_f32(u, wa, va, offset, numel, 0.1, 0.9, trust=0.01)
    rb = eo.sgd_lars_f32(u * np.float32(1024), wb, vb, offset, numel, 0.1, 0.9, trust=0.01)
    assert np.array_equal(wa, wb) and np.array_equal(va, vb)
    assert [np.float32(x / 1024) for x in ra] == [np.float32(x) for x in rb]
    assert len(set(ra)) == len(ra)
    inside = np.zeros(arena, bool)
    for (lo, n), rate in zip(zip(offset, numel), ra):
        inside[lo:lo + n] = True
        scaled = rate * u[lo:lo + n].astype(np.float64)
        assert np.isclose(np.linalg.norm(scaled), 0.01 * np.linalg.norm(w0[lo:lo + n].astype(np.float64)),
                          rtol=1e-6)
        assert np.allclose(va[lo:lo + n], 0.9 * v0[lo:lo + n].astype(np.float64) + scaled, rtol=1e-5, atol=1e-9)
    assert np.array_equal(wa[~inside], w0[~inside]) and np.array_equal(va[~inside], v0[~inside])

    for wd, nesterov in [(0.0, False), (5e-4, True)]:
        params = [torch.tensor(w0[lo:lo + n].copy(), requires_grad=True) for lo, n in zip(offset, numel)]
        opt = torch.optim.SGD(params, lr=0.1, momentum=0.9, nesterov=nesterov)
        w, v = w0.copy(), np.zeros(arena, np.float32)
        for t in range(5):
            ut = (1e-3 * rng.standard_normal(arena)).astype(np.float32)
            eo.sgd_lars_f32(ut, w, v, offset, numel, 0.1, 0.9, trust=0.02, eps=1e-9, wd=wd,
                            nesterov=nesterov)
            for prm, lo, n in zip(params, offset, numel):
                g = torch.tensor(ut[lo:lo + n]).double()
                pw = prm.detach().double()
                nw, ng = torch.linalg.norm(pw), torch.linalg.norm(g)
                rate = 0.02 * nw / (ng + wd * nw + 1e-9)
                prm.grad = (rate * (g + wd * pw)).float()
            opt.step()
            for prm, lo, n in zip(params, offset, numel):
                assert np.allclose(w[lo:lo + n], prm.detach().numpy(), rtol=1e-5, atol=1e-8), (wd, t)


def test_divides_by_P_not_by_contributors():
    """Algorithm 2 line 6 scales by 1/P whatever the number of active processes.  With
    fresh = 1 and null = 0 the delivered value times P is the number of active
    processes; the artifact appendix expects solo < majority < full for this average."""
    P, n = 32, 8
    ones = [np.ones(n, dtype=np.float32) for _ in range(P)]
    arrival = [float(p + 1) for p in range(P)]
    means = {}
    for name, mode, kw in (("solo", eo.SOLO, {}), ("majority", eo.MAJORITY, {}),
                           ("full", eo.QUORUM, {"quorum": P})):
        tot = 0.0
        for it in range(64):
            plan = eo.plan_participation(mode, P, arrival, 42, it, **kw)
            recv = np.empty(n, dtype=np.float32)
            eo.round_f32(ones, _empty_R(P, n), 0, plan.mask, None, None, 0, 0, recv)
            assert np.array_equal(recv * P, np.full(n, plan.nap, dtype=np.float32))
            tot += float(recv[0])
        means[name] = tot / 64
    assert means["solo"] < means["majority"] < means["full"] == 1.0


# ------------------------------------------------------------------ fp32 C vs fp64 numpy
@pytest.mark.parametrize("P,bf16", [(3, False), (8, False), (16, True), (64, False)])
def test_c_recurrence_matches_independent_fp64(P, bf16):
    """Random real-valued data, random masks, many rounds: the fp32 C recurrence stays
    within fp32 rounding of the independently written fp64 one (send buffers, validity,
    parameters, momentum)."""
    n, T, lr, mu = 257, 10, 0.1, 0.9
    rng = np.random.default_rng(P)
    w0 = rng.normal(0, 0.02, n).astype(np.float32)
    w, v = w0.copy(), np.zeros(n, dtype=np.float32)
    R, valid = _empty_R(P, n), 0
    w64, v64, R64 = w0.astype(np.float64), np.zeros(n), [None] * P
    for t in range(T):
        G32 = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(P)]
        if bf16:
            tb = [torch.from_numpy(g).to(torch.bfloat16) for g in G32]
            G = [x.view(torch.int16).numpy().view(np.uint16).copy() for x in tb]
            Gf = [x.to(torch.float32).numpy() for x in tb]   # torch's own widening
        else:
            G, Gf = G32, G32
        mask = int(rng.integers(0, 1 << P, dtype=np.uint64)) if P < 64 else \
            int(rng.integers(0, 1 << 63, dtype=np.uint64)) * 2 + int(rng.integers(0, 2))
        recv = np.empty(n, dtype=np.float32)
        valid = eo.round_f32(G, R, valid, mask, w, v, lr, mu, recv)
        u64, R64, w64, v64 = eo.round_f64(Gf, R64, mask, w64, v64, lr, mu)
        assert np.allclose(recv, u64, rtol=0, atol=1e-6 * np.abs(u64).max())
        assert np.allclose(w, w64, rtol=0, atol=1e-6 * np.abs(w64).max())
        assert np.allclose(v, v64, rtol=0, atol=2e-6 * np.abs(v64).max())
        for p in range(P):
            assert ((valid >> p) & 1) == (R64[p] is not None)
            if R64[p] is not None:
                assert np.array_equal(R[p].astype(np.float64), R64[p])


def test_bf16_widening_matches_torch():
    """All finite bf16 bit patterns: the oracle's widening equals torch's conversion."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    keep = np.isfinite(f)
    recv = np.empty(bits.size, dtype=np.float32)
    eo.round_f32([bits], _empty_R(1, bits.size), 0, 1, None, None, 0, 0, recv)
    assert np.array_equal(recv[keep], f[keep])


def test_threaded_oracle_is_bitwise_the_scalar_one():
    P, n, T = 8, 100003, 4
    rng = np.random.default_rng(5)
    st = []
    for nthreads in (1, 4):
        rs = np.random.default_rng(5)
        w = rs.normal(0, 0.02, n).astype(np.float32)
        v = np.zeros(n, dtype=np.float32)
        R, valid = _empty_R(P, n), 0
        for t in range(T):
            G = [rs.normal(0, 1e-3, n).astype(np.float32) for _ in range(P)]
            mask = int(rs.integers(1, 1 << P))
            valid = eo.round_f32(G, R, valid, mask, w, v, 0.1, 0.9, None, nthreads)
        st.append((w, v, R, valid))
    assert st[0][3] == st[1][3]
    assert np.array_equal(st[0][0], st[1][0]) and np.array_equal(st[0][1], st[1][1])
    for a, b in zip(st[0][2], st[1][2]):
        assert np.array_equal(a, b)


def test_nonfinite_gradients_propagate():
    n = 4
    G = [np.array([np.inf, -np.inf, np.nan, 1.0], dtype=np.float32),
         np.array([1.0, np.inf, 1.0, 1.0], dtype=np.float32)]
    recv = np.empty(n, dtype=np.float32)
    eo.round_f32(G, _empty_R(2, n), 0, 3, None, None, 0, 0, recv)
    assert recv[0] == np.inf and np.isnan(recv[1]) and np.isnan(recv[2]) and recv[3] == 1.0


# ------------------------------------------------------------------ participation plan
def test_plan_safety_and_quorum():
    """Lemma 1: the initiator's own update is always included (Q >= 1); the mask is
    determined by (times, seed, round) alone, so every bucket of a round sees the same
    one."""
    rng = np.random.default_rng(0)
    for it in range(300):
        P = int(rng.integers(1, 65))
        a = rng.random(P).tolist()
        for mode in (eo.SOLO, eo.MAJORITY):
            pl = eo.plan_participation(mode, P, a, 9, it)
            assert pl.nap == bin(pl.mask).count("1") >= 1
            assert (pl.mask >> pl.initiator) & 1 and pl.mask < (1 << P)
            assert pl == eo.plan_participation(mode, P, a, 9, it)


def test_plan_solo_and_majority_counts():
    """Section 7.1: with fully skewed (distinct) arrival times solo has exactly one
    active process, the earliest; majority has the initiator plus everyone earlier.
    Section 4.2: the designated initiator is uniform over ranks, so the expected number
    of active processes is (P + 1) / 2, about half (16 of 32 in Fig. 9)."""
    P = 32
    a = [float(p + 1) for p in range(P)]                  # linear skew 1..32 ms
    s = eo.plan_participation(eo.SOLO, P, a, 1, 0)
    assert s.initiator == 0 and s.mask == 1 and s.nap == 1
    naps, inits = [], []
    for it in range(6400):
        m = eo.plan_participation(eo.MAJORITY, P, a, 1234, it)
        assert m.nap == m.initiator + 1 and m.mask == (1 << m.nap) - 1
        naps.append(m.nap)
        inits.append(m.initiator)
    assert abs(np.mean(naps) - 16.5) < 0.5
    counts = np.bincount(inits, minlength=P)
    assert counts.min() > 120 and counts.max() < 290     # 200 expected per rank
    first64 = np.mean(naps[:64])
    assert 12.0 < first64 < 21.0                           # "on average 16 out of 32"
    # the slowest rank as initiator degenerates to a full allreduce
    b = list(a)
    it = next(i for i in range(1000)
              if eo.plan_participation(eo.MAJORITY, P, a, 1234, i).initiator == P - 1)
    assert eo.plan_participation(eo.MAJORITY, P, b, 1234, it).mask == (1 << P) - 1
    # different seeds give different initiator sequences
    seq = lambda sd: [eo.plan_participation(eo.MAJORITY, P, a, sd, i).initiator for i in range(16)]
    assert seq(1) != seq(2)


def test_plan_ties_window_quorum():
    a = [2.0, 1.0, 1.0, 3.0]
    s = eo.plan_participation(eo.SOLO, 4, a, 0, 0)
    assert s.initiator == 1 and s.mask == 0b0110
    s = eo.plan_participation(eo.SOLO, 4, a, 0, 0, window_ms=1.0)
    assert s.mask == 0b0111
    for k in range(1, 5):
        q = eo.plan_participation(eo.QUORUM, 4, [4.0, 1.0, 3.0, 2.0], 0, 0, quorum=k)
        assert q.nap == k
    assert eo.plan_participation(eo.QUORUM, 4, [4.0, 1.0, 3.0, 2.0], 0, 0, quorum=4).mask == 15
    # strict quorum: majority waits for ceil(P/2) arrivals when the initiator is early
    a = [1.0, 2.0, 3.0, 4.0, 5.0]
    for it in range(50):
        m = eo.plan_participation(eo.MAJORITY, 5, a, 7, it, flags=eo.FLAG_STRICT_QUORUM)
        loose = eo.plan_participation(eo.MAJORITY, 5, a, 7, it)
        assert m.nap == max(3, loose.nap) and (m.mask >> m.initiator) & 1


# ------------------------------------------------------------------ by-products
def test_bucket_stats_closed_forms_and_library_norm():
    """Known vectors: all ones give numel; k^2 sums; non-finite entries are counted and left
    out; padding between buckets is ignored; agrees with numpy's own norm routine."""
    off, num = [0, 8, 16, 16], [5, 7, 0, 9]
    u = np.full(25, 1e30, dtype=np.float32)          # padding poisoned with large values
    w = np.full(25, 1e30, dtype=np.float32)
    u[0:5] = 1.0
    u[8:15] = np.arange(1, 8)
    u[16:25] = 2.0
    u[17], u[20], u[24] = np.nan, np.inf, -np.inf
    w[0:5], w[8:15], w[16:25] = 3.0, 0.5, 1.0
    w[9] = np.nan
    got = eo.bucket_stats(u, w, off, num)
    assert got[0] == (5.0, 45.0, 0)
    assert got[1] == (140.0, 6 * 0.25, 0)            # 1^2 + ... + 7^2 = 140
    assert got[2] == (0.0, 0.0, 0)
    assert got[3] == (6 * 4.0, 9.0, 3)
    assert eo.bucket_stats(u, None, off, num)[0] == (5.0, 0.0, 0)
    rng = np.random.default_rng(0)
    x = rng.standard_normal(1000).astype(np.float32)
    (ssu, ssw, nf), = eo.bucket_stats(x, x, [0], [1000])
    assert nf == 0 and abs(ssu - np.linalg.norm(x.astype(np.float64)) ** 2) < 1e-9 * ssu
    assert ssu == ssw


# ------------------------------------------------------------------ memory safety of the C file
def test_c_oracle_under_address_and_ub_sanitizers(tmp_path):
    """The C oracle driven from C under AddressSanitizer and UndefinedBehaviorSanitizer: every
    mask sequence over three rounds plus a flush, ragged sizes including 0, fp32 and bf16,
    threaded and scalar; conservation checked exactly on integer-valued data."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "oracle_sanitized"
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-g", "-ffp-contract=off", "-fopenmp",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-Wall", "-Wextra",
                           os.path.join(root, "tests", "c", "oracle_sanitized.c"),
                           os.path.join(root, "oracle", "eager_oracle.c"), "-o", str(exe), "-lm"])
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stderr[-2000:]
