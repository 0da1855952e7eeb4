"""The entry point that allocates nothing (eager_sgd_step_lars_static: statistics workspace in
the library's fixed device array) against the entry point it is a variant of
(eager_sgd_step_lars with a caller-provided workspace): same kernels, so parameters, momentum,
norms and rates must agree bit for bit - on two calls in a row that share the fixed array, the
second on a smaller problem, and again on a third that reuses the first context.  Collected
last on purpose (the name sorts after every other test file)."""
import numpy as np
import pytest
import torch

from paper_1908_04207_amd import binding as eb

pytestmark = pytest.mark.gpu


def _layout(numels, align=4):
    off, pos = [], 0
    for n in numels:
        off.append(pos)
        pos = (pos + n + align - 1) // align * align
    return off, list(numels), pos


class _Case:
    """One problem: an update u, parameters and momentum, once for each entry point."""

    def __init__(self, numels, order, seed, wd=0.0, nesterov=False):
        self.off, self.num, self.n = _layout(numels)
        nb = len(numels)
        g = torch.Generator(device="cuda").manual_seed(seed)
        self.u = torch.randn(self.n, device="cuda", generator=g) * 1e-3
        w0 = torch.randn(self.n, device="cuda", generator=g) * 0.02
        v0 = torch.randn(self.n, device="cuda", generator=g) * 1e-3
        # one layer of zero parameters (rate 1), one non-finite update element
        w0[self.off[nb // 2]:self.off[nb // 2] + self.num[nb // 2]] = 0.0
        self.u[self.off[-1] + 1] = float("inf")
        self.w = [w0.clone(), w0.clone()]
        self.v = [v0.clone(), v0.clone()]
        self.ctx = [eb.Context(1, self.off, self.num, eb.F32, order) for _ in range(2)]
        for c in self.ctx:
            c.eager_set_update_rule(wd, nesterov)
        self.stats = [torch.full((nb * 4,), -1.0, dtype=torch.float64, device="cuda")
                      for _ in range(2)]
        nbytes = self.ctx[0].eager_stats_workspace_bytes()
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.ctx[0].eager_stats_attach(self.stats[0], self.ws, nbytes)

    def step(self, b0=0, b1=None, trust=0.02, eps=1e-9):
        lr, mu = 0.1, 0.9
        self.ctx[0].eager_sgd_step_lars(self.u, (self.w[0], self.v[0], lr, mu), trust, eps, b0, b1)
        self.ctx[1].eager_sgd_step_lars_static(self.u, (self.w[1], self.v[1], lr, mu), trust,
                                               self.stats[1], eps, b0, b1)
        torch.cuda.synchronize()

    def check(self, what):
        for name, pair in (("w", self.w), ("v", self.v)):
            a, b = pair[0].view(torch.int32), pair[1].view(torch.int32)
            assert torch.equal(a, b), f"{what}: {name} differs in {int((a != b).sum())} elements"
        a, b = self.stats[0].view(torch.int64), self.stats[1].view(torch.int64)
        assert torch.equal(a, b), f"{what}: per-bucket norms / rates differ"
        rates = self.stats[1].cpu().numpy().view(np.uint8).reshape(-1, 32)[:, 24:28].copy().view(np.float32)
        return rates[:, 0]


def test_static_scratch_matches_caller_workspace_on_consecutive_calls():
    # large: a bucket beyond a million elements (its records are added in slices), tiny and
    # ragged buckets that share wavefronts, a ragged tail
    big = _Case([5, 1000, 2_200_001, 64, 7, 300_003, 12], eb.ORDER_FIXED, seed=1, wd=5e-4)
    big.step()
    r_big = big.check("first call")
    assert r_big[3] == 1.0                       # the layer of zero parameters
    assert (r_big > 0).all() and np.isfinite(r_big).all()
    # smaller, right after, in the same fixed array (which still holds the first call's records)
    small = _Case([700, 3, 4097, 256, 90_001], eb.ORDER_FAST, seed=2, nesterov=True)
    small.step()
    small.check("second, smaller call")
    # a bucket range of the smaller problem, then the large one again
    small.step(b0=1, b1=4, trust=0.5)
    small.check("range call")
    big.step(trust=0.001, eps=0.0)
    big.check("large problem again")


def test_static_scratch_alone_in_a_fresh_state():
    """The entry point on its own, as the very first statistics call of a context: no
    eager_stats_attach anywhere on the static side."""
    c = _Case([4096, 33, 100_000], eb.ORDER_FIXED, seed=3)
    c.step()
    rates = c.check("single call")
    # norms against torch on the same data: |u| over finite elements
    torch.cuda.synchronize()
    raw = c.stats[1].cpu().numpy()
    for b, (o, n) in enumerate(zip(c.off, c.num)):
        u = c.u[o:o + n].double()
        fin = torch.isfinite(u)
        want = float((u[fin] ** 2).sum())
        assert abs(raw[4 * b] - want) <= 1e-10 * max(want, 1e-300)
        assert raw.view(np.uint64)[4 * b + 2] == int((~fin).sum())
    assert rates.shape == (3,)


def test_static_scratch_call_captured_in_a_graph():
    """What the entry point is for: under HIP graph capture nothing may allocate, copy from
    pageable memory or synchronise.  After one eager call (it looks up the array's address and
    loads the kernels) the call is captured - together with an eager_stats_attach, whose bucket
    table is written by a kernel - and replayed on new updates with eager work and
    synchronisations in between; every replay must leave the bits of the same calls made eagerly
    on a second copy of the state."""
    numels = [4096, 33, 100_000, 7, 260_000]
    off, num, n = _layout(numels)
    nb = len(numels)

    class Side:
        def __init__(self):
            g = torch.Generator(device="cuda").manual_seed(11)
            self.u = torch.zeros(n, device="cuda")
            self.w = torch.randn(n, device="cuda", generator=g) * 0.02
            self.v = torch.zeros(n, device="cuda")
            self.ctx = eb.Context(1, off, num, eb.F32, eb.ORDER_FIXED)
            self.stats = torch.zeros(nb * 4, dtype=torch.float64, device="cuda")
            self.attached = torch.zeros(nb * 4, dtype=torch.float64, device="cuda")
            nbytes = self.ctx.eager_stats_workspace_bytes()
            self.ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            self.nbytes = nbytes

        def calls(self, stream=None):
            self.ctx.eager_stats_attach(self.attached, self.ws, self.nbytes, stream=stream)
            self.ctx.eager_sgd_step_lars_static(self.u, (self.w, self.v, 0.1, 0.9), 0.02, self.stats,
                                                1e-9, stream=stream)

        def load(self, t):
            g = torch.Generator(device="cuda").manual_seed(100 + t)
            self.u.copy_(torch.randn(n, device="cuda", generator=g) * 1e-3)

    eager, replayed = Side(), Side()
    for side in (eager, replayed):
        side.load(0)
        side.calls()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        graph.capture_begin()
        replayed.calls(stream=stream)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(stream)
    for t in range(1, 5):
        eager.load(t)
        replayed.load(t)
        eager.calls()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(eager.w, replayed.w) and torch.equal(eager.v, replayed.v), t
        assert torch.equal(eager.stats.view(torch.int64), replayed.stats.view(torch.int64)), t
        table = replayed.ws[:nb * 16].view(torch.int64).cpu().tolist()
        assert table == [x for o, m in zip(off, num) for x in (o, o + m)]
        _ = (eager.w * 2).sum().item()                 # unrelated eager work and a sync
    eager.ctx.close()
    replayed.ctx.close()
