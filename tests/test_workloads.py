"""Input recipe: layouts match the sizes the paper's Table 1 and the benchmark list name;
generators are counter based and reproducible ("parity unpinned" by the paper: the seeds
and distributions are this benchmark's own, pinned here by stored checksums)."""
import hashlib
import json
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from workloads import grads, shapes, times  # noqa: E402

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "workload_checksums.json")


def test_layout_sizes():
    want = {1: (1048576, 1), 2: (25559081, 161), 3: (67332197, 8),
            4: (354823168, 73), 5: (1557611200, 145)}
    for k, (n, nb) in want.items():
        c = shapes.config(k)
        assert c.numel == n and c.buckets.n_buckets == nb
        bt = c.buckets
        for b in range(nb):
            assert bt.offset[b] % bt.align == 0
            if b:
                assert bt.offset[b] >= bt.offset[b - 1] + bt.numel[b - 1]
        assert bt.arena_numel >= bt.offset[-1] + bt.numel[-1]
    c2 = shapes.config(2)
    small = [n for n in c2.buckets.numel if n <= 2048]
    assert len(small) == 107 and sum(small) == 54121
    assert min(c2.buckets.numel) == 64 and max(c2.buckets.numel) == 2359296
    # 25 MiB cap: only single oversized tensors exceed it
    for k, gb in ((4, 4), (5, 2)):
        c = shapes.config(k)
        big = {n for _, n in c.tensors if n * gb > 25 * 2 ** 20}
        for n in c.buckets.numel:
            assert n * gb <= 25 * 2 ** 20 or n in big


def test_scaled_layout_keeps_structure():
    c = shapes.scaled(shapes.config(2), 5000)
    assert c.buckets.n_buckets == 161 and max(c.buckets.numel) == 5000
    assert min(c.buckets.numel) == 64


def _digest():
    out = {}
    for k in range(1, 6):
        c = shapes.config(k)
        ts = [times.compute_times(c.times, c.P, c.seed, t) for t in range(3)]
        out[f"times{k}"] = hashlib.sha256(np.asarray(ts).tobytes()).hexdigest()[:16]
    g = grads.fill(torch.empty(4099), 190804207, 3, 2, 1e-3, index_base=12345)
    out["grad_f32"] = hashlib.sha256(g.numpy().tobytes()).hexdigest()[:16]
    b = grads.fill(torch.empty(4099, dtype=torch.bfloat16), 190804207, 3, 2, 1e-3, 12345)
    out["grad_bf16"] = hashlib.sha256(b.view(torch.int16).numpy().tobytes()).hexdigest()[:16]
    return out


def test_generators_match_stored_checksums():
    got = _digest()
    if not os.path.exists(GOLDEN):          # written once by running this file as a script
        raise AssertionError("golden checksums missing: python tests/test_workloads.py")
    assert got == json.load(open(GOLDEN))


def test_gradient_generator_properties():
    x = grads.fill(torch.empty(1 << 18), 5, 0, 0, 1e-3)
    assert abs(float(x.std()) - 1e-3) < 2e-5 and abs(float(x.mean())) < 1e-5
    # any slice can be regenerated on its own, and by index
    y = grads.fill(torch.empty(1000), 5, 0, 0, 1e-3, index_base=777, chunk=300)
    assert torch.equal(y, x[777:1777])
    idx = torch.tensor([0, 5, 99999, 262143])
    assert torch.equal(grads.values_at(idx, 5, 0, 0, 1e-3), x[idx])
    assert not torch.equal(grads.fill(torch.empty(64), 5, 1, 0, 1e-3), x[:64])
    assert not torch.equal(grads.fill(torch.empty(64), 5, 0, 1, 1e-3), x[:64])
    # integer RNE to bf16 equals torch's conversion
    b = grads.fill(torch.empty(1 << 16, dtype=torch.bfloat16), 5, 0, 0, 1e-3)
    assert torch.equal(b, x[:1 << 16].to(torch.bfloat16))


def test_compute_time_recipes():
    P = 16
    for t in range(50):
        u = times.compute_times("uniform_1_2", P, 1, t)
        assert all(1.0 <= x < 2.0 for x in u)
        assert all(x >= 1.0 for x in times.compute_times("pareto_1.5", P, 1, t))
        a = times.compute_times("lognormal_0.3", P, 1, t)
        b = times.compute_times("lognormal_0.3_straggler2x", P, 1, t)
        r = times.straggler_rank(1, t, P)
        assert [y / x for x, y in zip(a, b)] == [2.0 if p == r else 1.0 for p in range(P)]
    assert times.compute_times("linear_skew", 4, 0, 0) == [1.0, 2.0, 3.0, 4.0]
    z = [np.log(x) for t in range(400) for x in times.compute_times("lognormal_0.5", P, 3, t)]
    assert abs(np.mean(z)) < 0.03 and abs(np.std(z) - 0.5) < 0.03


if __name__ == "__main__":
    json.dump(_digest(), open(GOLDEN, "w"), indent=1, sort_keys=True)
    print("wrote", GOLDEN)
