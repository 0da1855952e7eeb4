"""Seeded per-process, per-step compute times (milliseconds, host fp64).

The paper motivates partial collectives with measured batch-time distributions that
have one mode and a long tail (Section 2: LSTM on UCF101, Transformer on WMT16,
ResNet-50 on cloud instances) and, in its simulated-imbalance experiments, delays a few
randomly chosen ranks per step (Section 7.2).  These generators reproduce those shapes
synthetically.  They are inputs to the participation plan on both the CPU-oracle and the
GPU-library side; nothing here belongs to the method itself.

Everything is counter based: the value for (seed, step, rank, stream) is a pure function,
so any step can be regenerated in isolation.
"""
from __future__ import annotations

import math
from typing import List

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15


def _mix(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _u01(seed: int, step: int, rank: int, stream: int) -> float:
    """Uniform in (0, 1): 53 hashed bits, never exactly 0."""
    k = _mix(seed + _GAMMA * (step + 1))
    k = _mix(k + _GAMMA * (rank + 1))
    k = _mix(k + _GAMMA * (stream + 1))
    return ((k >> 11) + 0.5) / float(1 << 53)


def _normal(seed: int, step: int, rank: int) -> float:
    u1 = _u01(seed, step, rank, 1)
    u2 = _u01(seed, step, rank, 2)
    return math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2)


def straggler_rank(seed: int, step: int, P: int) -> int:
    return _mix(_mix(seed + _GAMMA * (step + 1)) + 0x5DEECE66D) % P


def compute_times(recipe: str, P: int, seed: int, step: int) -> List[float]:
    """Compute times of all P ranks at one step for a named recipe.

    uniform_1_2                 Uniform(1, 2) ms
    lognormal_<s>               exp(s * z) ms, z standard normal
    lognormal_<s>_straggler2x   same, with one seeded rank per step slowed down 2x
    pareto_<a>                  Pareto(alpha = a, x_m = 1 ms): (1 - u)^(-1/a)
    linear_skew                 rank p takes p + 1 ms (the paper's microbenchmark skew,
                                Section 7.1)
    """
    if recipe == "uniform_1_2":
        return [1.0 + _u01(seed, step, p, 0) for p in range(P)]
    if recipe.startswith("lognormal_"):
        parts = recipe.split("_")
        sigma = float(parts[1])
        t = [math.exp(sigma * _normal(seed, step, p)) for p in range(P)]
        if len(parts) > 2:
            if parts[2] != "straggler2x":
                raise ValueError(recipe)
            t[straggler_rank(seed, step, P)] *= 2.0
        return t
    if recipe.startswith("pareto_"):
        alpha = float(recipe.split("_")[1])
        return [(1.0 - _u01(seed, step, p, 0)) ** (-1.0 / alpha) for p in range(P)]
    if recipe == "linear_skew":
        return [float(p + 1) for p in range(P)]
    raise ValueError(f"unknown compute-time recipe {recipe!r}")
