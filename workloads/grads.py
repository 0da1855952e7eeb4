"""Counter-based synthetic gradients and initial parameters.

value(seed, step, rank, arena index) is a pure function built from 64-bit integer
hashing, an integer sum and ONE fp32 multiplication, written with torch tensor ops so
the very same code runs on the host (inputs of the CPU oracle) and on the GPU (inputs of
the HIP path) and yields identical bits on both: there is no transcendental function and
no reduction whose order could differ.  The distribution is an 8-term Irwin-Hall
approximation of N(0, sigma) with exact standard deviation sigma; the path under test
never looks at values, only at sizes, dtypes and masks, so the bell shape is only there
to give realistic rounding patterns.

bf16 gradients are the fp32 value rounded to nearest-even with integer operations.

Nothing of the method (participation, carry, update) lives in this module.
"""
from __future__ import annotations

import math

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

PARAM_RANK = 1 << 20   # "rank" slot used for the initial parameters


def _signed(x: int) -> int:
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _signed(_C1)
    z = (z ^ _lsr(z, 27)) * _signed(_C2)
    return z ^ _lsr(z, 31)


def _lanes(h: torch.Tensor) -> torch.Tensor:
    return (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)


def stream_key(seed: int, step: int, rank: int) -> int:
    k = _mix_int(seed + _GAMMA * (step + 1))
    return _mix_int(k + _GAMMA * (rank + 1))


_IH8_STD = math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)


def scale_f32(sigma: float) -> float:
    """The fp32 constant that maps the centred integer sum to standard deviation sigma."""
    return float(np.float32(sigma / _IH8_STD))


def values_at(index: torch.Tensor, seed: int, step: int, rank: int, sigma: float
              ) -> torch.Tensor:
    """fp32 values at the given int64 arena indices (any device)."""
    key = stream_key(seed, step, rank)
    h1 = _mix(index * _signed(_GAMMA) + _signed(key))
    h2 = _mix(h1 + _signed(_GAMMA))
    s = _lanes(h1) + _lanes(h2) - 4 * 65535
    return s.to(torch.float32) * scale_f32(sigma)


def f32_to_bf16_rne(x: torch.Tensor) -> torch.Tensor:
    """Round fp32 to bf16 (nearest even) with integer ops; finite inputs only."""
    b = x.view(torch.int32)
    r = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return r.to(torch.int16).view(torch.bfloat16)


def fill(out: torch.Tensor, seed: int, step: int, rank: int, sigma: float,
         index_base: int = 0, chunk: int = 1 << 24) -> torch.Tensor:
    """Fill the 1-D tensor `out` (float32 or bfloat16) with the values at arena indices
    index_base .. index_base + len(out) - 1.  Works in chunks to bound temporaries."""
    if out.dim() != 1:
        raise ValueError("fill expects a 1-D tensor")
    n = out.numel()
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        idx = torch.arange(index_base + a, index_base + b, dtype=torch.int64,
                           device=out.device)
        v = values_at(idx, seed, step, rank, sigma)
        if out.dtype == torch.bfloat16:
            v = f32_to_bf16_rne(v)
        elif out.dtype != torch.float32:
            raise ValueError("fill supports float32 and bfloat16")
        out[a:b] = v
    return out


def grad_at(index: torch.Tensor, seed: int, step: int, rank: int, sigma: float,
            dtype: torch.dtype) -> torch.Tensor:
    v = values_at(index, seed, step, rank, sigma)
    return f32_to_bf16_rne(v) if dtype == torch.bfloat16 else v
