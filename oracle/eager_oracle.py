"""CPU oracle for the eager-SGD hot path (Python side).

TEST INFRASTRUCTURE ONLY: used by the tests, the smoke check and the benchmark's
cpu_baseline leg.  Never imported by the GPU library or its binding, and shares no code
with them.

Contents
  plan_participation   who is active in a round (Sections 4.1, 4.2, 7.1 of the paper)
  round_f32 / sgd_f32  thin ctypes wrappers over eager_oracle.c (the fp32 definition)
  round_f64            the same recurrence in numpy fp64, written independently of the C
                       file; used to pin the C code and to bound fp32 rounding
  OracleState          per-bucket bookkeeping of send-buffer validity over many rounds
  bucket_stats         per-bucket by-products of a round (norms of update and parameters)
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "eager_oracle.c")
_LIB = os.path.join(_HERE, "libeager_oracle.so")

SOLO, MAJORITY, QUORUM = 0, 1, 2
FLAG_STRICT_QUORUM = 1

_M64 = (1 << 64) - 1


# --------------------------------------------------------------------------- build / load
def build(force: bool = False) -> str:
    """Compile eager_oracle.c with gcc (contraction off, OpenMP for the threaded leg)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp",
                               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.eager_oracle_round.restype = None
        lib.eager_oracle_round.argtypes = [
            ctypes.c_int, ctypes.c_int64, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
            ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_float,
            ctypes.c_void_p, ctypes.c_int]
        lib.eager_oracle_round_async.restype = None
        lib.eager_oracle_round_async.argtypes = [
            ctypes.c_int, ctypes.c_int64, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
            ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_float,
            ctypes.c_float, ctypes.c_int, ctypes.c_void_p, ctypes.c_int]
        lib.eager_oracle_stash.restype = None
        lib.eager_oracle_stash.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_int]
        lib.eager_oracle_round_ex.restype = None
        lib.eager_oracle_round_ex.argtypes = [
            ctypes.c_int, ctypes.c_int64, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
            ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_float,
            ctypes.c_float, ctypes.c_int, ctypes.c_void_p, ctypes.c_int]
        lib.eager_oracle_sgd_ex.restype = None
        lib.eager_oracle_sgd_ex.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int, ctypes.c_int]
        lib.eager_oracle_sgd_lars.restype = ctypes.c_float
        lib.eager_oracle_sgd_lars.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int, ctypes.c_float,
            ctypes.c_float]
        lib.eager_oracle_sgd.restype = None
        lib.eager_oracle_sgd.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_float, ctypes.c_float, ctypes.c_int]
        _lib = lib
    return _lib


# --------------------------------------------------------------------------- participation
def initiator_hash(seed: int, step: int) -> int:
    """64-bit counter hash shared by all processes for the designated initiator of a
    majority round (Section 4.2: consensus through a common seed).  The paper names no
    generator; this is the SplitMix64 output function applied to seed + (step+1)*gamma."""
    z = (seed + (step + 1) * 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


@dataclass(frozen=True)
class Plan:
    mode: int
    P: int
    step: int
    mask: int
    initiator: int
    nap: int


def plan_participation(mode: int, P: int, arrival_ms: Sequence[float], seed: int,
                       step: int, window_ms: float = 0.0, flags: int = 0,
                       quorum: int = 0) -> Plan:
    """Participation set of one round.

    Solo (Section 4.1): the first process to arrive is the initiator and triggers the
    collective at once.  Majority (Section 4.2): the initiator is a rank drawn from a
    seed all processes share; only it may trigger.  In both, the active processes are
    the initiator and everyone who reached the collective no later than it (Section
    7.1); the others take part passively.  Arrival times are measured from a common
    origin per round, as in the paper's microbenchmark which skews the processes anew
    before every call.

    window_ms widens "no later than" by the time an activation needs to spread
    (Section 4.2 speaks of processes arriving at a similar time as the initiator);
    default 0.  Ties count as on time; a tie for first place in solo mode goes to the
    lowest rank.  FLAG_STRICT_QUORUM (majority only) additionally waits until at least
    ceil(P/2) processes have arrived, the literal "at least half" of Section 4.2.
    QUORUM mode (the spectrum between solo and full the conclusions propose): the round
    triggers when `quorum` processes have arrived.
    """
    if not 1 <= P <= 64 or len(arrival_ms) != P:
        raise ValueError("P must be 1..64 and match arrival_ms")
    a = [float(x) for x in arrival_ms]
    if any(x != x for x in a):
        raise ValueError("arrival time is NaN")
    order = sorted(range(P), key=lambda p: (a[p], p))
    if mode == SOLO:
        init = order[0]
    elif mode == MAJORITY:
        init = initiator_hash(seed, step) % P
    elif mode == QUORUM:
        if not 1 <= quorum <= P:
            raise ValueError("quorum must be 1..P")
        init = order[quorum - 1]
    else:
        raise ValueError("mode")
    threshold = a[init] + window_ms
    if mode == MAJORITY and (flags & FLAG_STRICT_QUORUM):
        need = (P + 1) // 2
        kth = a[order[need - 1]]
        if kth > threshold:
            threshold = kth
    mask = 0
    for p in range(P):
        if a[p] <= threshold:
            mask |= 1 << p
    return Plan(mode, P, step, mask, init, bin(mask).count("1"))


# --------------------------------------------------------------------------- fp32 (C)
def _ptr_array(arrs: Sequence[np.ndarray]):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def round_f32(G: Sequence[np.ndarray], R: Sequence[np.ndarray], valid: int, mask: int,
              w: Optional[np.ndarray], v: Optional[np.ndarray], lr: float, mu: float,
              recv: Optional[np.ndarray] = None, nthreads: int = 1,
              wd: float = 0.0, nesterov: bool = False, absent: int = 0) -> int:
    """One round on one bucket, in place.  G[p]: float32 or uint16 (bf16 bit patterns);
    R[p], w, v, recv: float32.  wd, nesterov: variants of the update rule (off by
    default).  absent: processes (not in mask) that finish no gradient in this round's
    window: they contribute their send buffer and store nothing; their G[p] is not read
    (pass any array of the right shape).  Returns the new validity mask (the late
    processes that stored a gradient)."""
    P = len(G)
    n = G[0].shape[0]
    bf16 = G[0].dtype == np.uint16
    assert absent & mask == 0
    for p in range(P):
        assert G[p].dtype == (np.uint16 if bf16 else np.float32) and G[p].shape == (n,)
        assert R[p].dtype == np.float32 and R[p].shape == (n,)
        assert G[p].flags.c_contiguous and R[p].flags.c_contiguous
    for x in (w, v, recv):
        assert x is None or (x.dtype == np.float32 and x.shape == (n,) and x.flags.c_contiguous)
    assert (w is None) == (v is None)
    _load().eager_oracle_round_async(
        P, n, _ptr_array(G), int(bf16), _ptr_array(R), valid & _M64, mask & _M64, absent & _M64,
        None if w is None else w.ctypes.data, None if v is None else v.ctypes.data,
        lr, mu, wd, int(nesterov), None if recv is None else recv.ctypes.data, nthreads)
    return ~mask & ~absent & ((1 << P) - 1)


def stash_f32(G: np.ndarray, R: np.ndarray, has_stale: bool) -> None:
    """A gradient finished too late for its round goes into the send buffer: R = G if the
    buffer was empty, else R = R + G."""
    bf16 = G.dtype == np.uint16
    assert G.dtype == (np.uint16 if bf16 else np.float32) and R.dtype == np.float32
    assert G.shape == R.shape and G.flags.c_contiguous and R.flags.c_contiguous
    _load().eager_oracle_stash(G.shape[0], G.ctypes.data, int(bf16), R.ctypes.data,
                               int(has_stale))


def sgd_f32(u: np.ndarray, w: np.ndarray, v: np.ndarray, lr: float, mu: float,
            nthreads: int = 1, wd: float = 0.0, nesterov: bool = False) -> None:
    for x in (u, w, v):
        assert x.dtype == np.float32 and x.shape == u.shape and x.flags.c_contiguous
    _load().eager_oracle_sgd_ex(u.shape[0], u.ctypes.data, w.ctypes.data, v.ctypes.data,
                                lr, mu, wd, int(nesterov), nthreads)


def sgd_lars_f32(u: np.ndarray, w: np.ndarray, v: np.ndarray, offset: Sequence[int],
                 numel: Sequence[int], lr: float, mu: float, trust: float, eps: float = 0.0,
                 wd: float = 0.0, nesterov: bool = False) -> List[float]:
    """The update rule with a layer-wise rate (layer = bucket), in place on w and v; padding
    between buckets is not touched.  Returns the rate of every bucket."""
    for x in (u, w, v):
        assert x.dtype == np.float32 and x.shape == u.shape and x.flags.c_contiguous
    lib, rates = _load(), []
    for lo, n in zip(offset, numel):
        rates.append(float(lib.eager_oracle_sgd_lars(
            n, u[lo:].ctypes.data, w[lo:].ctypes.data, v[lo:].ctypes.data, lr, mu, wd,
            int(nesterov), trust, eps)))
    return rates


# --------------------------------------------------------------------------- fp64 (numpy)
def round_f64(G: Sequence[np.ndarray], R: List[Optional[np.ndarray]], mask: int,
              w: np.ndarray, v: np.ndarray, lr: float, mu: float):
    """The same round in real-number terms (numpy fp64).  R[p] is None for an empty send
    buffer (G_null).  Returns (u, R', w', v'); inputs are not modified.

    Written from the paper's walk-through (Section 5) and Algorithm 2, not from the C
    file: contributions are collected as whole vectors, late gradients replace the send
    buffer, on-time processes end with an empty one."""
    P = len(G)
    total = np.zeros_like(np.asarray(G[0], dtype=np.float64))
    R_next: List[Optional[np.ndarray]] = []
    for p in range(P):
        fresh = np.asarray(G[p], dtype=np.float64)
        pending = R[p]
        if (mask >> p) & 1:
            total = total + fresh
            if pending is not None:
                total = total + pending
            R_next.append(None)
        else:
            if pending is not None:
                total = total + pending
            R_next.append(fresh.copy())
    u = total / P
    v_next = mu * v + u
    w_next = w - lr * v_next
    return u, R_next, w_next, v_next


# --------------------------------------------------------------------------- many rounds
class OracleState:
    """fp32 oracle over a bucketed arena: w, v, R_p as flat float32 arrays plus one
    validity mask per bucket.  Buckets are independent (layer-wise reductions, Section
    3), so a round may be applied to any bucket range."""

    def __init__(self, P: int, offset: Sequence[int], numel: Sequence[int],
                 arena_numel: int, w0: np.ndarray, lr: float, mu: float,
                 wd: float = 0.0, nesterov: bool = False):
        self.P, self.lr, self.mu = P, float(lr), float(mu)
        self.wd, self.nesterov = float(wd), bool(nesterov)
        self.offset, self.numel = list(offset), list(numel)
        self.w = np.ascontiguousarray(w0, dtype=np.float32).copy()
        assert self.w.shape == (arena_numel,)
        self.v = np.zeros(arena_numel, dtype=np.float32)
        self.R = [np.zeros(arena_numel, dtype=np.float32) for _ in range(P)]
        self.valid = [0] * len(self.numel)

    def round(self, mask: int, G: Sequence[np.ndarray], b0: int = 0,
              b1: Optional[int] = None, recv: Optional[np.ndarray] = None,
              fused: bool = True, nthreads: int = 1, absent: int = 0) -> None:
        b1 = len(self.numel) if b1 is None else b1
        for b in range(b0, b1):
            lo, hi = self.offset[b], self.offset[b] + self.numel[b]
            self.valid[b] = round_f32(
                [g[lo:hi] for g in G], [r[lo:hi] for r in self.R], self.valid[b], mask,
                self.w[lo:hi] if fused else None, self.v[lo:hi] if fused else None,
                self.lr, self.mu, None if recv is None else recv[lo:hi], nthreads,
                self.wd, self.nesterov, absent)

    def stash(self, p: int, G: np.ndarray, b0: int = 0, b1: Optional[int] = None) -> None:
        b1 = len(self.numel) if b1 is None else b1
        for b in range(b0, b1):
            lo, hi = self.offset[b], self.offset[b] + self.numel[b]
            stash_f32(G[lo:hi], self.R[p][lo:hi], bool((self.valid[b] >> p) & 1))
            self.valid[b] |= 1 << p

    def sgd(self, u: np.ndarray, b0: int = 0, b1: Optional[int] = None,
            nthreads: int = 1) -> None:
        b1 = len(self.numel) if b1 is None else b1
        for b in range(b0, b1):
            lo, hi = self.offset[b], self.offset[b] + self.numel[b]
            sgd_f32(u[lo:hi], self.w[lo:hi], self.v[lo:hi], self.lr, self.mu, nthreads,
                    self.wd, self.nesterov)


# --------------------------------------------------------------------------- by-products
def bucket_stats(u: np.ndarray, w_before: Optional[np.ndarray], offset: Sequence[int],
                 numel: Sequence[int]):
    """Per bucket: sum of u_i^2 over finite u_i, sum of w_i^2 over finite w_i (parameters
    before the update; 0 if None), number of non-finite u_i.  Plain fp64 numpy over each
    bucket's slice; padding between buckets is not part of any bucket."""
    out = []
    for lo, n in zip(offset, numel):
        ub = np.asarray(u[lo:lo + n], dtype=np.float64)
        fin = np.isfinite(ub)
        ssu = float(np.sum(np.square(ub[fin])))
        ssw = 0.0
        if w_before is not None:
            wb = np.asarray(w_before[lo:lo + n], dtype=np.float64)
            ssw = float(np.sum(np.square(wb[np.isfinite(wb)])))
        out.append((ssu, ssw, int(n - np.count_nonzero(fin))))
    return out
