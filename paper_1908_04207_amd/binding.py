"""ctypes binding of libeager.so: argument marshalling only.

Every step of a round runs in the library's HIP kernels; nothing here computes.  There
is no fallback: if the shared library is missing the import of this module fails.
PyTorch tensors are accepted as device buffers (their data_ptr is passed on) and the
current torch stream is used unless a stream is given.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libeager.so")

SOLO, MAJORITY, QUORUM = 0, 1, 2
F32, BF16 = 0, 1
ORDER_FIXED, ORDER_FAST = 0, 1
OK, EINVAL, ESHAPE, ESTATE, EDEVICE, ENOMEM, ELIMIT = range(7)
STATIC_MAX_BUCKETS, STATIC_MAX_ELEMENTS = 512, 1 << 27
FLAG_STRICT_QUORUM = 1
MAX_P = 64

EXPORTS = (
    "eager_create", "eager_destroy", "eager_last_error", "eager_status_string", "eager_source_hash",
    "eager_plan_participation", "eager_designated_initiator", "eager_plan_open_round",
    "eager_partial_allreduce_solo",
    "eager_partial_allreduce_majority", "eager_partial_allreduce_quorum", "eager_plan_quorum",
    "eager_partial_allreduce_lagging", "eager_partial_allreduce_exchange", "eager_stash",
    "eager_flush", "eager_sgd_step", "eager_sgd_step_lars",
    "eager_sgd_step_lars_static", "eager_sgd_step_views",
    "eager_average_views", "eager_set_update_rule", "eager_stats_workspace_bytes",
    "eager_stats_attach", "eager_get_valid",
    "eager_set_valid", "eager_set_launch", "eager_calib_copy", "eager_calib_read",
    "eager_calib_mix",
)


class EagerError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{text} (status {status})")
        self.status = status


class Plan(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("P", ctypes.c_int32), ("step", ctypes.c_uint64),
                ("mask", ctypes.c_uint64), ("initiator", ctypes.c_int32),
                ("nap", ctypes.c_int32), ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]

    def __repr__(self):
        return (f"Plan(mode={self.mode}, P={self.P}, step={self.step}, mask={self.mask:#x}, "
                f"initiator={self.initiator}, nap={self.nap})")


class Opt(ctypes.Structure):
    _fields_ = [("params", ctypes.c_void_p), ("momentum", ctypes.c_void_p),
                ("lr", ctypes.c_float), ("mu", ctypes.c_float)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1908_04207_amd.build` "
            "(hipcc, gfx950); there is no fallback path")
    # The library and PyTorch must share ONE HIP runtime (streams and device pointers cross
    # between them).  PyTorch ships its own copy under the same SONAME: loaded first, it
    # also serves this library; loaded second, the process would hold two runtimes and the
    # second one finds no device.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64
    lib.eager_create.argtypes = [ctypes.POINTER(vp), i32, i32, ctypes.POINTER(i64),
                                 ctypes.POINTER(i64), i32, i32]
    lib.eager_destroy.argtypes = [vp]
    lib.eager_last_error.argtypes = [vp]
    lib.eager_last_error.restype = ctypes.c_char_p
    lib.eager_status_string.argtypes = [i32]
    lib.eager_status_string.restype = ctypes.c_char_p
    lib.eager_source_hash.argtypes = []
    lib.eager_source_hash.restype = ctypes.c_char_p
    lib.eager_plan_participation.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_double), u64, u64,
                                             ctypes.c_double, ctypes.c_uint32,
                                             ctypes.POINTER(Plan)]
    lib.eager_designated_initiator.argtypes = [u64, u64, i32, ctypes.POINTER(i32)]
    lib.eager_plan_open_round.argtypes = [i32, i32, u64, i32, i32, u64, u64, ctypes.POINTER(i32),
                                          ctypes.POINTER(Plan)]
    lib.eager_plan_quorum.argtypes = [i32, ctypes.POINTER(ctypes.c_double), i32, u64,
                                      ctypes.c_double, ctypes.POINTER(Plan)]
    for f in (lib.eager_partial_allreduce_solo, lib.eager_partial_allreduce_majority,
              lib.eager_partial_allreduce_quorum):
        f.argtypes = [vp, ctypes.POINTER(Plan), i32, i32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                      vp, ctypes.POINTER(Opt), vp]
    lib.eager_partial_allreduce_lagging.argtypes = [
        vp, ctypes.POINTER(Plan), u64, i32, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
        ctypes.POINTER(Opt), vp]
    lib.eager_partial_allreduce_exchange.argtypes = [
        vp, ctypes.POINTER(Plan), ctypes.POINTER(vp), ctypes.POINTER(vp), vp, ctypes.POINTER(Opt), vp]
    lib.eager_stash.argtypes = [vp, i32, i32, i32, vp, vp, vp]
    lib.eager_flush.argtypes = [vp, i32, i32, ctypes.POINTER(vp), vp, ctypes.POINTER(Opt), vp]
    lib.eager_sgd_step.argtypes = [vp, i32, i32, vp, ctypes.POINTER(Opt), vp]
    lib.eager_sgd_step_lars.argtypes = [vp, i32, i32, vp, ctypes.POINTER(Opt), ctypes.c_float,
                                        ctypes.c_float, vp]
    lib.eager_sgd_step_lars_static.argtypes = [vp, i32, i32, vp, ctypes.POINTER(Opt),
                                               ctypes.c_float, ctypes.c_float, vp, vp]
    lib.eager_sgd_step_views.argtypes = [vp, i32, i32, vp, i32, ctypes.POINTER(vp),
                                         ctypes.POINTER(vp), ctypes.c_float, ctypes.c_float, vp]
    lib.eager_average_views.argtypes = [vp, i32, i32, i32, ctypes.POINTER(vp), vp]
    lib.eager_get_valid.argtypes = [vp, i32, ctypes.POINTER(u64)]
    lib.eager_set_valid.argtypes = [vp, i32, u64]
    lib.eager_set_launch.argtypes = [vp, ctypes.c_char_p, i32]
    lib.eager_set_update_rule.argtypes = [vp, ctypes.c_float, i32]
    lib.eager_stats_workspace_bytes.argtypes = [vp, ctypes.POINTER(i64)]
    lib.eager_stats_attach.argtypes = [vp, vp, vp, i64, vp]
    lib.eager_calib_copy.argtypes = [vp, vp, i64, vp]
    lib.eager_calib_read.argtypes = [vp, i64, vp, vp]
    lib.eager_calib_mix.argtypes = [ctypes.POINTER(vp), i32, u64, ctypes.POINTER(vp), i32, i64, i32,
                                    vp, vp]
    return lib


lib = _load()


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()            # torch tensor


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def source_hash() -> str:
    """Digest of the sources the loaded library was built from."""
    return lib.eager_source_hash().decode()


def status_string(status: int) -> str:
    return lib.eager_status_string(status).decode()


def eager_plan_participation(mode: int, arrival_ms: Sequence[float], seed: int, step: int,
                             window_ms: float = 0.0, flags: int = 0) -> Plan:
    P = len(arrival_ms)
    arr = (ctypes.c_double * max(P, 1))(*arrival_ms)
    plan = Plan()
    st = lib.eager_plan_participation(mode, P, arr, seed & (2 ** 64 - 1), step, window_ms, flags,
                                      ctypes.byref(plan))
    if st != OK:
        raise EagerError(st, f"eager_plan_participation: {status_string(st)}")
    return plan


def eager_plan_quorum(arrival_ms: Sequence[float], quorum: int, step: int,
                      window_ms: float = 0.0) -> Plan:
    P = len(arrival_ms)
    arr = (ctypes.c_double * max(P, 1))(*arrival_ms)
    plan = Plan()
    st = lib.eager_plan_quorum(P, arr, quorum, step, window_ms, ctypes.byref(plan))
    if st != OK:
        raise EagerError(st, f"eager_plan_quorum: {status_string(st)}")
    return plan


def eager_designated_initiator(seed: int, round_: int, P: int) -> int:
    rank = ctypes.c_int()
    st = lib.eager_designated_initiator(seed & (2 ** 64 - 1), round_, P, ctypes.byref(rank))
    if st != OK:
        raise EagerError(st, f"eager_designated_initiator: {status_string(st)}")
    return rank.value


def eager_plan_open_round(mode: int, P: int, waiting: int, newest: int, round_: int,
                          quorum: int = 0, seed: int = 0) -> Optional[Plan]:
    """The plan of execution `round_` if the waiting processes trigger it, else None."""
    go, plan = ctypes.c_int(), Plan()
    st = lib.eager_plan_open_round(mode, P, waiting, newest, quorum, seed & (2 ** 64 - 1), round_,
                                   ctypes.byref(go), ctypes.byref(plan))
    if st != OK:
        raise EagerError(st, f"eager_plan_open_round: {status_string(st)}")
    return plan if go.value else None


def make_plan(mode: int, P: int, step: int, mask: int, initiator: Optional[int] = None,
              flags: int = 0) -> Plan:
    """A plan the caller decides itself (tests, forced masks)."""
    if initiator is None:
        initiator = (mask & -mask).bit_length() - 1
    return Plan(mode, P, step, mask, initiator, bin(mask).count("1"), flags, 0)


class Context:
    """Owns one eager_ctx.  Buffers are passed per call and stay owned by the caller."""

    def __init__(self, P: int, bucket_offset: Sequence[int], bucket_numel: Sequence[int],
                 grad_dtype: int = F32, order: int = ORDER_FIXED):
        n = len(bucket_offset)
        if len(bucket_numel) != n:
            raise ValueError("bucket_offset and bucket_numel differ in length")
        off = (ctypes.c_int64 * max(n, 1))(*bucket_offset)
        num = (ctypes.c_int64 * max(n, 1))(*bucket_numel)
        h = ctypes.c_void_p()
        st = lib.eager_create(ctypes.byref(h), P, n, off, num, grad_dtype, order)
        if st != OK:
            raise EagerError(st, f"eager_create: {status_string(st)}")
        self._h = h
        self.P, self.n_buckets = P, n

    def close(self) -> None:
        if getattr(self, "_h", None) and lib is not None:   # lib is None at interpreter exit
            lib.eager_destroy(self._h)
            self._h = None

    __del__ = close

    def _check(self, st: int, what: str) -> None:
        if st != OK:
            raise EagerError(st, f"{what}: {status_string(st)}: "
                                 f"{lib.eager_last_error(self._h).decode()}")

    @staticmethod
    def pointers(buffers):
        """The pointer table of a list of device buffers, marshalled once: pass it in place
        of the list to the partial allreduce calls of a tight loop."""
        return (ctypes.c_void_p * max(len(buffers), 1))(*[_ptr(x) for x in buffers])

    def _allreduce(self, fn, what, plan, grads, resid, recv, opt, b0, b1, stream):
        b1 = self.n_buckets if b1 is None else b1
        P = len(grads)
        g = grads if isinstance(grads, ctypes.Array) else self.pointers(grads)
        r = resid if isinstance(resid, ctypes.Array) else self.pointers(resid)
        o = None
        if opt is not None:
            params, momentum, lr, mu = opt
            o = ctypes.byref(Opt(_ptr(params), _ptr(momentum), lr, mu))
        if P != self.P or len(resid) != self.P:
            raise EagerError(EINVAL, f"{what}: expected {self.P} gradient and send buffers")
        self._check(fn(self._h, ctypes.byref(plan), b0, b1, g, r, _ptr(recv), o, _stream(stream)),
                    what)

    def eager_partial_allreduce_solo(self, plan: Plan, grads, resid, recv=None, opt=None,
                                     b0: int = 0, b1: Optional[int] = None, stream=None):
        self._allreduce(lib.eager_partial_allreduce_solo, "eager_partial_allreduce_solo", plan,
                        grads, resid, recv, opt, b0, b1, stream)

    def eager_partial_allreduce_majority(self, plan: Plan, grads, resid, recv=None, opt=None,
                                         b0: int = 0, b1: Optional[int] = None, stream=None):
        self._allreduce(lib.eager_partial_allreduce_majority, "eager_partial_allreduce_majority",
                        plan, grads, resid, recv, opt, b0, b1, stream)

    def eager_partial_allreduce_quorum(self, plan: Plan, grads, resid, recv=None, opt=None,
                                       b0: int = 0, b1: Optional[int] = None, stream=None):
        self._allreduce(lib.eager_partial_allreduce_quorum, "eager_partial_allreduce_quorum",
                        plan, grads, resid, recv, opt, b0, b1, stream)

    def eager_partial_allreduce_lagging(self, plan: Plan, absent: int, grads, resid, recv=None,
                                        opt=None, b0: int = 0, b1: Optional[int] = None,
                                        stream=None):
        """grads[p] may be None for the processes in `absent`."""
        fn = lambda h, pl, *rest: lib.eager_partial_allreduce_lagging(h, pl, absent, *rest)  # noqa: E731
        self._allreduce(fn, "eager_partial_allreduce_lagging", plan, grads, resid, recv, opt, b0,
                        b1, stream)

    def eager_partial_allreduce_exchange(self, plan: Plan, grads, resid, recv=None, opt=None,
                                         stream=None) -> None:
        """`grads` and `resid` are pointer tables from Context.pointers (the library exchanges
        the entries of late processes in them), or lists of device buffers - then the two lists
        are permuted in place the way the library permuted their pointers."""
        tables = isinstance(grads, ctypes.Array)
        g = grads if tables else self.pointers(grads)
        r = resid if tables else self.pointers(resid)
        o = None
        if opt is not None:
            params, momentum, lr, mu = opt
            o = ctypes.byref(Opt(_ptr(params), _ptr(momentum), lr, mu))
        if len(grads) != self.P or len(resid) != self.P:
            raise EagerError(EINVAL, f"eager_partial_allreduce_exchange: expected {self.P} "
                                     "gradient and send buffers")
        self._check(lib.eager_partial_allreduce_exchange(self._h, ctypes.byref(plan), g, r,
                                                         _ptr(recv), o, _stream(stream)),
                    "eager_partial_allreduce_exchange")
        if not tables:
            for p in range(self.P):
                if g[p] != _ptr(grads[p]):          # exchanged by the library
                    grads[p], resid[p] = resid[p], grads[p]

    def eager_stash(self, process: int, grad, resid, b0: int = 0, b1: Optional[int] = None,
                    stream=None) -> None:
        b1 = self.n_buckets if b1 is None else b1
        self._check(lib.eager_stash(self._h, process, b0, b1, _ptr(grad), _ptr(resid),
                                    _stream(stream)), "eager_stash")

    def eager_flush(self, resid, recv=None, opt=None, b0: int = 0, b1: Optional[int] = None,
                    stream=None) -> None:
        b1 = self.n_buckets if b1 is None else b1
        r = resid if isinstance(resid, ctypes.Array) else self.pointers(resid)
        o = None
        if opt is not None:
            params, momentum, lr, mu = opt
            o = ctypes.byref(Opt(_ptr(params), _ptr(momentum), lr, mu))
        self._check(lib.eager_flush(self._h, b0, b1, r, _ptr(recv), o, _stream(stream)),
                    "eager_flush")

    def eager_partial_allreduce(self, plan: Plan, *a, **kw):
        """Dispatch on plan.mode to the entry point of that name."""
        fn = {SOLO: self.eager_partial_allreduce_solo,
              MAJORITY: self.eager_partial_allreduce_majority,
              QUORUM: self.eager_partial_allreduce_quorum}[plan.mode]
        fn(plan, *a, **kw)

    def eager_sgd_step(self, update, opt, b0: int = 0, b1: Optional[int] = None, stream=None):
        b1 = self.n_buckets if b1 is None else b1
        params, momentum, lr, mu = opt
        o = Opt(_ptr(params), _ptr(momentum), lr, mu)
        self._check(lib.eager_sgd_step(self._h, b0, b1, _ptr(update), ctypes.byref(o),
                                       _stream(stream)), "eager_sgd_step")

    def eager_sgd_step_lars(self, update, opt, trust: float, eps: float = 0.0, b0: int = 0,
                            b1: Optional[int] = None, stream=None) -> None:
        b1 = self.n_buckets if b1 is None else b1
        params, momentum, lr, mu = opt
        o = Opt(_ptr(params), _ptr(momentum), lr, mu)
        self._check(lib.eager_sgd_step_lars(self._h, b0, b1, _ptr(update), ctypes.byref(o), trust,
                                            eps, _stream(stream)), "eager_sgd_step_lars")

    def eager_sgd_step_lars_static(self, update, opt, trust: float, stats, eps: float = 0.0,
                                   b0: int = 0, b1: Optional[int] = None, stream=None) -> None:
        """The layer-wise update with the library's fixed scratch as workspace; `stats` is the
        device buffer of n_buckets x 32 bytes that receives norms and rates."""
        b1 = self.n_buckets if b1 is None else b1
        params, momentum, lr, mu = opt
        o = Opt(_ptr(params), _ptr(momentum), lr, mu)
        self._check(lib.eager_sgd_step_lars_static(self._h, b0, b1, _ptr(update), ctypes.byref(o),
                                                   trust, eps, _ptr(stats), _stream(stream)),
                    "eager_sgd_step_lars_static")

    def eager_sgd_step_views(self, update, params, momentum, lr: float, mu: float, b0: int = 0,
                             b1: Optional[int] = None, stream=None) -> None:
        b1 = self.n_buckets if b1 is None else b1
        tab = lambda x: x if isinstance(x, ctypes.Array) else self.pointers(x)  # noqa: E731
        self._check(lib.eager_sgd_step_views(self._h, b0, b1, _ptr(update), len(params),
                                             tab(params), tab(momentum),
                                             lr, mu, _stream(stream)), "eager_sgd_step_views")

    def eager_average_views(self, views, b0: int = 0, b1: Optional[int] = None, stream=None) -> None:
        b1 = self.n_buckets if b1 is None else b1
        self._check(lib.eager_average_views(self._h, b0, b1, len(views), self.pointers(views),
                                            _stream(stream)), "eager_average_views")

    def eager_get_valid(self, bucket: int) -> int:
        v = ctypes.c_uint64()
        self._check(lib.eager_get_valid(self._h, bucket, ctypes.byref(v)), "eager_get_valid")
        return v.value

    def eager_set_valid(self, bucket: int, valid_mask: int) -> None:
        self._check(lib.eager_set_valid(self._h, bucket, valid_mask), "eager_set_valid")

    def eager_set_update_rule(self, weight_decay: float = 0.0, nesterov: bool = False) -> None:
        self._check(lib.eager_set_update_rule(self._h, weight_decay, int(nesterov)),
                    "eager_set_update_rule")

    def eager_stats_workspace_bytes(self) -> int:
        n = ctypes.c_int64()
        self._check(lib.eager_stats_workspace_bytes(self._h, ctypes.byref(n)),
                    "eager_stats_workspace_bytes")
        return n.value

    def eager_stats_attach(self, stats, workspace, workspace_bytes: int = 0, stream=None) -> None:
        """stats: device buffer of n_buckets x 32 bytes (sumsq_update f64, sumsq_params f64,
        nonfinite u64, rate f32, reserved u32), or None to detach; workspace: device buffer."""
        self._check(lib.eager_stats_attach(self._h, _ptr(stats), _ptr(workspace), workspace_bytes,
                                           _stream(stream)), "eager_stats_attach")

    def eager_set_launch(self, key: str, value: int) -> None:
        self._check(lib.eager_set_launch(self._h, key.encode(), value), "eager_set_launch")


def eager_calib_copy(dst, src, nbytes: int, stream=None) -> None:
    st = lib.eager_calib_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream))
    if st != OK:
        raise EagerError(st, f"eager_calib_copy: {status_string(st)}")


def eager_calib_read(src, nbytes: int, sink, stream=None) -> None:
    st = lib.eager_calib_read(_ptr(src), nbytes, _ptr(sink), _stream(stream))
    if st != OK:
        raise EagerError(st, f"eager_calib_read: {status_string(st)}")


def eager_calib_mix(read, write, n_vec: int, read_half_mask: int = 0, waves_per_cu: int = 0,
                    sink=None, stream=None) -> None:
    """A plain kernel that reads len(read) streams and writes len(write) streams (n_vec
    16-byte lane-vectors each).  `read` and `write` are lists of device buffers or pointer
    tables from Context.pointers."""
    r = read if isinstance(read, ctypes.Array) else Context.pointers(read)
    w = write if isinstance(write, ctypes.Array) else Context.pointers(write)
    st = lib.eager_calib_mix(r, len(read), read_half_mask, w, len(write), n_vec, waves_per_cu,
                             _ptr(sink), _stream(stream))
    if st != OK:
        raise EagerError(st, f"eager_calib_mix: {status_string(st)}")
