"""eager-SGD hot path on MI355X: partial allreduce (solo / majority) with stale-gradient
carry fused with momentum SGD, as hand-written gfx950 kernels behind a C ABI.

`paper_1908_04207_amd.binding` is the thin ctypes layer over libeager.so; it is loaded on
first use so that `python -m paper_1908_04207_amd.build` can run before the library exists.
"""
import importlib

__all__ = ["binding", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
