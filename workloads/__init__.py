"""Seeded synthetic inputs (layouts, compute times, gradients) shared by the CPU oracle's
tests and the GPU path's tests and benchmark.  Holds none of the method's arithmetic."""
from . import grads, shapes, times  # noqa: F401
