"""Seeded synthetic inputs: allocation traces, candidate placement orders and query windows.

This package only produces inputs (request rectangles, permutations, time windows).  It
holds no placement, validation or lower-bound arithmetic, so both the CPU
oracle's tests and the GPU path can draw the same arrays from it.
"""
from .traces import Trace, CONFIGS, make_trace, trace_stats
from .orderings import make_orderings, ordering_row
from .windows import make_windows

__all__ = ["Trace", "CONFIGS", "make_trace", "trace_stats", "make_orderings", "ordering_row",
           "make_windows"]
