"""Candidate placement orders for a trace.

Row p of the result is a permutation of 0..n-1: the order in which plan p
feeds the requests to the placement rule.

* row 0  size-desc      key (-size, t_alloc, id)  -- large requests first so that
                        smaller ones can fill the intervals they leave (Sec. 5.1,
                        "Global Planning")
* row 1  lifetime-desc  key (-(t_free - t_alloc), -size, id)
* row 2  start-asc      key (t_alloc, id)  -- the order Algorithm 1 sorts by
* rows p >= 3, p odd    uniform random permutation
* rows p >= 3, p even   size-desc with a random order inside every equal-size
                        class and a jitter of up to one class to either side

Random rows are stable argsorts of 64-bit keys from the splitmix64 output
function applied to a counter, so any row can be regenerated on its own.
"""
from __future__ import annotations

import numpy as np

from .traces import Trace

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 output function on uint64 arrays (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = (x + _GOLD).astype(np.uint64)
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _row_keys(n: int, stream: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        base = _mix64(np.asarray([np.uint64(stream)], dtype=np.uint64))[0]
        ctr = np.arange(n, dtype=np.uint64) * np.uint64(0xD1342543DE82EF95) + base
    return _mix64(ctr)


def ordering_row(tr: Trace, p: int, seed: int = 1000) -> np.ndarray:
    n = tr.n
    ids = np.arange(n, dtype=np.int64)
    size = tr.size.astype(np.int64)
    ta = tr.t_alloc.astype(np.int64)
    tf = tr.t_free.astype(np.int64)
    if p == 0:
        row = np.lexsort((ids, ta, -size))
    elif p == 1:
        row = np.lexsort((ids, -size, -(tf - ta)))
    elif p == 2:
        row = np.lexsort((ids, ta))
    elif p % 2 == 1:
        row = np.argsort(_row_keys(n, seed + p), kind="stable")
    else:
        # class index by descending distinct size, plus a jitter in [-1, 1) classes
        distinct = np.unique(tr.size)[::-1]
        cls = np.searchsorted(-distinct.astype(np.int64), -size).astype(np.uint64)
        jitter = _row_keys(n, seed + p) >> np.uint64(31)          # 33 bits, [0, 2^33)
        key = ((cls + np.uint64(1)) << np.uint64(32)) + jitter      # (cls+1)*2^32 + [0, 2^33) - offset folded in
        row = np.argsort(key, kind="stable")
    return row.astype(np.uint32)


def make_orderings(tr: Trace, n_orderings: int, seed: int = 1000, rows=None) -> np.ndarray:
    """uint32 [P][n]; `rows` optionally selects a subset of plan indices."""
    plan_ids = list(range(n_orderings)) if rows is None else list(rows)
    out = np.empty((len(plan_ids), tr.n), dtype=np.uint32)
    for k, p in enumerate(plan_ids):
        out[k] = ordering_row(tr, p, seed)
    return out
