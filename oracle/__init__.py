"""ctypes front end of the CPU oracle (oracle/stalloc_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; it is used by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  It shares no code with the GPU library.

All functions take and return numpy arrays:
    size    uint64 [n]   bytes
    t_s/t_e uint32 [n]   half-open lifetime [t_s, t_e)   (Sec. 4, request event m)
    order   uint32 [n]   placement order (a permutation)
    a       uint64 [n]   start address per request       (Sec. 5.1, decision d)
"""
from __future__ import annotations

import contextlib
import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stalloc_oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")

STATUS = {0: "ok", 1: "invalid argument", 2: "bad trace", 3: "overflow", 4: "out of memory"}


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle status {code}: {STATUS.get(code, '?')}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (plain C99, no other dependencies)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", tmp, _SRC])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def _bind(path: str):
    lib = ctypes.CDLL(path)
    u32, u64 = ctypes.c_uint32, ctypes.c_uint64
    p = ctypes.c_void_p
    lib.oracle_check_trace.argtypes = [u32, u32, p, p, p]
    lib.oracle_plan_allpairs.argtypes = [u32, p, p, p, p, p, p]
    lib.oracle_conflict_lists.argtypes = [u32, p, p, p, p]
    lib.oracle_plan_lists.argtypes = [u32, p, p, p, p, p, p]
    lib.oracle_best_plan.argtypes = [u32, p, p]
    lib.oracle_fuse_groups.argtypes = [u32, p, p, p, u32, p, u32, p, p, p, p, p, p]
    lib.oracle_validate.argtypes = [u32, p, p, p, p, p, p]
    lib.oracle_lower_bound_definition.argtypes = [u32, u32, p, p, p, p, p]
    lib.oracle_lower_bound_sweep.argtypes = [u32, u32, p, p, p, p, p]
    lib.oracle_best_over_all_orders.argtypes = [u32, p, p, p, p, p]
    lib.oracle_exact_optimum.argtypes = [u32, p, p, p, p, p]
    lib.oracle_reusable_space.argtypes = [u32, p, p, p, p, u32, u32, u64, p, p, p]
    lib.oracle_memory_layers.argtypes = [u32, p, p, p, p, p, p, p, p]
    lib.oracle_make_orders.argtypes = [u32, p, p, p, u32, u32, u64, p]
    lib.oracle_splitmix64.argtypes = [u64]
    lib.oracle_splitmix64.restype = u64
    for name in ("oracle_check_trace", "oracle_plan_allpairs", "oracle_conflict_lists",
                 "oracle_plan_lists", "oracle_best_plan", "oracle_validate",
                 "oracle_lower_bound_definition", "oracle_lower_bound_sweep",
                 "oracle_best_over_all_orders", "oracle_exact_optimum", "oracle_reusable_space",
                 "oracle_memory_layers", "oracle_make_orders"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        _lib = _bind(_SO)
    return _lib


@contextlib.contextmanager
def use_library(path: str):
    """Route all calls to another build of the oracle source (used by the tests that
    plant mistakes in a copy of the source and expect the pins to catch them)."""
    global _lib
    old = _lib
    _lib = _bind(path)
    try:
        yield
    finally:
        _lib = old


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _check(rc: int) -> None:
    if rc != 0:
        raise OracleError(rc)


def check_trace(size, t_s, t_e, t_end: int) -> int:
    """Status code for the trace: 0 ok, 2 bad trace, 3 overflow."""
    size, t_s, t_e = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32)
    return int(_load().oracle_check_trace(len(size), int(t_end), _ptr(size), _ptr(t_s), _ptr(t_e)))


def plan_allpairs(size, t_s, t_e, order) -> Tuple[np.ndarray, int]:
    size, t_s, t_e, order = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32), _c(order, np.uint32)
    n = len(size)
    a = np.zeros(n, dtype=np.uint64)
    ext = np.zeros(1, dtype=np.uint64)
    _check(_load().oracle_plan_allpairs(n, _ptr(size), _ptr(t_s), _ptr(t_e), _ptr(order), _ptr(a), _ptr(ext)))
    return a, int(ext[0])


def conflict_lists(t_s, t_e) -> Tuple[np.ndarray, np.ndarray]:
    t_s, t_e = _c(t_s, np.uint32), _c(t_e, np.uint32)
    n = len(t_s)
    begin = np.zeros(n + 1, dtype=np.uint64)
    _check(_load().oracle_conflict_lists(n, _ptr(t_s), _ptr(t_e), _ptr(begin), None))
    nbr = np.zeros(max(int(begin[n]), 1), dtype=np.uint32)
    _check(_load().oracle_conflict_lists(n, _ptr(t_s), _ptr(t_e), _ptr(begin), _ptr(nbr)))
    return begin, nbr


def plan_lists(size, lists: Tuple[np.ndarray, np.ndarray], order) -> Tuple[np.ndarray, int]:
    size, order = _c(size, np.uint64), _c(order, np.uint32)
    begin, nbr = lists
    n = len(size)
    a = np.zeros(n, dtype=np.uint64)
    ext = np.zeros(1, dtype=np.uint64)
    _check(_load().oracle_plan_lists(n, _ptr(size), _ptr(begin), _ptr(nbr), _ptr(order), _ptr(a), _ptr(ext)))
    return a, int(ext[0])


def plan_many(size, t_s, t_e, orders, threads: int = 1, method: str = "allpairs",
              lists=None) -> Tuple[np.ndarray, np.ndarray]:
    """Every row of `orders` planned independently; returns (a [P][n], extent [P])."""
    orders = _c(orders, np.uint32)
    P, n = orders.shape
    a = np.zeros((P, n), dtype=np.uint64)
    ext = np.zeros(P, dtype=np.uint64)
    if method == "lists" and lists is None:
        lists = conflict_lists(t_s, t_e)

    def one(p: int) -> None:
        if method == "allpairs":
            a[p], ext[p] = plan_allpairs(size, t_s, t_e, orders[p])
        else:
            a[p], ext[p] = plan_lists(size, lists, orders[p])

    if threads <= 1:
        for p in range(P):
            one(p)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(one, range(P)))
    return a, ext


def best_plan(extent) -> int:
    extent = _c(extent, np.uint64)
    b = np.zeros(1, dtype=np.uint32)
    _check(_load().oracle_best_plan(len(extent), _ptr(extent), _ptr(b)))
    return int(b[0])


def validate(size, t_s, t_e, a) -> Tuple[int, Tuple[int, int]]:
    size, t_s, t_e, a = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32), _c(a, np.uint64)
    cnt = np.zeros(1, dtype=np.uint64)
    pair = np.zeros(2, dtype=np.uint32)
    _check(_load().oracle_validate(len(size), _ptr(size), _ptr(t_s), _ptr(t_e), _ptr(a), _ptr(cnt), _ptr(pair)))
    return int(cnt[0]), (int(pair[0]), int(pair[1]))


def lower_bound(size, t_s, t_e, t_end: int, method: str = "sweep") -> Tuple[int, int]:
    size, t_s, t_e = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32)
    lb = np.zeros(1, dtype=np.uint64)
    t_at = np.zeros(1, dtype=np.uint32)
    fn = _load().oracle_lower_bound_sweep if method == "sweep" else _load().oracle_lower_bound_definition
    _check(fn(len(size), int(t_end), _ptr(size), _ptr(t_s), _ptr(t_e), _ptr(lb), _ptr(t_at)))
    return int(lb[0]), int(t_at[0])


def best_over_all_orders(size, t_s, t_e) -> Tuple[int, np.ndarray]:
    size, t_s, t_e = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32)
    ext = np.zeros(1, dtype=np.uint64)
    order = np.zeros(len(size), dtype=np.uint32)
    _check(_load().oracle_best_over_all_orders(len(size), _ptr(size), _ptr(t_s), _ptr(t_e), _ptr(ext), _ptr(order)))
    return int(ext[0]), order


def exact_optimum(size, t_s, t_e) -> Tuple[int, np.ndarray]:
    size, t_s, t_e = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32)
    ext = np.zeros(1, dtype=np.uint64)
    a = np.zeros(len(size), dtype=np.uint64)
    _check(_load().oracle_exact_optimum(len(size), _ptr(size), _ptr(t_s), _ptr(t_e), _ptr(ext), _ptr(a)))
    return int(ext[0]), a


def reusable_space(size, t_s, t_e, a, window: Tuple[int, int], cap: Optional[int] = None) -> Tuple[np.ndarray, int, int]:
    """Idle address intervals of plan `a` throughout the window [w_lo, w_hi): (ranges [c][2], count, idle bytes)."""
    size, t_s, t_e, a = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32), _c(a, np.uint64)
    cap = len(size) + 1 if cap is None else int(cap)       # k met decisions leave at most k + 1 intervals
    ranges = np.zeros((cap, 2), dtype=np.uint64)
    count = np.zeros(1, dtype=np.uint64)
    idle = np.zeros(1, dtype=np.uint64)
    _check(_load().oracle_reusable_space(len(size), _ptr(size), _ptr(t_s), _ptr(t_e), _ptr(a), int(window[0]),
                                         int(window[1]), cap, _ptr(ranges), _ptr(count), _ptr(idle)))
    return ranges[:min(cap, int(count[0]))], int(count[0]), int(idle[0])


def memory_layers(size, t_s, t_e):
    """Algorithm 1 for every HomoSize group: (layer_of [n], layer_size [L], layer_t_s [L], layer_t_e [L])."""
    size, t_s, t_e = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32)
    n = len(size)
    layer_of = np.zeros(n, dtype=np.uint32)
    count = np.zeros(1, dtype=np.uint32)
    l_size = np.zeros(n, dtype=np.uint64)
    l_ts = np.zeros(n, dtype=np.uint32)
    l_te = np.zeros(n, dtype=np.uint32)
    _check(_load().oracle_memory_layers(n, _ptr(size), _ptr(t_s), _ptr(t_e), _ptr(layer_of), _ptr(count),
                                        _ptr(l_size), _ptr(l_ts), _ptr(l_te)))
    L = int(count[0])
    return layer_of, l_size[:L].copy(), l_ts[:L].copy(), l_te[:L].copy()


def tmp(size, t_s, t_e, a) -> float:
    """Time-memory product of a plan (Eq. 2, with the whole plan as the group D_g): the memory-time the
    requests use, sum of s * (t_e - t_s), over the memory-time the plan reserves, its extent max(a + s)
    times its span max(t_e) - min(t_s).  Exact integers, one rounding to double at the end."""
    from fractions import Fraction
    used = sum(int(s) * (int(e) - int(b)) for s, b, e in zip(size, t_s, t_e))
    extent = max(int(x) + int(s) for x, s in zip(a, size))
    span = max(int(e) for e in t_e) - min(int(b) for b in t_s)
    return float(Fraction(used, extent * span))


def fuse_groups(size, t_s, t_e, members1, members2):
    """Fusion of two HomoPhase groups (Sec. 5.1): -> dict with `order` (request numbers: the larger group's in
    packing order, then the smaller group's by allocation time), `a` (their addresses in the fused plan),
    `extent` [3] and `span` [3][2] of plan 1, plan 2 and the fused plan, `accepted` (bool)."""
    size, t_s, t_e = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32)
    m1, m2 = _c(members1, np.uint32), _c(members2, np.uint32)
    order = np.zeros(len(m1) + len(m2), dtype=np.uint32)
    a = np.zeros(len(m1) + len(m2), dtype=np.uint64)
    extent = np.zeros(3, dtype=np.uint64)
    span = np.zeros((3, 2), dtype=np.uint32)
    accepted = np.zeros(1, dtype=np.uint32)
    _check(_load().oracle_fuse_groups(len(size), _ptr(size), _ptr(t_s), _ptr(t_e), len(m1), _ptr(m1), len(m2), _ptr(m2),
                                      _ptr(order), _ptr(a), _ptr(extent), _ptr(span), _ptr(accepted)))
    return {"order": order, "a": a, "extent": extent, "span": span, "accepted": bool(accepted[0])}


def splitmix64(x: int) -> int:
    """Output of the SplitMix64 generator whose state before the step is x."""
    return int(_load().oracle_splitmix64(int(x) & 0xFFFFFFFFFFFFFFFF))


def make_orders(size, t_s, t_e, P: int, seed: int = 1000, first_plan: int = 0) -> np.ndarray:
    """Candidate placement orders first_plan .. first_plan + P - 1 as uint32 [P][n]."""
    size, t_s, t_e = _c(size, np.uint64), _c(t_s, np.uint32), _c(t_e, np.uint32)
    orders = np.zeros((P, len(size)), dtype=np.uint32)
    _check(_load().oracle_make_orders(len(size), _ptr(size), _ptr(t_s), _ptr(t_e), int(first_plan), int(P), int(seed),
                                      _ptr(orders)))
    return orders
