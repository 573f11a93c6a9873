"""Pins of the oracle's time-memory product (Eq. 2): closed forms, the area bound for plans without
conflicts, invariance under shifts of time and address units, and the identity with Eq. 1's efficiency
when every request lives through the whole span."""
from fractions import Fraction

import numpy as np
import pytest

from helpers import random_trace


def test_closed_forms(oracle):
    u64, u32 = np.uint64, np.uint32
    # one request fills its own rectangle
    assert oracle.tmp(np.array([7], u64), np.array([3], u32), np.array([9], u32), np.array([0], u64)) == 1.0
    # two requests of one lifetime stacked: still full; side by side in time at one address: full
    s, a = np.array([4, 4], u64), np.array([0, 4], u64)
    assert oracle.tmp(s, np.array([0, 0], u32), np.array([5, 5], u32), a) == 1.0
    assert oracle.tmp(s, np.array([0, 5], u32), np.array([5, 10], u32), np.array([0, 0], u64)) == 1.0
    # the same two one after the other but stacked: half of the reserved rectangle is a bubble
    assert oracle.tmp(s, np.array([0, 5], u32), np.array([5, 10], u32), a) == 0.5
    # 2 x [0,3) at 0 and 1 x [1,2) at 5: used 6 + 1, reserved 6 x 3
    got = oracle.tmp(np.array([2, 1], u64), np.array([0, 1], u32), np.array([3, 2], u32), np.array([0, 5], u64))
    assert got == float(Fraction(7, 18))
    # a plan that starts above address 0 reserves everything below as well (Eq. 2 takes max(a + s))
    assert oracle.tmp(np.array([4], u64), np.array([0], u32), np.array([2], u32), np.array([12], u64)) == 0.25


@pytest.mark.parametrize("seed", range(8))
def test_area_bound_and_invariances(oracle, seed):
    rng = np.random.default_rng(8300 + seed)
    n = int(rng.integers(2, 80))
    size, ts, te, _ = random_trace(rng, n, t_max=max(4, n // 2), unique_times=(seed % 2 == 1))
    a, extent = oracle.plan_allpairs(size, ts, te, rng.permutation(n).astype(np.uint32))
    t = oracle.tmp(size, ts, te, a)
    assert 0.0 < t <= 1.0                                   # rectangles without conflicts fit the reserved one
    assert oracle.tmp(size, ts + np.uint32(1000), te + np.uint32(1000), a) == t          # shift of the time origin
    assert oracle.tmp(size * np.uint64(4096), ts, te, a * np.uint64(4096)) == t          # change of the byte unit
    assert oracle.tmp(size, ts * np.uint32(3), te * np.uint32(3), a) == t                # change of the time unit
    # used memory-time = sum over instants of the live bytes, counted instant by instant
    used = sum(int(size[(ts <= x) & (x < te)].sum()) for x in range(int(ts.min()), int(te.max())))
    assert t == float(Fraction(used, int(extent) * (int(te.max()) - int(ts.min()))))


def test_equals_efficiency_when_everything_lives_through_the_span(oracle):
    rng = np.random.default_rng(8400)
    n = 20
    size = rng.integers(1, 50, n).astype(np.uint64)
    ts, te = np.zeros(n, np.uint32), np.full(n, 9, np.uint32)
    a, extent = oracle.plan_allpairs(size, ts, te, np.arange(n, dtype=np.uint32))
    lb, _ = oracle.lower_bound(size, ts, te, 9)
    assert oracle.tmp(size, ts, te, a) == lb / int(extent) == 1.0
