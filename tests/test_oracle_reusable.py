"""Pins for the oracle's dynamic reusable space (Sec. 5.2): a hand-worked example, a byte-by-byte
occupancy map written independently in numpy, closed forms and invariants."""
import os

import numpy as np
import pytest

from helpers import GOLDEN_DIR, random_trace


def load_reusable_golden():
    dec, windows = [], []
    with open(os.path.join(GOLDEN_DIR, "reusable_space.txt")) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            key, rest = line.split(":", 1)
            if key == "dec":
                dec.append([int(x) for x in rest.split()])
            elif key == "window":
                w, idle = rest.split(";")
                lo, hi = (int(x) for x in w.split())
                v = [int(x) for x in idle.split()[1:]]
                windows.append(((lo, hi), np.asarray(v, np.uint64).reshape(-1, 2)))
    d = np.asarray(dec, np.int64)
    return (d[:, 0].astype(np.uint64), d[:, 1].astype(np.uint32), d[:, 2].astype(np.uint32),
            d[:, 3].astype(np.uint64), windows)


def idle_by_byte_map(size, ts, te, a, window):
    """One flag per byte of the pool; the idle intervals are the runs of clear flags."""
    size, a = np.asarray(size, np.int64), np.asarray(a, np.int64)
    lo, hi = int(a.min()), int((a + size).max())
    busy = np.zeros(hi - lo, dtype=bool)
    for i in range(len(size)):
        if int(ts[i]) < window[1] and window[0] < int(te[i]):
            busy[a[i] - lo:a[i] - lo + size[i]] = True
    edge = np.diff(np.concatenate([[True], busy, [True]]).astype(np.int8))
    starts = np.nonzero(edge == -1)[0] + lo
    ends = np.nonzero(edge == 1)[0] + lo
    return np.stack([starts, ends], axis=1).astype(np.uint64).reshape(-1, 2)


def test_hand_worked_windows(oracle):
    size, ts, te, a, windows = load_reusable_golden()
    for window, expect in windows:
        ranges, count, idle = oracle.reusable_space(size, ts, te, a, window)
        assert count == len(expect) and np.array_equal(ranges, expect), window
        assert idle == int((expect[:, 1] - expect[:, 0]).sum())


def random_plan(rng, n, pool):
    """Random decisions that need not form a valid plan: the definition only unions address ranges."""
    size = rng.integers(1, 9, n).astype(np.uint64)
    a = rng.integers(0, pool, n).astype(np.uint64)
    _, ts, te, t_end = random_trace(rng, n, t_max=20)
    return size, ts, te, a, t_end


@pytest.mark.parametrize("seed", range(12))
def test_matches_byte_map(oracle, seed):
    rng = np.random.default_rng(3000 + seed)
    n = [1, 2, 5, 17, 40, 90][seed % 6]
    size, ts, te, a, t_end = random_plan(rng, n, pool=[20, 200][seed % 2])
    for _ in range(25):
        lo = int(rng.integers(0, t_end))
        hi = int(rng.integers(lo + 1, t_end + 2))
        ranges, count, idle = oracle.reusable_space(size, ts, te, a, (lo, hi))
        expect = idle_by_byte_map(size, ts, te, a, (lo, hi))
        assert count == len(expect) and np.array_equal(ranges, expect), (seed, lo, hi)
        assert idle == int((expect[:, 1] - expect[:, 0]).sum())


def test_closed_forms(oracle):
    size = np.array([3, 5, 2], np.uint64)
    a = np.array([10, 20, 40], np.uint64)
    ts = np.array([0, 4, 8], np.uint32)
    te = np.array([4, 8, 12], np.uint32)
    # a window that meets nothing: the whole pool [10, 42)
    r, c, idle = oracle.reusable_space(size, ts, te, a, (12, 15))
    assert c == 1 and r.tolist() == [[10, 42]] and idle == 32
    # half-open on both sides: [4, 8) meets only the middle decision
    r, c, idle = oracle.reusable_space(size, ts, te, a, (4, 8))
    assert r.tolist() == [[10, 20], [25, 42]] and idle == 27
    # everything alive: the complement of the union; the pool starts at the lowest address, not at 0
    r, c, idle = oracle.reusable_space(size, ts, te, a, (0, 12))
    assert r.tolist() == [[13, 20], [25, 40]] and idle == 22
    # only the count is truncated by the capacity
    r, c, idle = oracle.reusable_space(size, ts, te, a, (0, 12), cap=1)
    assert c == 2 and r.tolist() == [[13, 20]] and idle == 22
    # a block inside another adds nothing; touching blocks leave no gap
    size = np.array([10, 2, 5], np.uint64)
    a = np.array([0, 3, 10], np.uint64)
    ts = np.zeros(3, np.uint32)
    te = np.full(3, 2, np.uint32)
    r, c, idle = oracle.reusable_space(size, ts, te, a, (0, 1))
    assert c == 0 and idle == 0


@pytest.mark.parametrize("seed", range(6))
def test_lowest_fit_plans_have_no_idle_space_over_the_whole_iteration(oracle, seed):
    """The address ranges of a lowest-fit plan, taken together, are a gap-free prefix (a lowest fit always
    touches a block below it), so over the whole iteration nothing is reusable; and whatever is idle in
    a window is idle in every window inside it."""
    rng = np.random.default_rng(3100 + seed)
    n = 60
    size, ts, te, t_end = random_trace(rng, n, t_max=30)
    a, extent = oracle.plan_allpairs(size, ts, te, rng.permutation(n).astype(np.uint32))
    _, count, idle = oracle.reusable_space(size, ts, te, a, (0, t_end))
    assert count == 0 and idle == 0
    outer = (3, 20)
    inner = (7, 12)
    _, _, idle_outer = oracle.reusable_space(size, ts, te, a, outer)
    r_in, _, idle_inner = oracle.reusable_space(size, ts, te, a, inner)
    assert idle_inner >= idle_outer
    # every idle interval is free of the decisions that meet the window, and cannot be extended
    met = [(int(a[i]), int(a[i] + size[i])) for i in range(n) if ts[i] < inner[1] and inner[0] < te[i]]
    for lo, hi in r_in.tolist():
        assert all(e <= lo or s >= hi for s, e in met)
        assert lo == 0 or any(s < lo <= e for s, e in met)
        assert hi == extent or any(s <= hi < e for s, e in met)
