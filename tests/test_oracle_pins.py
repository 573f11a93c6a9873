"""Pins of the CPU oracle against things that do not come from the oracle:
hand-worked fixtures, closed forms, Algorithm 1's layer count, exhaustive and
exact searches on tiny traces, and re-derivations written with numpy only."""
import itertools
import os

import numpy as np
import pytest

from helpers import (check_lowest_fit, count_conflicts, count_conflicts_fast, load_golden,
                     max_live_numpy, random_trace)
from workloads import make_orderings, make_trace

GOLDEN = ["running_max.txt", "hole_and_tie.txt", "gap_fit.txt"]


@pytest.mark.parametrize("name", GOLDEN)
@pytest.mark.parametrize("method", ["allpairs", "lists"])
def test_hand_worked_examples(oracle, name, method):
    g = load_golden(name)
    for case in g["cases"]:
        a, ext = oracle.plan_many(g["size"], g["t_s"], g["t_e"], np.asarray([case["order"]], np.uint32),
                                  method=method)
        assert a[0].tolist() == case["a"]
        assert int(ext[0]) == case["extent"]
        assert oracle.validate(g["size"], g["t_s"], g["t_e"], a[0]) == (0, (0xFFFFFFFF, 0xFFFFFFFF))
    for method_lb in ("definition", "sweep"):
        assert oracle.lower_bound(g["size"], g["t_s"], g["t_e"], g["t_end"], method_lb) == g["max_live"]


def test_time_clique_gives_prefix_sums(oracle):
    """All lifetimes conflict: nothing can share addresses, so each request sits on top of
    all earlier ones and the extent is the sum of sizes, for every order."""
    rng = np.random.default_rng(1)
    n = 40
    size = rng.integers(1, 1000, n).astype(np.uint64)
    ts = rng.integers(0, 10, n).astype(np.uint32)
    te = (20 + rng.integers(0, 10, n)).astype(np.uint32)
    for _ in range(5):
        order = rng.permutation(n).astype(np.uint32)
        for plan in (oracle.plan_allpairs(size, ts, te, order),
                     oracle.plan_lists(size, oracle.conflict_lists(ts, te), order)):
            a, ext = plan
            expect = np.zeros(n, dtype=np.uint64)
            expect[order] = np.concatenate([[0], np.cumsum(size[order])[:-1]]).astype(np.uint64)
            assert np.array_equal(a, expect)
            assert ext == int(size.sum())
    assert oracle.lower_bound(size, ts, te, 30)[0] == int(size.sum())


def test_time_disjoint_all_at_zero(oracle):
    rng = np.random.default_rng(2)
    n = 30
    size = rng.integers(1, 1000, n).astype(np.uint64)
    ts = (np.arange(n) * 3).astype(np.uint32)
    te = ts + np.uint32(3)          # touching lifetimes: released at the next one's allocation
    order = rng.permutation(n).astype(np.uint32)
    a, ext = oracle.plan_allpairs(size, ts, te, order)
    assert not a.any() and ext == int(size.max())
    a, ext = oracle.plan_lists(size, oracle.conflict_lists(ts, te), order)
    assert not a.any() and ext == int(size.max())
    assert oracle.lower_bound(size, ts, te, 3 * n)[0] == int(size.max())


def _memory_layers(ts, te):
    """Algorithm 1 (Memory-Layer Construction): requests of one size sorted by allocation
    time; each goes to the layer whose last release is the latest one before its allocation,
    else opens a new layer.  Returns the number of layers."""
    ends = []
    for i in np.argsort(ts, kind="stable"):
        fitting = [k for k, e in enumerate(ends) if e < ts[i]]
        if fitting:
            k = max(fitting, key=lambda q: ends[q])
            ends[k] = te[i]
        else:
            ends.append(te[i])
    return len(ends)


@pytest.mark.parametrize("seed", range(6))
def test_equal_sizes_start_order_reaches_layer_count(oracle, seed):
    """One size S, requests fed by allocation time: the lowest-address rule needs exactly
    S x (number of memory-layers of Algorithm 1) = S x (max simultaneously live) bytes,
    the minimum Sec. 5.1 'HomoSize Group Planning' aims at."""
    rng = np.random.default_rng(seed)
    n, S = 200, 4096
    _, ts, te, t_end = random_trace(rng, n, unique_times=True)
    size = np.full(n, S, dtype=np.uint64)
    order = np.argsort(ts, kind="stable").astype(np.uint32)
    a, ext = oracle.plan_allpairs(size, ts, te, order)
    layers = _memory_layers(ts.astype(np.int64), te.astype(np.int64))
    live = max_live_numpy(size, ts, te, t_end)[0]
    assert ext == S * layers == live
    assert oracle.lower_bound(size, ts, te, t_end)[0] == live
    assert set((a // np.uint64(S)).tolist()) == set(range(layers))


def test_stack_discipline_reaches_lower_bound(oracle):
    """Scoped tensors allocated in order and released in reverse order (Sec. 2.3, temporal
    regularity): fed by allocation time each request lands at the current stack depth."""
    rng = np.random.default_rng(3)
    size, ts, te, depth_at = [], [], [], []
    stack, t, depth = [], 0, 0
    for _ in range(400):
        if stack and rng.random() < 0.45:
            i = stack.pop(); te[i] = t; depth -= size[i]
        else:
            s = int(rng.integers(1, 50)) * 512
            stack.append(len(size)); size.append(s); ts.append(t); te.append(-1)
            depth_at.append(depth); depth += s
        t += 1
    while stack:
        i = stack.pop(); te[i] = t; t += 1
    size = np.asarray(size, np.uint64); ts = np.asarray(ts, np.uint32); te = np.asarray(te, np.uint32)
    order = np.arange(len(size), dtype=np.uint32)
    a, ext = oracle.plan_allpairs(size, ts, te, order)
    assert a.tolist() == depth_at
    assert ext == oracle.lower_bound(size, ts, te, t)[0] == max_live_numpy(size, ts, te, t)[0]


@pytest.mark.parametrize("seed", range(25))
def test_all_orders_reach_exact_optimum(oracle, seed):
    """n <= 6: the best extent over all n! orders equals the optimum found by a search that
    uses no placement order at all; and max-live <= optimum <= any plan's extent."""
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(2, 7))
    size, ts, te, t_end = random_trace(rng, n, t_max=6)
    best_ext, best_order = oracle.best_over_all_orders(size, ts, te)
    opt, opt_a = oracle.exact_optimum(size, ts, te)
    assert best_ext == opt
    assert count_conflicts(size, ts, te, opt_a)[0] == 0
    lb = oracle.lower_bound(size, ts, te, t_end, "definition")[0]
    assert lb <= opt
    a, ext = oracle.plan_allpairs(size, ts, te, best_order)
    assert ext == best_ext
    check_lowest_fit(size, ts, te, best_order, a)


@pytest.mark.parametrize("seed", range(4))
def test_exhaustive_orders_n8_bounds(oracle, seed):
    rng = np.random.default_rng(200 + seed)
    n = 8
    size, ts, te, t_end = random_trace(rng, n, t_max=8)
    best_ext, _ = oracle.best_over_all_orders(size, ts, te)
    lb = oracle.lower_bound(size, ts, te, t_end)[0]
    assert lb <= best_ext <= int(size.sum())
    # python enumeration of the same n! orders on a sample: none beats the reported best
    perms = list(itertools.permutations(range(n)))
    for k in rng.choice(len(perms), size=200, replace=False):
        order = np.asarray(perms[k], np.uint32)
        a, ext = oracle.plan_allpairs(size, ts, te, order)
        assert ext >= best_ext
        assert count_conflicts(size, ts, te, a)[0] == 0


@pytest.mark.parametrize("seed", range(20))
@pytest.mark.parametrize("unique_times", [False, True])
def test_random_traces_valid_and_minimal(oracle, seed, unique_times):
    rng = np.random.default_rng(300 + seed)
    n = int(rng.integers(1, 60))
    size, ts, te, t_end = random_trace(rng, n, t_max=20, unique_times=unique_times)
    lists = oracle.conflict_lists(ts, te)
    lb = max_live_numpy(size, ts, te, t_end)
    assert oracle.lower_bound(size, ts, te, t_end, "definition") == lb
    assert oracle.lower_bound(size, ts, te, t_end, "sweep") == lb
    for _ in range(3):
        order = rng.permutation(n).astype(np.uint32)
        a, ext = oracle.plan_allpairs(size, ts, te, order)
        a2, ext2 = oracle.plan_lists(size, lists, order)
        assert np.array_equal(a, a2) and ext == ext2
        assert ext == int((a + size).max())
        assert count_conflicts(size, ts, te, a) == (0, (0xFFFFFFFF, 0xFFFFFFFF))
        assert oracle.validate(size, ts, te, a) == (0, (0xFFFFFFFF, 0xFFFFFFFF))
        check_lowest_fit(size, ts, te, order, a)
        assert lb[0] <= ext <= int(size.sum())


@pytest.mark.parametrize("seed", range(10))
def test_validate_counts_planted_conflicts(oracle, seed):
    """Corrupt a valid plan by moving blocks onto lifetime-conflicting neighbours; the count
    and the first pair must match a direct evaluation of Sec. 5.1's constraint."""
    rng = np.random.default_rng(400 + seed)
    n = 50
    size, ts, te, _ = random_trace(rng, n, t_max=15)
    a, _ = oracle.plan_allpairs(size, ts, te, rng.permutation(n).astype(np.uint32))
    bad = a.copy()
    for i in rng.choice(n, size=int(rng.integers(1, 6)), replace=False):
        bad[i] = rng.integers(0, int(a.max()) + 1)
    want = count_conflicts(size, ts, te, bad)
    assert oracle.validate(size, ts, te, bad) == want
    assert count_conflicts_fast(size, ts, te, bad) == want[0]


def test_validate_known_single_conflict(oracle):
    size = np.asarray([4, 4, 4], np.uint64)
    ts = np.asarray([0, 0, 5], np.uint32); te = np.asarray([5, 5, 9], np.uint32)
    assert oracle.validate(size, ts, te, np.asarray([0, 4, 0], np.uint64)) == (0, (0xFFFFFFFF, 0xFFFFFFFF))
    assert oracle.validate(size, ts, te, np.asarray([0, 3, 0], np.uint64)) == (1, (0, 1))
    assert oracle.validate(size, ts, te, np.asarray([0, 0, 0], np.uint64)) == (1, (0, 1))


def test_best_plan_prefers_lowest_index(oracle):
    assert oracle.best_plan(np.asarray([9, 7, 8, 7, 7], np.uint64)) == 1
    assert oracle.best_plan(np.asarray([5], np.uint64)) == 0


def test_check_trace_rejects_degenerate_requests(oracle):
    ok = (np.asarray([1, 2], np.uint64), np.asarray([0, 1], np.uint32), np.asarray([1, 3], np.uint32))
    assert oracle.check_trace(*ok, 3) == 0
    assert oracle.check_trace(np.asarray([1, 0], np.uint64), ok[1], ok[2], 3) == 2
    assert oracle.check_trace(ok[0], np.asarray([0, 3], np.uint32), ok[2], 3) == 2
    assert oracle.check_trace(*ok, 2) == 2
    assert oracle.check_trace(np.asarray([2 ** 62, 2 ** 62], np.uint64), ok[1], ok[2], 3) == 3


def test_lists_equal_allpairs_on_configs(oracle):
    tr = make_trace(1)
    orders = make_orderings(tr, 64)
    a1, e1 = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, method="allpairs")
    a2, e2 = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, method="lists")
    assert np.array_equal(a1, a2) and np.array_equal(e1, e2)
    lb = oracle.lower_bound(tr.size, tr.t_alloc, tr.t_free, tr.t_end)[0]
    assert lb == max_live_numpy(tr.size, tr.t_alloc, tr.t_free, tr.t_end)[0]
    assert (e1 >= lb).all()
    for p in (0, 1, 2, 3, 4):
        check_lowest_fit(tr.size, tr.t_alloc, tr.t_free, orders[p], a1[p])

    tr = make_trace(2)
    rows = [0, 1, 2, 3, 4, 513, 1022, 1023]
    orders = make_orderings(tr, 1024, rows=rows)
    a1, e1 = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=4, method="allpairs")
    for k in range(len(rows)):
        assert count_conflicts_fast(tr.size, tr.t_alloc, tr.t_free, a1[k]) == 0
        assert int(e1[k]) == int((a1[k] + tr.size).max())


def test_lists_equal_allpairs_on_every_order_of_config_2_and_sampled_orders_of_config_3(oracle):
    """The conflict-list oracle, which the comparisons on the larger configurations rest on, against the
    all-pairs oracle: all 1024 orders of config 2, and eight orders of config 3 (the three heuristic
    rows, uniform permutations and rows sorted by size with jitter)."""
    threads = min(8, os.cpu_count() or 1)
    tr = make_trace(2)
    orders = make_orderings(tr, 1024)
    lists = oracle.conflict_lists(tr.t_alloc, tr.t_free)
    for r0 in range(0, 1024, 256):                      # in four parts: 50 MB of addresses at a time
        part = orders[r0:r0 + 256]
        a1, e1 = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, part, threads=threads, method="allpairs")
        a2, e2 = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, part, threads=threads, method="lists", lists=lists)
        assert np.array_equal(a1, a2) and np.array_equal(e1, e2), f"rows {r0}..{r0 + 255}"
    tr = make_trace(3)
    rows = [0, 1, 2, 3, 4, 1025, 2046, 2047]
    orders = make_orderings(tr, 2048, rows=rows)
    a1, e1 = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=threads, method="allpairs")
    a2, e2 = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=threads, method="lists")
    assert np.array_equal(a1, a2) and np.array_equal(e1, e2)
