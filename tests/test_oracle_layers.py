"""Pins of the oracle's memory-layer construction (Sec. 5.1, Algorithm 1): a hand-worked example,
the textbook optimum of interval partitioning (as many layers as requests of that size are ever
alive at once), structural invariants, closed forms, and that the layers planned as single
requests expand to a conflict-free plan."""
import os

import numpy as np
import pytest

from helpers import random_trace

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_layers_golden():
    req, layers, layer_of = [], [], None
    with open(os.path.join(GOLDEN_DIR, "memory_layers.txt")) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            key, rest = line.split(":", 1)
            vals = [int(x) for x in rest.split()]
            if key == "req":
                req.append(vals)
            elif key == "layer":
                layers.append(vals)
            elif key == "layer_of":
                layer_of = vals
    r = np.asarray(req, np.int64)
    return (r[:, 0].astype(np.uint64), r[:, 1].astype(np.uint32), r[:, 2].astype(np.uint32),
            np.asarray(layer_of, np.uint32), np.asarray(layers, np.int64))


def max_alive(ts, te):
    """Largest number of lifetimes [ts, te) containing one instant, by looking at every instant."""
    if len(ts) == 0:
        return 0
    return max(int(((ts <= t) & (t < te)).sum()) for t in range(int(ts.min()), int(te.max())))


def check_structure(size, ts, te, layer_of, l_size, l_ts, l_te):
    n, L = len(size), len(l_size)
    assert sorted(set(layer_of.tolist())) == list(range(L))                 # every layer is used, numbering is dense
    assert (np.diff(l_size.astype(np.int64)) <= 0).all()                    # groups in descending size
    for l in range(L):
        members = np.nonzero(layer_of == l)[0]
        assert (size[members] == l_size[l]).all()
        order = members[np.lexsort((members, ts[members]))]
        assert (te[order][:-1] <= ts[order][1:]).all()                      # no two members alive at once
        assert int(l_ts[l]) == int(ts[order[0]]) and int(l_te[l]) == int(te[order[-1]])
    for s in np.unique(size):
        grp = size == s
        assert len(set(layer_of[grp].tolist())) == max_alive(ts[grp].astype(np.int64), te[grp].astype(np.int64))
        ids = sorted(set(layer_of[grp].tolist()))
        assert ids == list(range(ids[0], ids[0] + len(ids)))                # a group's layers are numbered in a row
        # opened in the order of their first requests
        firsts = [(int(l_ts[l]), int(np.nonzero((layer_of == l) & (ts == l_ts[l]))[0].min())) for l in ids]
        assert firsts == sorted(firsts)


def test_hand_worked_example(oracle):
    size, ts, te, want_of, want_layers = load_layers_golden()
    layer_of, l_size, l_ts, l_te = oracle.memory_layers(size, ts, te)
    assert np.array_equal(layer_of, want_of)
    assert np.array_equal(np.stack([l_size.astype(np.int64), l_ts, l_te], axis=1), want_layers)
    check_structure(size, ts, te, layer_of, l_size, l_ts, l_te)


@pytest.mark.parametrize("seed", range(12))
def test_random_traces_structure_and_minimum(oracle, seed):
    rng = np.random.default_rng(8100 + seed)
    n = int(rng.integers(1, 160))
    size, ts, te, _ = random_trace(rng, n, t_max=max(4, n // 3), unique_times=(seed % 3 == 0), sizes=[8, 16, 16, 24, 512])
    layer_of, l_size, l_ts, l_te = oracle.memory_layers(size, ts, te)
    check_structure(size, ts, te, layer_of, l_size, l_ts, l_te)


def test_closed_forms(oracle):
    n = 9
    one = np.full(n, 64, np.uint64)
    # all alive together: one layer each, in order of allocation
    ts, te = np.arange(n, dtype=np.uint32), np.full(n, 20, np.uint32)
    layer_of, l_size, _, _ = oracle.memory_layers(one, ts, te)
    assert np.array_equal(layer_of, np.arange(n)) and len(l_size) == n
    # back to back: one layer holds them all
    ts, te = np.arange(n, dtype=np.uint32) * 2, np.arange(n, dtype=np.uint32) * 2 + 2
    layer_of, l_size, l_ts, l_te = oracle.memory_layers(one, ts, te)
    assert not layer_of.any() and len(l_size) == 1 and (int(l_ts[0]), int(l_te[0])) == (0, 2 * n)
    # all sizes distinct: every request is its own layer, numbered by descending size
    size = np.asarray([5, 9, 1, 7], np.uint64)
    layer_of, l_size, _, _ = oracle.memory_layers(size, np.zeros(4, np.uint32), np.ones(4, np.uint32))
    assert layer_of.tolist() == [2, 0, 3, 1] and l_size.tolist() == [9, 7, 5, 1]
    # two layers in turn: a request takes the layer that was released last, not the first one
    size = np.full(4, 8, np.uint64)
    ts, te = np.asarray([0, 0, 5, 5], np.uint32), np.asarray([1, 3, 6, 6], np.uint32)
    layer_of, *_ = oracle.memory_layers(size, ts, te)
    assert layer_of.tolist() == [0, 1, 1, 0]
    # two layers released at the same instant: the one opened first is taken first
    ts, te = np.asarray([0, 0, 5, 5], np.uint32), np.asarray([3, 3, 6, 6], np.uint32)
    layer_of, *_ = oracle.memory_layers(size, ts, te)
    assert layer_of.tolist() == [0, 1, 0, 1]


@pytest.mark.parametrize("seed", range(6))
def test_layers_planned_as_requests_expand_to_a_valid_plan(oracle, seed):
    """Local plan of a group = its layers stacked; planned as single requests (size, first allocation,
    last release) by the placement rule, every request inherits its layer's address: no conflicts, and
    the extent is the extent of the layer plan."""
    rng = np.random.default_rng(8200 + seed)
    n = int(rng.integers(2, 120))
    size, ts, te, _ = random_trace(rng, n, t_max=max(4, n // 2), sizes=[8, 16, 24])
    layer_of, l_size, l_ts, l_te = oracle.memory_layers(size, ts, te)
    L = len(l_size)
    a_layer, extent = oracle.plan_allpairs(l_size, l_ts, l_te, np.arange(L, dtype=np.uint32))
    a = a_layer[layer_of]
    conflicts, _ = oracle.validate(size, ts, te, a)
    assert conflicts == 0 and int((a + size).max()) == int(extent)
