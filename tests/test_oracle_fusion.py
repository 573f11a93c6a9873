"""Pins of the oracle's fusion of two HomoPhase groups (Sec. 5.1, HomoPhase Group Planning): a hand-worked
fixture, closed forms, invariants of the fused plan and the equivalence of its integer accept test with
the time-memory products of Eq. 2."""
import os
from fractions import Fraction

import numpy as np
import pytest

from helpers import GOLDEN_DIR, count_conflicts


def load_cases():
    size, ts, te, cases = [], [], [], []
    for raw in open(os.path.join(GOLDEN_DIR, "fusion.txt")):
        line = raw.split("#", 1)[0].strip()
        if not line:
            continue
        key, rest = line.split(":", 1)
        if key == "req":
            s, a, b = (int(x) for x in rest.split())
            size.append(s); ts.append(a); te.append(b)
        else:
            parts = {p.split()[0]: p.split()[1:] for p in rest.split(";")}
            cases.append({"g1": [int(x) for x in parts["g1"]], "g2": [int(x) for x in parts["g2"]],
                          "plan": {int(x.split(":")[0]): int(x.split(":")[1]) for x in parts["plan"]},
                          "extents": [int(x) for x in parts["extents"]], "accepted": bool(int(parts["accepted"][0]))})
    return np.asarray(size, np.uint64), np.asarray(ts, np.uint32), np.asarray(te, np.uint32), cases


def test_hand_worked_fusions(oracle):
    size, ts, te, cases = load_cases()
    assert len(cases) == 4
    for c in cases:
        got = oracle.fuse_groups(size, ts, te, c["g1"], c["g2"])
        assert dict(zip(got["order"].tolist(), got["a"].tolist())) == c["plan"]
        assert got["extent"].tolist() == c["extents"] and got["accepted"] == c["accepted"]


def tmp_of(size, ts, te, ids, a):
    """Eq. 2 for the decisions `ids` at addresses `a`, as an exact fraction."""
    used = sum(int(size[i]) * (int(te[i]) - int(ts[i])) for i in ids)
    extent = max(int(x) + int(size[i]) for i, x in zip(ids, a))
    span = max(int(te[i]) for i in ids) - min(int(ts[i]) for i in ids)
    return Fraction(used, extent * span), extent * span, used


def random_groups(rng, n1, n2, overlap):
    """Group 1 allocated in [0, 20), released in [40, 60); group 2 allocated from 60 - overlap on."""
    n = n1 + n2
    size = rng.integers(1, 9, n).astype(np.uint64) * np.uint64(rng.choice([1, 512]))
    ts = np.concatenate([rng.integers(0, 20, n1), rng.integers(60 - overlap, 80 - overlap, n2)])
    te = np.concatenate([rng.integers(40, 60, n1), rng.integers(100, 120, n2)])
    return size, ts.astype(np.uint32), te.astype(np.uint32), np.arange(n1), np.arange(n1, n)


@pytest.mark.parametrize("seed", range(12))
def test_fused_plans_are_valid_and_the_accept_test_is_the_tmp_test(oracle, seed):
    rng = np.random.default_rng(4100 + seed)
    size, ts, te, g1, g2 = random_groups(rng, int(rng.integers(1, 40)), int(rng.integers(1, 40)), int(rng.choice([0, 5, 15, 30])))
    got = oracle.fuse_groups(size, ts, te, g1, g2)
    order, a = got["order"], got["a"]
    assert sorted(order.tolist()) == sorted(g1.tolist() + g2.tolist())             # every request once
    assert count_conflicts(size[order], ts[order], te[order], a)[0] == 0            # the constraint of Sec. 5.1
    ext = [int(size[g].astype(np.int64).sum()) for g in (g1, g2)]
    assert got["extent"][:2].tolist() == ext                                        # contiguous local plans
    assert int(got["extent"][2]) == int((a + size[order]).max())
    assert max(ext) <= int(got["extent"][2]) <= sum(ext)
    # the larger plan: packed from 0, latest release first
    nl = len(g1) if ext[0] >= ext[1] else len(g2)
    large = order[:nl]
    assert sorted(large.tolist()) == sorted((g1 if ext[0] >= ext[1] else g2).tolist())
    assert (np.diff(te[large].astype(np.int64)) <= 0).all()
    assert a[:nl].tolist() == np.concatenate([[0], np.cumsum(size[large])[:-1]]).tolist()
    # the smaller plan: listed by allocation time; each sits on a start address of the larger plan,
    # on the end of another of its requests, or (left over) on top
    small = order[nl:]
    assert (np.diff(ts[small].astype(np.int64)) >= 0).all()
    spots = set(a[:nl].tolist()) | set((a[nl:] + size[small]).tolist()) | {int((a[:nl] + size[large]).max())}
    assert all(int(x) in spots for x in a[nl:])
    # Eq. 2: accepted iff the fused product exceeds the average of the two weighted by reserved memory-time
    t1, r1, u1 = tmp_of(size, ts, te, g1, np.concatenate([[0], np.cumsum(size[g1])[:-1]]))
    t2, r2, u2 = tmp_of(size, ts, te, g2, np.concatenate([[0], np.cumsum(size[g2])[:-1]]))
    tf, rf, uf = tmp_of(size, ts, te, order, a)
    assert uf == u1 + u2
    assert got["accepted"] == (tf > (t1 * r1 + t2 * r2) / (r1 + r2))
    assert abs(float(tf) - oracle.tmp(size[order], ts[order], te[order], a)) < 1e-12


def test_closed_forms(oracle):
    rng = np.random.default_rng(7)
    size = rng.integers(1, 20, 30).astype(np.uint64)
    g1, g2 = np.arange(18), np.arange(18, 30)
    # one common lifetime: everything conflicts, nothing fits at any start address, the plans end up
    # stacked, the reserved memory-time is unchanged and the fusion is rejected
    ts, te = np.full(30, 3, np.uint32), np.full(30, 9, np.uint32)
    got = oracle.fuse_groups(size, ts, te, g1, g2)
    s1, s2 = int(size[g1].sum()), int(size[g2].sum())
    assert int(got["extent"][2]) == s1 + s2 and not got["accepted"]
    nl = 18 if s1 >= s2 else 12
    assert got["a"][nl:].tolist() == (max(s1, s2) + np.concatenate([[0], np.cumsum(size[got["order"][nl:]])[:-1]])).tolist()
    # the second group lives after the first: it is packed from 0 inside the larger plan's range
    ts = np.concatenate([np.zeros(18), np.arange(10, 22)]).astype(np.uint32)
    te = np.concatenate([np.full(18, 10), np.full(12, 30)]).astype(np.uint32)
    got = oracle.fuse_groups(size, ts, te, g1, g2)
    assert int(got["extent"][2]) == max(s1, s2)
    small = got["order"][nl:]
    assert got["a"][nl:].tolist() == np.concatenate([[0], np.cumsum(size[small])[:-1]]).tolist()
    # equal extents and adjacent, equally long spans: reserved memory-time equal, so not accepted (no increase)
    size2 = np.asarray([5, 5], np.uint64)
    got = oracle.fuse_groups(size2, np.asarray([0, 4], np.uint32), np.asarray([4, 8], np.uint32), [0], [1])
    assert got["a"].tolist() == [0, 0] and not got["accepted"]


def test_first_placement_is_the_earliest_request_that_fits_at_the_lowest_start_address(oracle):
    """Re-derived from the text for the first step only: walk the larger plan's start addresses upwards;
    at the first one where any request of the smaller plan conflicts with nothing, the earliest such
    request (request number among equals) is placed."""
    for seed in range(10):
        rng = np.random.default_rng(4200 + seed)
        size, ts, te, g1, g2 = random_groups(rng, int(rng.integers(2, 30)), int(rng.integers(2, 30)), int(rng.choice([5, 15, 30])))
        got = oracle.fuse_groups(size, ts, te, g1, g2)
        ext = [int(size[g].astype(np.int64).sum()) for g in (g1, g2)]
        nl = len(g1) if ext[0] >= ext[1] else len(g2)
        large, a_large, small = got["order"][:nl], got["a"][:nl], got["order"][nl:]
        want = None
        for addr in sorted(set(a_large.tolist())):
            fits = [j for j in small
                    if not any(ts[i] < te[j] and ts[j] < te[i] and x < addr + size[j] and addr < x + size[i]
                               for i, x in zip(large, a_large))]
            if fits:
                want = (min(fits, key=lambda j: (int(ts[j]), int(j))), addr)
                break
        placed = dict(zip(small.tolist(), got["a"][nl:].tolist()))
        if want is None:
            assert min(placed.values()) >= int((a_large + size[large]).max())           # all left over, on top
        else:
            assert placed[int(want[0])] == want[1]
