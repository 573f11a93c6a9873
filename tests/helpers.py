"""Independent checks used by the tests (numpy only; no oracle, no GPU code)."""
from __future__ import annotations

import os
from typing import Dict, List

import numpy as np

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_golden(name: str) -> Dict:
    size, ts, te, cases = [], [], [], []
    max_live = None
    with open(os.path.join(GOLDEN_DIR, name)) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            key, rest = line.split(":", 1)
            if key == "req":
                s, a, b = (int(x) for x in rest.split())
                size.append(s); ts.append(a); te.append(b)
            elif key == "case":
                parts = [p.strip().split() for p in rest.split(";")]
                d = {p[0]: [int(x) for x in p[1:]] for p in parts}
                cases.append({"order": d["order"], "a": d["a"], "extent": d["extent"][0]})
            elif key == "max_live":
                v, t = (int(x) for x in rest.split())
                max_live = (v, t)
    return {"size": np.asarray(size, np.uint64), "t_s": np.asarray(ts, np.uint32),
            "t_e": np.asarray(te, np.uint32), "t_end": int(max(te)), "cases": cases,
            "max_live": max_live}


def lifetime_conflict_matrix(ts, te) -> np.ndarray:
    ts = np.asarray(ts, np.int64); te = np.asarray(te, np.int64)
    return (ts[:, None] < te[None, :]) & (ts[None, :] < te[:, None])


def count_conflicts(size, ts, te, a):
    """(number of conflicting unordered pairs, first pair) straight from Sec. 5.1's constraint."""
    size = np.asarray(size, np.int64).astype(object)
    a = np.asarray(a, np.uint64).astype(object)
    n = len(size)
    tm = lifetime_conflict_matrix(ts, te)
    cnt, first = 0, (0xFFFFFFFF, 0xFFFFFFFF)
    for i in range(n):
        for j in range(i + 1, n):
            if tm[i, j] and a[i] < a[j] + size[j] and a[j] < a[i] + size[i]:
                if cnt == 0:
                    first = (i, j)
                cnt += 1
    return cnt, first


def count_conflicts_fast(size, ts, te, a) -> int:
    """Vectorised version for a few thousand requests (int64 arithmetic; values < 2^62)."""
    size = np.asarray(size, np.int64); a = np.asarray(a, np.uint64).astype(np.int64)
    tm = lifetime_conflict_matrix(ts, te)
    am = (a[:, None] < (a + size)[None, :]) & (a[None, :] < (a + size)[:, None])
    both = np.triu(tm & am, k=1)
    return int(both.sum())


def check_lowest_fit(size, ts, te, order, a) -> None:
    """Re-derive every placement from the definition: the address of the k-th request in
    `order` is the smallest x in {0} U {ends of earlier lifetime-conflicting blocks} at
    which it conflicts with none of them (any feasible minimum lies in that set)."""
    size = [int(x) for x in size]; ts = [int(x) for x in ts]; te = [int(x) for x in te]
    a = [int(x) for x in a]
    placed: List[int] = []
    for i in (int(x) for x in order):
        nb = [j for j in placed if ts[i] < te[j] and ts[j] < te[i]]
        cands = sorted({0} | {a[j] + size[j] for j in nb})
        want = None
        for x in cands:
            if all(x + size[i] <= a[j] or a[j] + size[j] <= x for j in nb):
                want = x
                break
        assert want is not None
        assert a[i] == want, f"request {i}: address {a[i]}, lowest free address is {want}"
        placed.append(i)


def max_live_numpy(size, ts, te, t_end):
    net = np.zeros(int(t_end) + 1, dtype=np.int64)
    np.add.at(net, np.asarray(ts, np.int64), np.asarray(size, np.int64))
    np.add.at(net, np.asarray(te, np.int64), -np.asarray(size, np.int64))
    live = np.cumsum(net)[: int(t_end)]
    t = int(np.argmax(live))
    return int(live[t]), t


def random_trace(rng, n, t_max=None, unique_times=False, sizes=None):
    """Small random trace for property tests."""
    if unique_times:
        stamps = rng.permutation(2 * n)
        pairs = np.sort(stamps.reshape(n, 2), axis=1)
        ts, te = pairs[:, 0], pairs[:, 1]
        t_end = 2 * n
    else:
        t_max = t_max or max(4, n)
        ts = rng.integers(0, t_max, size=n)
        te = ts + rng.integers(1, t_max, size=n)
        t_end = int(te.max())
    if sizes is None:
        size = rng.integers(1, 9, size=n)
    else:
        size = rng.choice(np.asarray(sizes), size=n)
    return size.astype(np.uint64), ts.astype(np.uint32), te.astype(np.uint32), int(t_end)
