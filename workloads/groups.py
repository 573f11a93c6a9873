"""HomoPhase groups of a trace and the candidate pairs handed to the fusion step (inputs only).

A group is the set of requests with one (allocation phase, release phase) pair of labels
(Sec. 5.1, HomoPhase Group Planning).  Two groups are a candidate pair when the phase in which
one is released is the phase in which the other is allocated: their lifetimes touch there and
nowhere else.  Nothing of the fusion itself lives here."""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def homophase_groups(p_alloc: np.ndarray, p_free: np.ndarray) -> List[np.ndarray]:
    """Request numbers (ascending) of every group, groups in order of (p_alloc, p_free)."""
    key = p_alloc.astype(np.uint64) << np.uint64(32) | p_free.astype(np.uint64)
    order = np.argsort(key, kind="stable")
    cuts = np.flatnonzero(np.diff(key[order])) + 1
    return [g.astype(np.uint32) for g in np.split(order, cuts)]


def candidate_pairs(p_alloc: np.ndarray, p_free: np.ndarray) -> Tuple[List[np.ndarray], List[Tuple[int, int]]]:
    """-> (groups, pairs): pairs (g, h) of group numbers with release phase of g = allocation phase of h."""
    groups = homophase_groups(p_alloc, p_free)
    ps = [int(p_alloc[g[0]]) for g in groups]
    pe = [int(p_free[g[0]]) for g in groups]
    pairs = [(g, h) for g in range(len(groups)) for h in range(len(groups)) if g != h and pe[g] == ps[h]]
    return groups, pairs


def flatten_pairs(groups: List[np.ndarray], pairs: List[Tuple[int, int]]):
    """-> members uint32 [m], pair_begin uint32 [k+1], count1 uint32 [k], largest pair."""
    members, begin, count1 = [], [0], []
    for g, h in pairs:
        members += [groups[g], groups[h]]
        begin.append(begin[-1] + len(groups[g]) + len(groups[h]))
        count1.append(len(groups[g]))
    return (np.concatenate(members).astype(np.uint32), np.asarray(begin, dtype=np.uint32),
            np.asarray(count1, dtype=np.uint32), int(np.diff(begin).max()))
