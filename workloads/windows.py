"""Time windows for dynamic-reusable-space queries.

The paper queries the plan once per group of dynamic requests, over the span from the start of the
layer that allocates them to the end of the layer that frees them (Sec. 5.2).  The stand-in:
k half-open windows [w_lo, w_hi) with a uniform start and a log-uniform length between 2 events
and a quarter of the iteration -- short layer-level spans are the common case, long ones exist.
Seeded (numpy PCG64, seed 7000 + cfg index unless given); no method arithmetic here.
"""
from __future__ import annotations

import numpy as np

from .traces import Trace


def make_windows(tr: Trace, k: int, seed: int = 7000) -> np.ndarray:
    """uint32 [k][2], 0 <= w_lo < w_hi <= t_end."""
    rng = np.random.default_rng(seed)
    t_end = int(tr.t_end)
    longest = max(2, t_end // 4)
    length = np.exp(rng.uniform(np.log(2.0), np.log(float(longest)), size=k)).astype(np.int64)
    length = np.clip(length, 1, t_end)
    lo = rng.integers(0, t_end, size=k)
    hi = np.minimum(lo + length, t_end)
    lo = np.minimum(lo, hi - 1)
    return np.stack([lo, hi], axis=1).astype(np.uint32)
