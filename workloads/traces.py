"""Synthetic training-shaped allocation traces.

A trace is the list M of request events of one training iteration (Sec. 4):
each request is (s, t_s, t_e) = (size in bytes, allocation timestamp, free
timestamp).  The real traces come from profiling training runs and are not
available, so these generators imitate their published shape:

* few distinct sizes that repeat across layers and micro-batches
  (Sec. 2.3, "spatial regularity", Fig. 3);
* three lifetime classes -- persistent, scoped (allocated in a forward pass,
  released in reverse order in the matching backward pass) and transient
  (Sec. 2.3, "temporal regularity", Fig. 4);
* request counts per iteration of 10^4 .. 3*10^5 (Table 2);
* interleaving of allocation and release caused by pipeline schedules,
  virtual pipeline chunks and recomputation (Sec. 1, Sec. 2.1).

Every allocation and every release takes the next integer timestamp, so all
timestamps are distinct and the number of events is t_end = 2 n.  Lifetimes
are half-open, [t_alloc, t_free).

Configurations 6 and 7 are a second kind of workload derived from 2 and 4: several
iterations back to back, persistent tensors that live through all of them
(Sec. 2.3 names persistent tensors as the third lifetime class) and coarse
timestamps, as a profiler with a slower clock would record them, so that many
requests start and end at the same instant.

Only inputs are produced here; nothing in this file places, validates or
bounds anything.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 20250716
GRANULE = 512  # trace producers round sizes up to 512 B (Sec. 2.3 counts tensors > 512 B)


@dataclass
class Trace:
    name: str
    size: np.ndarray      # uint64 [n], bytes, > 0
    t_alloc: np.ndarray   # uint32 [n]
    t_free: np.ndarray    # uint32 [n], t_alloc < t_free <= t_end
    t_end: int
    meta: Dict = field(default_factory=dict)
    p_alloc: np.ndarray = None   # uint32 [n], computation phase (forward / backward pass of a micro-batch, optimizer
    p_free: np.ndarray = None    # step, in schedule order) in which the request is allocated / released (Sec. 4: p_s, p_e)

    @property
    def n(self) -> int:
        return int(self.size.shape[0])


def _round_up(x: int, g: int = GRANULE) -> int:
    return ((int(x) + g - 1) // g) * g


class _Emitter:
    """Hands out timestamps; keeps a countdown list for transient tensors."""

    def __init__(self) -> None:
        self.size: List[int] = []
        self.ta: List[int] = []
        self.tf: List[int] = []
        self.t = 0
        self.phase = 0                       # the computation phase the events that follow belong to
        self.ps: List[int] = []
        self.pe: List[int] = []
        self._pending: List[List[int]] = []  # [remaining further allocations, id]

    def free(self, rid: int) -> None:
        assert self.tf[rid] < 0
        self.tf[rid] = self.t
        self.pe[rid] = self.phase
        self.t += 1

    def _age_pending(self) -> None:
        if not self._pending:
            return
        keep = []
        for ent in self._pending:
            if ent[0] == 0:
                self.free(ent[1])
            else:
                ent[0] -= 1
                keep.append(ent)
        self._pending = keep

    def alloc(self, size: int) -> int:
        self._age_pending()
        rid = len(self.size)
        self.size.append(_round_up(size))
        self.ta.append(self.t)
        self.tf.append(-1)
        self.ps.append(self.phase)
        self.pe.append(-1)
        self.t += 1
        return rid

    def alloc_transient(self, size: int, further_allocs: int) -> int:
        """A tensor released after `further_allocs` more allocations happened."""
        rid = self.alloc(size)
        self._pending.append([int(further_allocs), rid])
        return rid

    def flush(self) -> None:
        for ent in self._pending:
            self.free(ent[1])
        self._pending = []

    def finish(self, name: str, meta: Dict) -> Trace:
        self.flush()
        assert all(t >= 0 for t in self.tf)
        n = len(self.size)
        assert self.t == 2 * n
        return Trace(
            name=name,
            size=np.asarray(self.size, dtype=np.uint64),
            t_alloc=np.asarray(self.ta, dtype=np.uint32),
            t_free=np.asarray(self.tf, dtype=np.uint32),
            t_end=self.t,
            meta=meta,
            p_alloc=np.asarray(self.ps, dtype=np.uint32),
            p_free=np.asarray(self.pe, dtype=np.uint32),
        )


# ---------------------------------------------------------------------------
# schedules: sequences of ("F" | "B", micro-batch, chunk)
# ---------------------------------------------------------------------------

def _schedule_1f1b(n_mb: int, warmup: int) -> List[Tuple[str, int, int]]:
    """One-forward-one-backward: `warmup` forwards, alternating F/B, cool-down."""
    w = min(warmup, n_mb)
    seq = [("F", m, 0) for m in range(w)]
    for k in range(n_mb - w):
        seq.append(("F", w + k, 0))
        seq.append(("B", k, 0))
    for k in range(n_mb - w, n_mb):
        seq.append(("B", k, 0))
    return seq


def _schedule_interleaved(n_mb: int, v: int, p: int) -> List[Tuple[str, int, int]]:
    """Interleaved 1F1B of the first pipeline rank with v model chunks.

    The k-th forward chunk-pass runs chunk (k div p) mod v on micro-batch
    (k div (p v)) p + k mod p; backward passes mirror it with chunks reversed.
    """
    total = n_mb * v

    def mb_of(k: int) -> int:
        return (k // (p * v)) * p + k % p

    def f_unit(k: int) -> Tuple[str, int, int]:
        return ("F", mb_of(k), (k // p) % v)

    def b_unit(k: int) -> Tuple[str, int, int]:
        return ("B", mb_of(k), v - 1 - (k // p) % v)

    w = min((p - 1) * 2 + (v - 1) * p, total)
    seq = [f_unit(k) for k in range(w)]
    for k in range(total - w):
        seq.append(f_unit(w + k))
        seq.append(b_unit(k))
    for k in range(total - w, total):
        seq.append(b_unit(k))
    return seq


# ---------------------------------------------------------------------------
# layer templates
# ---------------------------------------------------------------------------

@dataclass
class _Cfg:
    name: str
    description: str
    n_orderings: int
    layers_per_chunk: int
    chunks: int
    n_mb: int
    h: int
    s: int
    a_f: int = 12
    a_b: int = 12
    p_tmp: float = 0.3
    l_max: int = 5
    k_choices: Tuple[int, ...] = (1, 3, 4, 8)
    score_heads: int = 0          # one score buffer per layer-pass of heads*s*s*2/4 bytes
    warmup: int = 3
    kind: str = "dense"           # dense | recompute | moe | interleaved | tiny
    pipeline_depth: int = 4
    experts: int = 0
    tokens_per_mb: int = 0
    small_per_pass: int = 0
    base: int = 0                 # kind "multi": the configuration whose iteration is repeated
    iterations: int = 1
    persistent: int = 0           # tensors alive from the first to the last event
    quantum: int = 1              # events per recorded timestamp


CONFIGS: Dict[int, _Cfg] = {
    1: _Cfg("cfg1_tiny", "2-layer transformer, 1 micro-batch", 64, 2, 1, 1, 512, 512,
            l_max=3, k_choices=(1, 2, 3, 4), warmup=1, kind="tiny"),
    2: _Cfg("cfg2_1f1b_32l", "pipeline stage, 32 layers, h=4096, s=4096, 1F1B, 8 micro-batches (4 in flight)",
            1024, 32, 1, 8, 4096, 4096, score_heads=32, kind="dense"),
    3: _Cfg("cfg3_recompute_80l", "pipeline stage, 80 layers, h=8192, s=4096, selective recomputation",
            2048, 80, 1, 8, 8192, 4096, score_heads=64, kind="recompute"),
    4: _Cfg("cfg4_moe_16l", "MoE stage, 16 layers, 64 experts, top-2, 8192 tokens per micro-batch, h=4096",
            2048, 16, 1, 8, 4096, 8192, kind="moe", experts=64, tokens_per_mb=8192),
    5: _Cfg("cfg5_interleaved", "interleaved 1F1B, 4 chunks x 16 layers, 8 micro-batches, h=8192, s=8192",
            4096, 16, 4, 8, 8192, 8192, kind="interleaved", small_per_pass=183),
    6: _Cfg("cfg6_two_iterations", "two iterations of the 32-layer 1F1B stage, 256 persistent tensors, 4 events per timestamp",
            1024, 32, 1, 8, 4096, 4096, kind="multi", base=2, iterations=2, persistent=256, quantum=4),
    7: _Cfg("cfg7_moe_coarse_clock", "the MoE stage with 128 persistent tensors, 8 events per timestamp",
            2048, 16, 1, 8, 4096, 8192, kind="multi", base=4, iterations=1, persistent=128, quantum=8),
}

_SMALL_SIZES = (512, 1024, 1536, 2048, 3072, 4096, 6144, 8192, 12288, 16384,
                24576, 32768, 40960, 49152, 57344, 65536)


def _free_interleaved(em: _Emitter, scoped: List[int]) -> None:
    """Release one scoped tensor, most recent first (Fig. 4)."""
    if scoped:
        em.free(scoped.pop())


def _make_multi(cfg_id: int) -> Trace:
    """Iterations of a base configuration back to back, persistent tensors around them, coarse clock."""
    c = CONFIGS[cfg_id]
    base = make_trace(c.base)
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + cfg_id))
    act = c.s * c.h * 2
    pers_size = np.asarray([_round_up(act * int(rng.choice(c.k_choices))) for _ in range(c.persistent)], dtype=np.uint64)
    # events: the persistent allocations, then the iterations, then the persistent releases
    t0 = c.persistent
    span = base.t_end
    size = [pers_size]
    ta = [np.arange(c.persistent, dtype=np.int64)]
    tf = [t0 + c.iterations * span + np.arange(c.persistent, dtype=np.int64)[::-1]]
    for it in range(c.iterations):
        size.append(base.size)
        ta.append(base.t_alloc.astype(np.int64) + t0 + it * span)
        tf.append(base.t_free.astype(np.int64) + t0 + it * span)
    size = np.concatenate(size)
    ta = np.concatenate(ta) // c.quantum
    tf = np.concatenate(tf) // c.quantum
    tf = np.maximum(tf, ta + 1)                 # a lifetime shorter than the clock's tick still holds its memory for one
    meta = {"cfg": cfg_id, "description": c.description, "n_orderings": c.n_orderings, "seed": BASE_SEED + cfg_id}
    # phases: 0 = before the first iteration, then the base trace's phases once per iteration, then one for the end
    per_it = int(base.p_free.max()) + 1
    ps = [np.zeros(c.persistent, np.int64)] + [base.p_alloc.astype(np.int64) + 1 + it * per_it for it in range(c.iterations)]
    pe = [np.full(c.persistent, 1 + c.iterations * per_it, np.int64)] + \
         [base.p_free.astype(np.int64) + 1 + it * per_it for it in range(c.iterations)]
    return Trace(name=c.name, size=size, t_alloc=ta.astype(np.uint32), t_free=tf.astype(np.uint32),
                 t_end=int(tf.max()), meta=meta, p_alloc=np.concatenate(ps).astype(np.uint32),
                 p_free=np.concatenate(pe).astype(np.uint32))


def make_trace(cfg_id: int) -> Trace:
    """Build the trace of configuration `cfg_id` (1..7); fully determined by the id."""
    c = CONFIGS[cfg_id]
    if c.kind == "multi":
        return _make_multi(cfg_id)
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + cfg_id))
    em = _Emitter()
    act = c.s * c.h * 2  # one bf16 activation of s x h
    score = c.score_heads * c.s * c.s * 2 // 4 if c.score_heads else 0
    scoped: Dict[Tuple[int, int], List[int]] = {}
    recomputed: Dict[Tuple[int, int], List[int]] = {}   # sizes to re-allocate in backward
    expert_sizes: Dict[Tuple[int, int], List[int]] = {}
    persistent_until_end: List[int] = []

    def pick_size(j: int) -> int:
        if score and j == 5:
            return score
        return act * int(rng.choice(c.k_choices))

    def life() -> int:
        return int(rng.integers(1, c.l_max + 1))

    def fwd_layer(mb: int, layer: int) -> None:
        keep: List[int] = []
        if c.kind in ("dense", "tiny"):
            for j in range(c.a_f):
                sz = pick_size(j)
                if rng.random() < c.p_tmp:
                    em.alloc_transient(sz, life())
                else:
                    keep.append(em.alloc(sz))
        elif c.kind == "recompute":
            rec_idx = (1, 2, 4, 5, 7, 8, 10)
            rec_ids, rec_sizes = [], []
            for j in range(c.a_f):
                sz = pick_size(j)
                rid = em.alloc(sz)
                if j in rec_idx:
                    rec_ids.append(rid)
                    rec_sizes.append(sz)
                else:
                    keep.append(rid)
            for rid in reversed(rec_ids):   # dropped at the end of the forward layer-pass
                em.free(rid)
            recomputed[(mb, layer)] = rec_sizes
        elif c.kind == "moe":
            for j in range(6):
                sz = act * int(rng.choice(c.k_choices))
                if rng.random() < c.p_tmp:
                    em.alloc_transient(sz, life())
                else:
                    keep.append(em.alloc(sz))
            probs = rng.dirichlet(np.full(c.experts, 0.5))
            tokens = rng.multinomial(2 * c.tokens_per_mb, probs)   # top-2 routing
            sizes = []
            for e in range(c.experts):
                if tokens[e] == 0:
                    continue
                sz = int(tokens[e]) * c.h * 2
                sizes.append(sz)
                keep.append(em.alloc(sz))
                em.alloc_transient(sz, life())
                keep.append(em.alloc(sz))
            expert_sizes[(mb, layer)] = sizes
        elif c.kind == "interleaved":
            total = c.a_f + c.small_per_pass
            for j in range(total):
                if j % 16 == 0 and j // 16 < c.a_f:
                    sz = act * int(rng.choice(c.k_choices))
                    if rng.random() < c.p_tmp:
                        em.alloc_transient(sz, life())
                    else:
                        keep.append(em.alloc(sz))
                else:
                    em.alloc_transient(int(rng.choice(_SMALL_SIZES)), life())
        scoped[(mb, layer)] = keep

    def bwd_layer(mb: int, layer: int, extra_persistent: bool) -> None:
        keep = scoped.pop((mb, layer))
        rec_ids: List[int] = []
        if c.kind == "recompute":
            for sz in recomputed.pop((mb, layer)):
                rec_ids.append(em.alloc(sz))
        if c.kind == "moe":
            for sz in reversed(expert_sizes.pop((mb, layer))):
                for _ in range(3):
                    em.alloc_transient(sz, life())
                _free_interleaved(em, keep)
        elif c.kind == "interleaved":
            total = c.a_b + c.small_per_pass
            for j in range(total):
                if j % 16 == 0 and j // 16 < c.a_b:
                    em.alloc_transient(act * int(rng.choice(c.k_choices)), life())
                    _free_interleaved(em, keep)
                else:
                    em.alloc_transient(int(rng.choice(_SMALL_SIZES)), life())
        else:
            for j in range(c.a_b):
                em.alloc_transient(pick_size(j), life())
                if extra_persistent:   # weight-gradient buffer kept until the optimizer step
                    persistent_until_end.append(em.alloc(act * int(rng.choice(c.k_choices))))
                _free_interleaved(em, keep)
        while keep:
            em.free(keep.pop())
        for rid in reversed(rec_ids):
            em.free(rid)

    if c.chunks == 1:
        schedule = _schedule_1f1b(c.n_mb, c.warmup)
    else:
        schedule = _schedule_interleaved(c.n_mb, c.chunks, c.pipeline_depth)

    last_backward_of_chunk = {}
    for idx, (ph, mb, ch) in enumerate(schedule):
        if ph == "B":
            last_backward_of_chunk[ch] = idx

    for idx, (ph, mb, ch) in enumerate(schedule):
        em.phase = idx                               # one phase per forward / backward pass of the schedule
        layers = range(ch * c.layers_per_chunk, (ch + 1) * c.layers_per_chunk)
        if ph == "F":
            for layer in layers:
                fwd_layer(mb, layer)
        else:
            for layer in reversed(layers):
                bwd_layer(mb, layer, extra_persistent=(c.kind == "tiny"))
            if c.kind == "interleaved" and last_backward_of_chunk[ch] == idx:
                persistent_until_end.append(em.alloc(25 * 2 ** 20))   # gradient bucket

    # optimizer step
    em.phase = len(schedule)
    if c.kind == "tiny":
        for _layer in range(c.layers_per_chunk):
            for _ in range(12):
                em.alloc_transient(act * int(rng.choice(c.k_choices)), life())
    elif c.kind == "interleaved":
        params_per_layer = 12 * c.h * c.h
        for _layer in range(c.chunks * c.layers_per_chunk):
            em.alloc_transient(2 * params_per_layer * 4, int(rng.integers(1, 4)))
    em.flush()
    for rid in reversed(persistent_until_end):
        em.free(rid)

    meta = {"cfg": cfg_id, "description": c.description, "n_orderings": c.n_orderings,
            "seed": BASE_SEED + cfg_id}
    return em.finish(c.name, meta)


def trace_stats(tr: Trace) -> Dict:
    """Shape statistics of a trace (no planning): n, T, number of lifetime-overlapping
    pairs E, distinct sizes and the share of short-lived requests."""
    n = tr.n
    ta = tr.t_alloc.astype(np.int64)
    tf = tr.t_free.astype(np.int64)
    # E = number of unordered pairs with ta_i < tf_j and ta_j < tf_i.  For each i
    # count the j that started before i's release minus those released by i's start
    # (those two sets are nested), then subtract the self pair and halve.
    ta_sorted = np.sort(ta)
    tf_sorted = np.sort(tf)
    started_before_my_free = np.searchsorted(ta_sorted, tf, side="left")
    freed_by_my_alloc = np.searchsorted(tf_sorted, ta, side="right")
    deg = started_before_my_free - freed_by_my_alloc - 1
    life = tf - ta
    return {
        "n": n,
        "T": int(tr.t_end),
        "E": int(deg.sum() // 2),
        "mean_degree": float(deg.mean()) if n else 0.0,
        "max_degree": int(deg.max()) if n else 0,
        "distinct_sizes": int(np.unique(tr.size).shape[0]),
        "sum_size": int(tr.size.astype(object).sum()) if n else 0,
        "short_lived_share": float((life <= 16).mean()) if n else 0.0,
        "max_size": int(tr.size.max()) if n else 0,
    }
