"""Parity of the placement kernel that keeps only long-lived blocks in its sorted list (long traces
with few long-lived requests) with the CPU oracle, through the C ABI: every address, bit by bit."""
import os

import numpy as np
import pytest

from workloads import Trace

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    return S


def _plan(S, tr, orders):
    import torch
    size, ta, tf = S.trace_to_device(tr)
    o = torch.from_numpy(np.ascontiguousarray(orders).view(np.int32)).cuda()
    out = S.stalloc_plan(size, ta, tf, tr.t_end, o)
    torch.cuda.synchronize()
    info = S.stalloc_plan_report(out)
    return {"status": int(out["status"].item()), "offsets": out["offsets"].cpu().numpy().view(np.uint64),
            "peaks": out["peaks"].cpu().numpy().view(np.uint64), "best_plan": int(out["best_plan"].item()),
            "best_offsets": out["best_offsets"].cpu().numpy().view(np.uint64), "info": info, "raw": out}


def _validate(S, tr, offsets_dev):
    import torch
    size, ta, tf = S.trace_to_device(tr)
    out = S.stalloc_validate(size, ta, tf, tr.t_end, offsets_dev)
    torch.cuda.synchronize()
    assert int(out["status"].item()) == 0
    return out["conflicts"].cpu().numpy().view(np.uint64)


def two_kinds(rng, n, n_long, short_life, sizes_long, sizes_short, quantum=1, long_span=(8, 2)):
    """n requests on 2n distinct timestamps; n_long of them live for an eighth to a half of the trace, the
    others for 1..short_life timestamps; `quantum` timestamps share one recorded instant."""
    T = 2 * n
    ts = rng.permutation(T)[:n].astype(np.int64)
    life = rng.integers(1, short_life + 1, n)
    long_ids = rng.choice(n, n_long, replace=False)
    life[long_ids] = rng.integers(T // long_span[0], T // long_span[1], n_long)
    te = np.minimum(ts + life, T)
    size = rng.choice(np.asarray(sizes_short, dtype=np.uint64), n)
    size[long_ids] = rng.choice(np.asarray(sizes_long, dtype=np.uint64), n_long)
    ts //= quantum
    te = np.maximum(te // quantum, ts + 1)
    return Trace(name="two kinds", size=size, t_alloc=ts.astype(np.uint32), t_free=te.astype(np.uint32),
                 t_end=int(te.max()))


def _orders(rng, tr, random_rows):
    n = tr.n
    rows = [np.argsort(-tr.size.astype(np.int64), kind="stable"),                      # all long blocks first
            np.lexsort((np.arange(n), tr.t_alloc)),                                      # by time: one long chain of waits
            np.lexsort((np.arange(n), -(tr.t_free.astype(np.int64) - tr.t_alloc)))]
    rows += [rng.permutation(n) for _ in range(random_rows)]
    return np.stack(rows).astype(np.uint32)


def _compare(S, oracle, tr, orders, want_kernel="long_list", method="allpairs", lists=None):
    got = _plan(S, tr, orders)
    assert got["status"] == 0
    assert got["info"]["kernel"] == want_kernel, got["info"]
    a, ext = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=THREADS, method=method, lists=lists)
    assert np.array_equal(got["peaks"], ext), "extents differ"
    bad = np.nonzero((got["offsets"] != a).any(axis=1))[0]
    assert bad.size == 0, f"addresses differ in plans {bad[:8]}"
    assert got["best_plan"] == oracle.best_plan(ext)
    assert np.array_equal(got["best_offsets"], a[got["best_plan"]])
    return got, a, ext


@pytest.mark.parametrize("seed", range(8))
def test_random_traces_of_two_kinds(S, oracle, seed):
    """Sizes in 512-byte units and odd byte sizes (32-bit granule counts tried plan by plan), with and
    without tied timestamps, lifetime thresholds from 1 to 31, 50 to 1100 long-lived requests."""
    rng = np.random.default_rng(8800 + seed)
    n = int(rng.integers(9500, 14000))
    assert n > S.lib.stalloc_plan_lds_capacity()
    odd = seed % 4 == 3
    sizes_long = [1 << 20, 3 << 20, 5 << 19] if not odd else [1048577, 3145731, 2621443]
    sizes_short = [512, 1024, 4096, 1 << 16, 3 << 9] if not odd else [513, 1025, 4099, 65537, 1537, 999_999]
    quantum = int(rng.choice([1, 1, 2]))
    short_life = int(rng.choice([3, 7, 15, 31] if quantum == 1 else [3, 7, 15]))     # windows of short requests fit a wave
    n_long = int(rng.integers(50, 1100))
    tr = two_kinds(rng, n, n_long, short_life, sizes_long, sizes_short, quantum=quantum)
    got, a, ext = _compare(S, oracle, tr, _orders(rng, tr, 3))
    assert got["info"]["lifetime_threshold"] in (1, 3, 7, 15, 31) and n_long - 8 <= got["info"]["long_requests"] <= n_long      # (a lifetime cut at the end of the trace may be short)
    assert got["info"]["granule_log2"] == (0 if odd else 9)


@pytest.mark.parametrize("seed", range(6))
def test_large_short_lived_blocks_have_a_table_of_their_own(S, oracle, seed):
    """A twelfth to a tenth of the short-lived requests are as large as the long-lived ones, the others
    small, with empty size classes between (as in a training trace): the large ones are also kept in a
    table that a long-lived request reads whole.  Several large sizes, tied timestamps, bursts that give
    large short requests wide windows of their own; a trace in which too many are large has no such table."""
    rng = np.random.default_rng(9100 + seed)
    n = int(rng.integers(9600, 13000))
    small = [512, 1024, 1536, 4096, 1 << 16]
    large = [1 << 20, 3 << 19, 1 << 21] if seed % 2 == 0 else [1 << 24]
    share = 11 if seed < 4 else 3                                     # one large size among `share` + 1 choices
    sizes_short = [int(rng.choice(small)) for _ in range(share * len(large))] + large
    quantum = 2 if seed == 3 else 1
    tr = two_kinds(rng, n, int(rng.integers(100, 900)), 15 if quantum == 1 else 7, [1 << 20, 3 << 20, 1 << 22], sizes_short,
                   quantum=quantum)
    if seed == 1:                                                     # a burst of short-lived requests, large ones among them
        ts, te = tr.t_alloc.astype(np.int64), tr.t_free.astype(np.int64)
        burst = np.nonzero(te - ts <= 15)[0][:120]
        life = te[burst] - ts[burst]
        ts[burst] = 7000
        te[burst] = 7000 + life
        tr = Trace(name="burst", size=tr.size, t_alloc=ts.astype(np.uint32), t_free=te.astype(np.uint32), t_end=int(te.max()))
    got, a, ext = _compare(S, oracle, tr, _orders(rng, tr, 3))
    short = (tr.t_free.astype(np.int64) - tr.t_alloc) <= got["info"]["lifetime_threshold"]
    # (the smallest size class from which at most an eighth are large, at the widest gap between classes)
    want = {0: 1 << 20, 1: 1 << 24, 2: 1 << 20, 3: 1 << 24, 4: 1 << 21, 5: 0}[seed]   # 4: only the largest of three; 5: a quarter in one class
    assert got["info"]["large_size"] == want
    if want:
        assert got["info"]["large_requests"] == int((short & (tr.size >= want)).sum()) > 500
    else:
        assert got["info"]["large_requests"] == 0


def test_crowded_short_lived_requests_overflow_the_window_pool(S, oracle):
    """Short lifetimes of up to 31 timestamps: late in an order a request finds some twenty placed
    short blocks in its window, more than the LDS pool of a batch holds for all 64 requests; the windows
    that do not fit are read again when their request is settled."""
    rng = np.random.default_rng(31)
    tr = two_kinds(rng, 10240, 400, 31, [1 << 22, 1 << 23], [512, 1536, 2048, 8192])
    _compare(S, oracle, tr, _orders(rng, tr, 2))


def test_bursts_give_some_short_lived_requests_wide_windows(S, oracle):
    """Ninety short-lived requests allocated at one instant, twice: their windows hold more ranks than
    a wave has lanes, so they are settled by the whole workgroup like the long-lived ones."""
    rng = np.random.default_rng(77)
    tr = two_kinds(rng, 9800, 300, 7, [1 << 21, 3 << 20], [512, 1024, 2560])
    ts, te = tr.t_alloc.astype(np.int64), tr.t_free.astype(np.int64)
    short = np.nonzero(te - ts <= 7)[0]
    for burst, at in ((short[:90], 5000), (short[90:180], 12001)):
        life = te[burst] - ts[burst]
        ts[burst] = at
        te[burst] = at + life
    tr = Trace(name="bursts", size=tr.size, t_alloc=ts.astype(np.uint32), t_free=te.astype(np.uint32), t_end=int(te.max()))
    _compare(S, oracle, tr, _orders(rng, tr, 3))


def test_more_orders_than_resident_workgroups(S, oracle):
    """1100 orders (two workgroups per CU are resident): sampled plans address by address, every plan
    free of conflicts, every extent at least the lower bound."""
    import torch
    rng = np.random.default_rng(5)
    tr = two_kinds(rng, 9600, 250, 15, [1 << 20, 1 << 21], [512, 1024, 16384])
    P = 1100
    orders = np.stack([rng.permutation(tr.n) for _ in range(P)]).astype(np.uint32)
    got = _plan(S, tr, orders)
    assert got["status"] == 0 and got["info"]["kernel"] == "long_list"
    rows = np.r_[0, 1, 2, np.arange(17, P, 64), P - 1]
    lists = oracle.conflict_lists(tr.t_alloc, tr.t_free)
    a, ext = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders[rows], threads=THREADS, method="lists", lists=lists)
    assert np.array_equal(got["peaks"][rows], ext) and np.array_equal(got["offsets"][rows], a)
    assert not _validate(S, tr, got["raw"]["offsets"]).any()
    lb = oracle.lower_bound(tr.size, tr.t_alloc, tr.t_free, tr.t_end)[0]
    assert (got["peaks"] >= lb).all() and got["best_plan"] == int(np.argmin(got["peaks"]))


@pytest.mark.parametrize("fill", [0.80, 0.97, 1.04])
def test_plans_that_outgrow_32_bit_counts_are_placed_again(S, oracle, fill):
    """Odd byte sizes, 300 long-lived requests that all overlap and stack up to `fill` x 2^32 bytes, and
    ten thousand short-lived ones: depending on `fill` none, some or all plans come too close to 2^32
    granules and are handed to the kernel with 64-bit addresses."""
    rng = np.random.default_rng(2032)
    n_long, n = 300, 10300
    tr = two_kinds(rng, n, n_long, 15, [1], [1537, 4099, 70001], long_span=(3, 2))
    size = tr.size.copy()
    ts, te = tr.t_alloc.astype(np.int64), tr.t_free.astype(np.int64)
    long_ids = np.nonzero(te - ts > 15)[0]
    ts[long_ids] = rng.integers(0, 1000, n_long)                     # all long-lived requests overlap around the middle
    te[long_ids] = tr.t_end - rng.integers(0, 1000, n_long)
    raw = rng.integers(1 << 22, 3 << 22, n_long).astype(np.float64)
    size[long_ids] = (raw * (fill * 2 ** 32 / raw.sum())).astype(np.uint64) | np.uint64(1)
    tr = Trace(name="near 2^32", size=size, t_alloc=ts.astype(np.uint32), t_free=te.astype(np.uint32), t_end=tr.t_end)
    orders = np.stack([rng.permutation(n) for _ in range(6)]).astype(np.uint32)
    got, a, ext = _compare(S, oracle, tr, orders)
    assert got["info"]["granule_log2"] == 0
    redone = got["info"]["plans_64bit"]
    assert (fill < 0.9 and redone == 0) or (0.9 < fill < 1.0) or (fill > 1.0 and redone == 6), redone
    assert bool((ext > np.uint64(2 ** 32)).all()) == (fill > 1.0)


def test_both_forms_of_the_list(S, oracle):
    """The list holds 8 bytes a block (ranks among the long-lived requests' allocation and release times
    in place of the times, a size class) when those requests have at most 64 sizes and the timestamps
    are not far apart, else 16 bytes; tied timestamps, and long-lived requests that begin or end together,
    in both."""
    rng = np.random.default_rng(1212)
    few = two_kinds(rng, 9800, 700, 15, [1 << 20, 3 << 20, 5 << 19, 1 << 22], [512, 1024, 4096])
    many = two_kinds(rng, 9800, 700, 15, [(k + 1) << 16 for k in range(80)], [512, 1024, 4096])
    tied = two_kinds(rng, 9900, 600, 7, [1 << 20, 3 << 20], [512, 1536], quantum=2)
    ts, te = tied.t_alloc.astype(np.int64), tied.t_free.astype(np.int64)
    long_ids = np.nonzero(te - ts > 7)[0]
    ts[long_ids[:40]] = ts[long_ids[:40]].min()                          # forty begin together, forty end together
    te[long_ids[40:80]] = te[long_ids[40:80]].max()
    tied = Trace(name="tied", size=tied.size, t_alloc=ts.astype(np.uint32), t_free=te.astype(np.uint32), t_end=int(te.max()))
    sparse = Trace(name="sparse", size=few.size, t_alloc=few.t_alloc * np.uint32(9), t_free=few.t_free * np.uint32(9),
                   t_end=int(few.t_end) * 9)
    for tr, want in ((few, 8), (many, 16), (tied, 8), (sparse, 16)):
        got, _, _ = _compare(S, oracle, tr, _orders(rng, tr, 2))
        assert got["info"]["list_entry_bytes"] == want, (tr.name, got["info"])


def test_traces_the_kernel_leaves_to_the_sorted_list(S, oracle):
    """Too many long-lived requests for the LDS list, and timestamps so coarse that every window is
    wide: the sorted-list kernel places these; results equal the oracle's all the same."""
    rng = np.random.default_rng(404)
    many_long = two_kinds(rng, 10000, 4000, 15, [1 << 20], [512, 4096])
    coarse = two_kinds(rng, 10000, 200, 15, [1 << 20], [512, 4096], quantum=400)
    for tr in (many_long, coarse):
        _compare(S, oracle, tr, _orders(rng, tr, 1)[[0, 3]], want_kernel="list_memory")


def test_malformed_orders_end_normally(S):
    """An entry beyond n is reported; a row that repeats requests gives an unspecified plan, but the
    call ends and stays inside its buffers."""
    rng = np.random.default_rng(9)
    tr = two_kinds(rng, 9700, 200, 15, [1 << 20], [512, 4096])
    orders = np.stack([rng.permutation(tr.n) for _ in range(2)]).astype(np.uint32)
    bad = orders.copy()
    bad[1, 100] = tr.n + 7
    assert _plan(S, tr, bad)["status"] == 6
    repeated = orders.copy()
    long_ids = np.nonzero(tr.t_free.astype(np.int64) - tr.t_alloc > 15)[0]
    repeated[0, :] = np.resize(long_ids, tr.n)                         # 9700 long blocks for a list of a few thousand
    got = _plan(S, tr, repeated)
    assert got["status"] == 0 and got["info"]["kernel"] == "long_list"
