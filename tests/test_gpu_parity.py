"""Parity of the HIP library (through its C ABI) with the CPU oracle: bit-exact addresses,
extents, conflict counts, first pairs and live-byte maxima on the same seeded inputs."""
import os

import numpy as np
import pytest

from helpers import count_conflicts_fast, load_golden, random_trace
from workloads import CONFIGS, Trace, make_orderings, make_trace

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)
NONE_PAIR = (0xFFFFFFFF, 0xFFFFFFFF)


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    return S


class _T:
    def __init__(self, size, ts, te, t_end):
        self.size, self.t_alloc, self.t_free, self.t_end = size, ts, te, t_end


def _gpu_plan(S, tr, orders, **kw):
    import torch
    size, ta, tf = S.trace_to_device(tr)
    o = torch.from_numpy(np.ascontiguousarray(orders).view(np.int32)).cuda()
    out = S.stalloc_plan(size, ta, tf, tr.t_end, o, **kw)
    torch.cuda.synchronize()
    res = {"status": int(out["status"].item()), "info": S.stalloc_plan_report(out)}
    if res["status"] == 0:
        res["peaks"] = out["peaks"].cpu().numpy().view(np.uint64)
        res["best_plan"] = int(out["best_plan"].item())
        if out["offsets"] is not None:
            res["offsets"] = out["offsets"].cpu().numpy().view(np.uint64)
        if out["best_offsets"] is not None:
            res["best_offsets"] = out["best_offsets"].cpu().numpy().view(np.uint64)
    return res


def _gpu_validate(S, tr, offsets, want_status=0):
    import torch
    size, ta, tf = S.trace_to_device(tr)
    off = torch.from_numpy(np.ascontiguousarray(offsets).view(np.int64)).cuda()
    out = S.stalloc_validate(size, ta, tf, tr.t_end, off)
    torch.cuda.synchronize()
    assert int(out["status"].item()) == want_status
    return (out["conflicts"].cpu().numpy().view(np.uint64),
            out["first_pair"].cpu().numpy().view(np.uint32))


def _gpu_lower_bound(S, tr):
    import torch
    size, ta, tf = S.trace_to_device(tr)
    out = S.stalloc_lower_bound(size, ta, tf, tr.t_end)
    torch.cuda.synchronize()
    return int(out["status"].item()), int(out["lower_bound"].cpu().numpy().view(np.uint64)[0]), int(out["t_at_max"].item())


def _compare_plans(S, oracle, tr, orders, method="lists", lists=None):
    got = _gpu_plan(S, tr, orders)
    assert got["status"] == 0
    a, ext = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=THREADS, method=method, lists=lists)
    assert np.array_equal(got["peaks"], ext), "extents differ"
    bad = np.nonzero((got["offsets"] != a).any(axis=1))[0]
    assert bad.size == 0, f"addresses differ in plans {bad[:8]}"
    best = oracle.best_plan(ext)
    assert got["best_plan"] == best
    assert np.array_equal(got["best_offsets"], a[best])
    return got, a, ext


# --------------------------------------------------------------------------- lower bound

@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_lower_bound_configs(S, oracle, cfg):
    tr = make_trace(cfg)
    status, lb, t_at = _gpu_lower_bound(S, tr)
    assert status == 0
    assert (lb, t_at) == oracle.lower_bound(tr.size, tr.t_alloc, tr.t_free, tr.t_end, "sweep")


@pytest.mark.parametrize("seed", range(8))
def test_lower_bound_random_with_ties(S, oracle, seed):
    rng = np.random.default_rng(700 + seed)
    n = int(rng.integers(1, 9000))
    size, ts, te, t_end = random_trace(rng, n, t_max=int(rng.integers(2, 5000)))
    size = size * np.uint64(rng.integers(1, 2 ** 30))
    tr = _T(size, ts, te, t_end)
    status, lb, t_at = _gpu_lower_bound(S, tr)
    assert status == 0
    assert (lb, t_at) == oracle.lower_bound(size, ts, te, t_end, "sweep")


def test_lower_bound_plateau_reports_earliest_time(S, oracle):
    size = np.asarray([5, 5, 5], np.uint64)
    ts = np.asarray([10, 4100, 9000], np.uint32)
    te = np.asarray([20, 4200, 9100], np.uint32)
    tr = _T(size, ts, te, 10000)
    assert _gpu_lower_bound(S, tr) == (0, 5, 10)
    assert oracle.lower_bound(size, ts, te, 10000) == (5, 10)


# --------------------------------------------------------------------------- validate

def test_validate_hand_worked_and_planted(S, oracle):
    for name in ("running_max.txt", "hole_and_tie.txt", "gap_fit.txt"):
        g = load_golden(name)
        tr = _T(g["size"], g["t_s"], g["t_e"], g["t_end"])
        offs = np.asarray([c["a"] for c in g["cases"]], np.uint64)
        cnt, pair = _gpu_validate(S, tr, offs)
        assert not cnt.any() and (pair == 0xFFFFFFFF).all()
        zero = np.zeros_like(offs[:1])
        cnt, pair = _gpu_validate(S, tr, zero)
        want = oracle.validate(tr.size, tr.t_alloc, tr.t_free, zero[0])
        assert (int(cnt[0]), tuple(int(x) for x in pair[0])) == want and want[0] > 0


@pytest.mark.parametrize("cfg", [1, 2])
def test_validate_configs_with_planted_conflicts(S, oracle, cfg):
    tr = make_trace(cfg)
    rng = np.random.default_rng(800 + cfg)
    orders = make_orderings(tr, 6)
    a, _ = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=THREADS, method="lists")
    bad = a.copy()
    for p in range(1, 6):                      # plan 0 stays valid
        for i in rng.choice(tr.n, size=p * 3, replace=False):
            bad[p, i] = rng.integers(0, int(a[p].max()) + 1)
    cnt, pair = _gpu_validate(S, tr, bad)
    for p in range(6):
        want = oracle.validate(tr.size, tr.t_alloc, tr.t_free, bad[p])
        assert (int(cnt[p]), tuple(int(x) for x in pair[p])) == want
    assert int(cnt[0]) == 0 and tuple(int(x) for x in pair[0]) == NONE_PAIR
    assert int(cnt[1:].sum()) > 0


def test_validate_ragged_tile_sizes(S, oracle):
    rng = np.random.default_rng(810)
    for n in (1, 2, 255, 256, 257, 513, 1000):
        size, ts, te, t_end = random_trace(rng, n, t_max=40)
        tr = _T(size, ts, te, t_end)
        offs = rng.integers(0, 64, size=(3, n)).astype(np.uint64)
        cnt, pair = _gpu_validate(S, tr, offs)
        for p in range(3):
            want = oracle.validate(size, ts, te, offs[p])
            assert (int(cnt[p]), tuple(int(x) for x in pair[p])) == want


def test_plan_sized_leaves_the_bitmap_kernel_and_its_index_out_when_the_sizes_rule_it_out(S, oracle):
    """Config 2 suits the occupancy-bitmap kernel (sizes of 1 to 8 granules of 32 MiB).  Told the truth about
    its sizes, the sized call does what stalloc_plan does; told that sizes reach 64 granules, it leaves
    that kernel and its index of lifetime-overlapping pairs (76 MB here) out and the sorted list places the
    trace: same addresses either way.  Nonsense figures are refused on the host."""
    import torch
    tr = make_trace(2)
    orders = make_orderings(tr, 16)
    size, ta, tf = S.trace_to_device(tr)
    o = torch.from_numpy(orders.view(np.int32)).cuda()
    a, ext = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=THREADS, method="lists")
    plain = S.stalloc_plan(size, ta, tf, tr.t_end, o)
    kinds = {}
    for name, largest, granule in (("true", int(tr.size.max()), 1 << 25), ("ruled out", 64 << 25, 1 << 25),
                                   ("no granule known", int(tr.size.max()), 1)):
        out = S.stalloc_plan_sized(size, ta, tf, tr.t_end, o, largest, granule)
        torch.cuda.synchronize()
        assert int(out["status"].item()) == 0
        assert np.array_equal(out["offsets"].cpu().numpy().view(np.uint64), a), name
        assert np.array_equal(out["peaks"].cpu().numpy().view(np.uint64), ext), name
        kinds[name] = (S.stalloc_plan_report(out)["kernel"], out["workspace_bytes"])
    assert kinds["true"] == ("bitmap", plain["workspace_bytes"])
    assert kinds["ruled out"][0] == kinds["no granule known"][0] == "list_lds"
    assert kinds["ruled out"][1] == kinds["no granule known"][1] < plain["workspace_bytes"] - 70_000_000
    for largest, granule in ((0, 512), (4096, 0), (4096, 768)):
        with pytest.raises(S.StallocError) as err:
            S.stalloc_plan_sized(size, ta, tf, tr.t_end, o, largest, granule)
        assert err.value.code == 1


def test_validate_reports_an_address_range_that_would_wrap(S, oracle):
    """A corrupted plan with an address near 2^64: offset + size wraps to a small number and the block
    would look disjoint from everything.  The call reports it and still counts what the block covers."""
    rng = np.random.default_rng(811)
    n = 700
    size, ts, te, t_end = random_trace(rng, n, t_max=40, sizes=[4, 8, 12])
    tr = _T(size, ts, te, t_end)
    a, _ = oracle.plan_many(size, ts, te, np.arange(n, dtype=np.uint32)[None, :], threads=1, method="lists")
    cnt, pair = _gpu_validate(S, tr, a)
    assert int(cnt[0]) == 0
    for victim in (0, 300, n - 1):
        bad = np.concatenate([a, a])
        bad[1, victim] = np.uint64(2 ** 64 - 1) - size[victim] + np.uint64(1)      # ends exactly at 2^64: wraps to 0
        cnt, pair = _gpu_validate(S, tr, bad, want_status=3)
        assert int(cnt[0]) == 0
        # up to 2^64 - 1 the range is still counted: a second block planted inside it conflicts with it
        other = int(np.flatnonzero((ts < te[victim]) & (ts[victim] < te) & (np.arange(n) != victim))[0])
        bad[1, other] = np.uint64(2 ** 64 - 2) - size[other]
        cnt, pair = _gpu_validate(S, tr, bad, want_status=3)
        assert int(cnt[1]) == 1 and tuple(int(x) for x in pair[1]) == (min(victim, other), max(victim, other))


# --------------------------------------------------------------------------- plan

@pytest.mark.parametrize("name", ["running_max.txt", "hole_and_tie.txt", "gap_fit.txt"])
def test_plan_hand_worked_examples(S, name):
    g = load_golden(name)
    tr = _T(g["size"], g["t_s"], g["t_e"], g["t_end"])
    orders = np.asarray([c["order"] for c in g["cases"]], np.uint32)
    got = _gpu_plan(S, tr, orders)
    assert got["status"] == 0
    assert got["offsets"].tolist() == [c["a"] for c in g["cases"]]
    assert got["peaks"].tolist() == [c["extent"] for c in g["cases"]]
    status, lb, t_at = _gpu_lower_bound(S, tr)
    assert (lb, t_at) == g["max_live"]


def test_plan_config1_all_orderings(S, oracle):
    tr = make_trace(1)
    orders = make_orderings(tr, CONFIGS[1].n_orderings)
    got, a, ext = _compare_plans(S, oracle, tr, orders, method="allpairs")
    cnt, pair = _gpu_validate(S, tr, got["offsets"])
    assert not cnt.any()


def test_plan_config2_all_orderings(S, oracle):
    """Full size of the benchmark workload: 6144 requests x 1024 orders, every address compared."""
    tr = make_trace(2)
    orders = make_orderings(tr, CONFIGS[2].n_orderings)
    got, a, ext = _compare_plans(S, oracle, tr, orders, method="lists")
    cnt, pair = _gpu_validate(S, tr, got["offsets"])
    assert not cnt.any() and (pair == 0xFFFFFFFF).all()
    status, lb, _ = _gpu_lower_bound(S, tr)
    assert (got["peaks"] >= lb).all()
    # no outputs wanted except extents and the best plan
    lean = _gpu_plan(S, tr, orders, want_offsets=False)
    assert np.array_equal(lean["peaks"], ext) and np.array_equal(lean["best_offsets"], got["best_offsets"])


@pytest.mark.parametrize("wide", [False, "coarse", "medium", True])
@pytest.mark.parametrize("seed", range(12))
def test_plan_random_traces(S, oracle, seed, wide):
    """Ties in timestamps, single requests, list lengths around wave / workgroup / batch sizes.
    False: sizes of 1-8 granules (bitmap variant); "coarse": 33-264 granules (sorted list, 16-bit
    cells while the sum stays below 2^16 granules); "medium": more than 2^16 granules (32-bit cells);
    True: odd byte sizes with a sum far above 2^31, which forces 64-bit addresses in the kernel."""
    rng = np.random.default_rng(900 + seed)
    n = [1, 2, 63, 64, 65, 127, 129, 1023, 1025, 2049, 700, 3000][seed]
    size, ts, te, t_end = random_trace(rng, n, t_max=max(4, n // 3), unique_times=(seed % 2 == 1))
    size = size * np.uint64(512)
    if wide == "coarse":
        size = size * np.uint64(33)
    elif wide == "medium":
        size = size * np.uint64(70001)
    elif wide:
        size = size * np.uint64(2 ** 31 + 12345) + np.uint64(1)
    tr = _T(size, ts, te, t_end)
    P = 9
    orders = np.stack([rng.permutation(n) for _ in range(P)]).astype(np.uint32)
    orders[0] = np.argsort(-size.astype(np.int64), kind="stable")
    orders[1] = np.argsort(ts, kind="stable")
    _compare_plans(S, oracle, tr, orders, method="allpairs")


def test_plan_closed_forms(S):
    rng = np.random.default_rng(950)
    n = 300
    size = (rng.integers(1, 1000, n) * 512).astype(np.uint64)
    order = rng.permutation(n).astype(np.uint32)[None, :]
    clique = _T(size, np.zeros(n, np.uint32), np.full(n, 7, np.uint32), 7)
    got = _gpu_plan(S, clique, order)
    expect = np.zeros(n, np.uint64)
    expect[order[0]] = np.concatenate([[0], np.cumsum(size[order[0]])[:-1]]).astype(np.uint64)
    assert np.array_equal(got["offsets"][0], expect) and int(got["peaks"][0]) == int(size.sum())
    ts = (np.arange(n) * 2).astype(np.uint32)
    disjoint = _T(size, ts, ts + np.uint32(2), 2 * n)
    got = _gpu_plan(S, disjoint, order)
    assert not got["offsets"].any() and int(got["peaks"][0]) == int(size.max())


def _nudge_to_sum(sizes, total, lo, hi, keep=()):
    """Moves entries (not those in `keep`) one by one within [lo, hi] until the sum is `total`."""
    sizes = sizes.copy()
    while int(sizes.sum()) != total:
        step = 1 if total > int(sizes.sum()) else -1
        before = int(sizes.sum())
        for i in range(len(sizes)):
            if int(sizes.sum()) == total:
                break
            if i not in keep and lo <= sizes[i] + step <= hi:
                sizes[i] += step
        assert int(sizes.sum()) != before, "cannot reach the requested sum"
    return sizes


def test_plan_bitmap_full_address_range(S):
    """Occupancy-bitmap variant at its limits: a clique whose extent is the whole 32704-granule
    range (closed form: prefix sums in placement order), blocks of the longest size allowed."""
    rng = np.random.default_rng(960)
    g = 1 << 20
    sizes = rng.integers(25, 31, 1200)
    sizes = np.append(sizes[np.cumsum(sizes) <= 32704 - 31], 31)
    sizes = _nudge_to_sum(sizes, 32704, 1, 31)
    assert sizes.max() == 31
    n = len(sizes)
    size = (sizes * g).astype(np.uint64)
    clique = _T(size, np.zeros(n, np.uint32), np.full(n, 5, np.uint32), 5)
    order = rng.permutation(n).astype(np.uint32)[None, :]
    got = _gpu_plan(S, clique, order)
    assert got["info"]["kernel"] == "bitmap"
    expect = np.zeros(n, np.uint64)
    expect[order[0]] = np.concatenate([[0], np.cumsum(size[order[0]])[:-1]]).astype(np.uint64)
    assert np.array_equal(got["offsets"][0], expect) and int(got["peaks"][0]) == 32704 * g


@pytest.mark.parametrize("n,largest,total,bitmap", [(2500, 31, 32704, True), (2500, 32, 32704, False),
                                                     (9000, 31, 200000, True)])
def test_plan_bitmap_applicability_limits(S, oracle, n, largest, total, bitmap):
    """Just inside and just outside what the bitmap variant takes (no size above 31 granules), and an
    address range that only the one-workgroup-per-CU shape can hold: the plans are the oracle's."""
    rng = np.random.default_rng(961 + n + largest)
    sizes = rng.integers(1, 26, n)
    sizes[7] = largest
    sizes = _nudge_to_sum(sizes, total, 1, 30, keep=(7,))
    assert int(sizes.sum()) == total and sizes.max() == largest
    _, ts, te, t_end = random_trace(rng, n, t_max=400)
    tr = _T((sizes * 4096).astype(np.uint64), ts, te, t_end)
    orders = np.stack([rng.permutation(n) for _ in range(5)]).astype(np.uint32)
    orders[0] = np.argsort(-sizes, kind="stable")
    got, _, _ = _compare_plans(S, oracle, tr, orders, method="allpairs")
    assert (got["info"]["kernel"] == "bitmap") == bitmap


def test_plan_bitmap_tall_plans_small_pool(S, oracle):
    """Many requests (the per-plan table leaves little LDS for bitmaps) and extents that grow to
    ~30000 granules: the batches shrink as the bitmaps get longer."""
    rng = np.random.default_rng(962)
    n = 8500
    sizes = rng.integers(1, 7, n)
    sizes[rng.choice(n, 20, replace=False)] = 31
    assert int(sizes.sum()) <= 32704
    ts = rng.integers(0, 50, n)
    te = ts + rng.integers(150, 200, n)
    short = rng.random(n) < 0.2                         # a fifth lives briefly: holes open up under the rest
    te[short] = ts[short] + rng.integers(1, 4, int(short.sum()))
    tr = _T((sizes * 65536).astype(np.uint64), ts.astype(np.uint32), te.astype(np.uint32), int(te.max()))
    orders = np.stack([rng.permutation(n) for _ in range(3)]).astype(np.uint32)
    orders[0] = np.argsort(-sizes, kind="stable")
    got, a, ext = _compare_plans(S, oracle, tr, orders, method="allpairs")
    assert got["info"]["kernel"] == "bitmap"
    assert int(ext.max()) // 65536 > 20000


def test_plan_config3_sampled_orderings(S, oracle):
    """Config 3 (19 840 requests, 86 748 granules: bitmap variant, one workgroup per CU): sampled
    orders, every address compared."""
    tr = make_trace(3)
    rows = [0, 1, 2, 3, 4, 1025, 2046, 2047]
    orders = make_orderings(tr, CONFIGS[3].n_orderings, rows=rows)
    lists = oracle.conflict_lists(tr.t_alloc, tr.t_free)
    got, a, ext = _compare_plans(S, oracle, tr, orders, method="lists", lists=lists)
    assert got["info"]["kernel"] == "bitmap"
    cnt, _ = _gpu_validate(S, tr, got["offsets"])
    assert not cnt.any()


_FULL = {}       # configuration -> what its full launch gave (kept between the parts of a test)


def _full_launch(S, cfg):
    """All orders of a configuration in one call, as the benchmark launches them: the orders made on the
    device, every plan checked over all pairs by stalloc_validate, the lower bound beside them."""
    import torch
    if cfg in _FULL:
        return _FULL[cfg]
    _FULL.clear()                                             # one configuration's arrays at a time
    tr = make_trace(cfg)
    P = CONFIGS[cfg].n_orderings
    size, ta, tf = S.trace_to_device(tr)
    made = S.stalloc_make_orders(size, ta, tf, tr.t_end, P)
    plan = S.stalloc_plan(size, ta, tf, tr.t_end, made["orders"], want_best_offsets=False)
    val = S.stalloc_validate(size, ta, tf, tr.t_end, plan["offsets"])
    lb = S.stalloc_lower_bound(size, ta, tf, tr.t_end)
    torch.cuda.synchronize()
    assert [int(x["status"].item()) for x in (made, plan, val, lb)] == [0, 0, 0, 0]
    res = {"tr": tr, "P": P, "made": made, "plan": plan, "info": S.stalloc_plan_report(plan),
           "conflicts": val["conflicts"].cpu().numpy().view(np.uint64),
           "peaks": plan["peaks"].cpu().numpy().view(np.uint64), "best_plan": int(plan["best_plan"].item()),
           "lower_bound": int(lb["lower_bound"].item())}
    _FULL[cfg] = res
    return res


def _compare_rows_of_full_launch(S, oracle, cfg, rows):
    full = _full_launch(S, cfg)
    tr, P = full["tr"], full["P"]
    assert not full["conflicts"].any()
    assert (full["peaks"] >= np.uint64(full["lower_bound"])).all()
    assert full["best_plan"] == int(np.argmin(full["peaks"]))
    rows = np.asarray(rows)
    orders = full["made"]["orders"][rows].cpu().numpy().view(np.uint32)
    assert np.array_equal(orders[:4], make_orderings(tr, P, rows=rows[:4]))       # the rows the host would make
    lists = oracle.conflict_lists(tr.t_alloc, tr.t_free)
    a, ext = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, orders, threads=THREADS, method="lists", lists=lists)
    assert np.array_equal(full["peaks"][rows], ext)
    got = full["plan"]["offsets"][rows].cpu().numpy().view(np.uint64)
    bad = np.nonzero((got != a).any(axis=1))[0]
    assert bad.size == 0, f"addresses differ in plans {rows[bad][:8]}"
    return full


@pytest.mark.parametrize("part", range(4))
def test_plan_config3_full_launch_every_ordering(S, oracle, part):
    """All 2048 orders of config 3 in one call (more orders than resident workgroups), every plan
    compared with the oracle address by address, 512 plans per part of this test."""
    full = _compare_rows_of_full_launch(S, oracle, 3, np.arange(512 * part, 512 * (part + 1)))
    assert full["info"]["kernel"] == "bitmap"


def _stratified(P):
    """Rows 0, 1, 2 and every ceil(P / 64)-th row."""
    return np.unique(np.r_[0, 1, 2, np.arange(0, P, -(-P // 64))])


def test_plan_config4_full_launch_stratified_orderings(S, oracle):
    """Config 4 (47 748 requests, 1229 distinct sizes) with all its 2048 orders: rows 0-2 and every 32nd
    row compared address by address, every plan of the launch checked for conflicts over all pairs."""
    full = _compare_rows_of_full_launch(S, oracle, 4, _stratified(2048))
    assert full["info"]["kernel"] == "list_memory" and full["info"]["plans_64bit"] == 0


@pytest.mark.parametrize("half", range(2))
def test_plan_config5_full_launch_stratified_orderings(S, oracle, half):
    """Config 5 (199 748 requests) with all its 4096 orders in one call: rows 0-2 and every 64th row
    compared address by address (in two halves), all 4096 plans checked over all n(n-1)/2 pairs."""
    rows = _stratified(4096)
    full = _compare_rows_of_full_launch(S, oracle, 5, rows[half::2])
    assert full["info"]["kernel"] == "long_list" and full["info"]["plans_64bit"] == 0
    assert full["info"]["lifetime_threshold"] == 15 and full["info"]["long_requests"] == 4271
    # the short-lived requests of 128 MiB and more (nothing between 64 KiB and them) have a table of their own
    tr = make_trace(5)
    short = tr.t_free.astype(np.int64) - tr.t_alloc <= 15
    assert full["info"]["large_size"] == 1 << 27
    assert full["info"]["large_requests"] == int((short & (tr.size >= 1 << 27)).sum()) > 0
    assert full["info"]["list_entry_bytes"] == 8                           # (six sizes among the 4271 long-lived requests)


@pytest.mark.parametrize("n_clique,n_extra,unit,fill", [(230, 70, 1 << 24, 0.80), (230, 70, 1 << 24, 0.875),
                                                         (230, 70, 1 << 24, 0.885), (9000, 1500, 1 << 18, 0.970),
                                                         (9000, 1500, 1 << 18, 0.9711), (9000, 1500, 1 << 18, 0.972)])
def test_plan_32_bit_counts_tried_plan_by_plan(S, oracle, n_clique, n_extra, unit, fill):
    """Odd byte sizes whose sum exceeds 2^32 while no request is large: the 32-bit list kernel takes every
    plan as far as its extent certainly fits 32 bits and leaves the others to the 64-bit kernel.  The
    traces stack a clique of `fill` x 2^32 bytes plus shorter-lived requests, so that, from one case to
    the next, none, some or all of the plans end above 2^32 (list in LDS for 300 requests, in the
    workspace for 10 500)."""
    rng = np.random.default_rng(5)
    size = np.concatenate([rng.integers(unit // 2, unit * 3 // 2, n_clique),
                           rng.integers(unit // 4, unit * 2, n_extra)]).astype(np.uint64) | np.uint64(1)
    scale = fill * 2 ** 32 / int(size[:n_clique].sum())
    size[:n_clique] = (size[:n_clique].astype(np.float64) * scale).astype(np.uint64) | np.uint64(1)
    ts = np.concatenate([np.zeros(n_clique, np.int64), rng.integers(0, 90, n_extra)])
    te = np.concatenate([np.full(n_clique, 100, np.int64), ts[n_clique:] + rng.integers(1, 40, n_extra)])
    n = n_clique + n_extra
    tr = Trace(name="near 2^32", size=size, t_alloc=ts.astype(np.uint32), t_free=te.astype(np.uint32), t_end=int(te.max()))
    rng = np.random.default_rng(9)
    orders = np.stack([rng.permutation(n) for _ in range(12 if n < 5000 else 6)]).astype(np.uint32)
    got, a, ext = _compare_plans(S, oracle, tr, orders, method="allpairs")
    info = got["info"]
    assert info["kernel"] == ("list_lds" if n < 5000 else "list_memory") and info["address_bits"] == 32
    assert info["granule_log2"] == 0 and info["granules"] >= 2 ** 31          # 32-bit counts are tried plan by plan
    above = int((ext > np.uint64(2 ** 32)).sum())
    assert (fill < 0.87 and above == 0) or (fill > 0.88 and above > 0) or 0.87 <= fill <= 0.88 or n > 5000
    cnt, _ = _gpu_validate(S, tr, got["offsets"])
    assert not cnt.any()


def test_plan_second_workload_sampled_orderings(S, oracle):
    """Iterations back to back, persistent tensors that overlap every request, a coarse clock with
    thousands of tied timestamps: two iterations of config 2 (occupancy-bitmap kernel) and the MoE
    stage (sorted-list kernel)."""
    for cfg, rows in ((6, [0, 1, 2, 3, 4, 511, 1022, 1023]), (7, [0, 3, 2046])):
        tr = make_trace(cfg)
        orders = make_orderings(tr, CONFIGS[cfg].n_orderings, rows=rows)
        lists = oracle.conflict_lists(tr.t_alloc, tr.t_free)
        got, a, ext = _compare_plans(S, oracle, tr, orders, method="lists", lists=lists)
        del lists
        assert got["info"]["kernel"] == ("bitmap" if cfg == 6 else "list_memory")
        cnt, _ = _gpu_validate(S, tr, got["offsets"])
        assert not cnt.any()
        status, lb, t_at = _gpu_lower_bound(S, tr)
        assert status == 0 and (got["peaks"] >= lb).all()
        assert (int(lb), int(t_at)) == oracle.lower_bound(tr.size, tr.t_alloc, tr.t_free, tr.t_end)


def test_validate_config5_best_plan_and_a_corrupted_copy(S, oracle):
    """Largest trace: the best of a few plans validated over all n(n-1)/2 pairs, and a corrupted copy
    against the oracle's count and first pair."""
    tr = make_trace(5)
    rows = [0, 3]
    orders = make_orderings(tr, CONFIGS[5].n_orderings, rows=rows)
    got = _gpu_plan(S, tr, orders)
    assert got["status"] == 0
    best = got["best_offsets"][None, :]
    cnt, pair = _gpu_validate(S, tr, best)
    assert int(cnt[0]) == 0 and tuple(int(x) for x in pair[0]) == NONE_PAIR
    rng = np.random.default_rng(555)
    bad = best.copy()
    for i in rng.choice(tr.n, size=5, replace=False):
        bad[0, i] = rng.integers(0, int(best.max()))
    cnt, pair = _gpu_validate(S, tr, bad)
    assert (int(cnt[0]), tuple(int(x) for x in pair[0])) == oracle.validate(tr.size, tr.t_alloc, tr.t_free, bad[0])


@pytest.mark.parametrize("wide", [False, True])
def test_plan_list_beyond_lds(S, oracle, wide):
    """A random trace too long for the LDS-resident sorted list (and with a size above 31 granules, which
    rules the bitmap variant out), with 32-bit and with 64-bit addresses."""
    rng = np.random.default_rng(960 + int(wide))
    n = 11000
    assert n > S.lib.stalloc_plan_lds_capacity()
    size, ts, te, t_end = random_trace(rng, n, t_max=2000, sizes=[1, 2, 3, 5, 8, 13, 40])
    size = size * np.uint64(4096)
    if wide:
        size = size * np.uint64(2 ** 31 + 7) + np.uint64(1)
    tr = _T(size, ts, te, t_end)
    orders = np.stack([rng.permutation(n) for _ in range(4)]).astype(np.uint32)
    orders[0] = np.argsort(-size.astype(np.int64), kind="stable")
    got, _, _ = _compare_plans(S, oracle, tr, orders, method="lists")
    assert got["info"]["kernel"] == "list_memory" and got["info"]["address_bits"] == (64 if wide else 32)


@pytest.mark.parametrize("sizes", [[1, 2, 3, 4], [1, 2, 3, 40]])
def test_plan_more_orders_than_resident_workgroups(S, oracle, sizes):
    """5000 orders of a small trace: every workgroup places several plans in a row (per-plan state
    must start clean), in the bitmap kernel (sizes up to 4 granules) and in the sorted-list kernel."""
    rng = np.random.default_rng(970)
    n = 150
    size, ts, te, t_end = random_trace(rng, n, t_max=60, sizes=sizes)
    tr = _T(size * np.uint64(1024), ts, te, t_end)
    P = 5000
    orders = np.stack([rng.permutation(n) for _ in range(P)]).astype(np.uint32)
    got, _, _ = _compare_plans(S, oracle, tr, orders, method="allpairs")
    assert (got["info"]["kernel"] == "bitmap") == (max(sizes) <= 31)


def test_plan_reports_malformed_inputs(S):
    g = load_golden("gap_fit.txt")
    orders = np.asarray([g["cases"][0]["order"]], np.uint32)
    size = g["size"].copy(); size[2] = 0
    assert _gpu_plan(S, _T(size, g["t_s"], g["t_e"], g["t_end"]), orders)["status"] == 2
    te = g["t_e"].copy(); te[1] = g["t_s"][1]
    assert _gpu_plan(S, _T(g["size"], g["t_s"], te, g["t_end"]), orders)["status"] == 2
    assert _gpu_plan(S, _T(g["size"], g["t_s"], g["t_e"], g["t_end"] - 1), orders)["status"] == 2
    big = g["size"].copy(); big[:] = 2 ** 61
    assert _gpu_plan(S, _T(big, g["t_s"], g["t_e"], g["t_end"]), orders)["status"] == 3
    bad_order = orders.copy(); bad_order[0, 3] = 6
    assert _gpu_plan(S, _T(g["size"], g["t_s"], g["t_e"], g["t_end"]), bad_order)["status"] == 6
    assert _gpu_lower_bound(S, _T(size, g["t_s"], g["t_e"], g["t_end"]))[0] == 2


def test_plan_is_deterministic(S):
    tr = make_trace(2)
    orders = make_orderings(tr, 64)
    a = _gpu_plan(S, tr, orders)
    b = _gpu_plan(S, tr, orders)
    assert np.array_equal(a["offsets"], b["offsets"]) and np.array_equal(a["peaks"], b["peaks"])
