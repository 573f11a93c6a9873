"""stalloc_make_orders (through the C ABI) against the oracle's orders, entry by entry."""
import numpy as np
import pytest

from helpers import random_trace
from workloads import CONFIGS, make_orderings, make_trace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    return S


def _gpu_orders(S, size, ts, te, t_end, P, seed=1000, first_plan=0):
    import torch
    d = lambda x, t: torch.from_numpy(np.ascontiguousarray(x).view(t)).cuda()
    out = S.stalloc_make_orders(d(size, np.int64), d(ts, np.int32), d(te, np.int32), t_end, P, seed=seed, first_plan=first_plan)
    torch.cuda.synchronize()
    return int(out["status"].item()), out["orders"].cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("seed", range(10))
def test_random_traces(S, oracle, seed):
    """Counts around the tile size and its multiples (partial tiles, odd numbers of runs to merge),
    few and many sizes, tied and unique times, sizes above 2^32."""
    rng = np.random.default_rng(9400 + seed)
    n = [1, 2, 255, 256, 257, 768, 769, 1000, 3000, 5121][seed]
    sizes = [[8, 16, 24], None, list(range(1, 60))][seed % 3]
    size, ts, te, t_end = random_trace(rng, n, t_max=max(4, n // 3), unique_times=(seed % 2 == 1), sizes=sizes)
    if seed % 4 == 0:
        size = size * np.uint64(1 << 33) + np.uint64(512)
    P = 21
    status, got = _gpu_orders(S, size, ts, te, t_end, P, seed=40 + seed)
    assert status == 0
    assert np.array_equal(got, oracle.make_orders(size, ts, te, P, seed=40 + seed))
    status, got = _gpu_orders(S, size, ts, te, t_end, 6, seed=40 + seed, first_plan=1001)
    assert status == 0
    assert np.array_equal(got, oracle.make_orders(size, ts, te, 6, seed=40 + seed, first_plan=1001))


@pytest.mark.parametrize("cfg", [1, 2])
def test_all_orders_of_small_configs(S, oracle, cfg):
    tr = make_trace(cfg)
    P = CONFIGS[cfg].n_orderings
    status, got = _gpu_orders(S, tr.size, tr.t_alloc, tr.t_free, tr.t_end, P)
    assert status == 0
    assert np.array_equal(got, oracle.make_orders(tr.size, tr.t_alloc, tr.t_free, P))
    assert np.array_equal(got, make_orderings(tr, P))          # the arrays the benchmark feeds from the host


@pytest.mark.parametrize("cfg,first,P", [(3, 0, 12), (3, 2040, 8), (4, 0, 6), (5, 0, 4), (5, 3900, 196), (6, 500, 10)])
def test_windows_of_rows_of_large_configs(S, oracle, cfg, first, P):
    """(5, 3900, 196): more rows than one batch of sort buffers holds."""
    tr = make_trace(cfg)
    status, got = _gpu_orders(S, tr.size, tr.t_alloc, tr.t_free, tr.t_end, P, first_plan=first)
    assert status == 0
    assert np.array_equal(got, oracle.make_orders(tr.size, tr.t_alloc, tr.t_free, P, first_plan=first))


def test_orders_feed_the_placement(S, oracle):
    """Orders made on the device, planned on the device: the same plans as from the host's arrays."""
    import torch
    tr = make_trace(1)
    size, ta, tf = S.trace_to_device(tr)
    made = S.stalloc_make_orders(size, ta, tf, tr.t_end, 64)
    plan = S.stalloc_plan(size, ta, tf, tr.t_end, made["orders"])
    torch.cuda.synchronize()
    assert int(made["status"].item()) == 0 and int(plan["status"].item()) == 0
    a, ext = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, oracle.make_orders(tr.size, tr.t_alloc, tr.t_free, 64),
                              threads=4, method="allpairs")
    assert np.array_equal(plan["offsets"].cpu().numpy().view(np.uint64), a)
    assert np.array_equal(plan["peaks"].cpu().numpy().view(np.uint64), ext)


def test_reports_malformed_trace(S):
    size = np.array([8, 0, 8], np.uint64)
    status, _ = _gpu_orders(S, size, np.array([0, 1, 2], np.uint32), np.array([3, 4, 5], np.uint32), 5, 4)
    assert status == 2                                                   # STALLOC_ERR_BAD_TRACE
