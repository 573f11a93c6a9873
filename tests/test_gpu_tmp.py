"""stalloc_tmp (through the C ABI) against the oracle's exact ratio (Eq. 2).  Tolerance: the kernel sums
the numerator exactly and then rounds at most eight times in double precision (three limb conversions,
two additions, the extent, the denominator's product, the division): 10 * 2^-53 relative."""
import numpy as np
import pytest

from helpers import random_trace
from workloads import CONFIGS, make_orderings, make_trace

pytestmark = pytest.mark.gpu
REL = 10 * 2.0 ** -53


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    return S


def _gpu_tmp(S, size, ts, te, t_end, extents):
    import torch
    d = lambda x, t: torch.from_numpy(np.ascontiguousarray(x).view(t)).cuda()
    out = S.stalloc_tmp(d(size, np.int64), d(ts, np.int32), d(te, np.int32), t_end, d(np.asarray(extents, np.uint64), np.int64))
    torch.cuda.synchronize()
    return int(out["status"].item()), out["tmp"].cpu().numpy()


@pytest.mark.parametrize("seed", range(8))
def test_random_plans(S, oracle, seed):
    rng = np.random.default_rng(9300 + seed)
    n = [1, 2, 64, 65, 300, 1000, 1025, 5000][seed]
    size, ts, te, t_end = random_trace(rng, n, t_max=max(4, n // 2), unique_times=(seed % 2 == 1))
    if seed % 3 == 0:
        size = size * np.uint64(1 << 40) + np.uint64(512)            # products beyond 64 bits
        ts, te = ts * np.uint32(100000), te * np.uint32(100000)
        t_end *= 100000
    orders = np.stack([rng.permutation(n) for _ in range(5)]).astype(np.uint32)
    a, ext = oracle.plan_many(size, ts, te, orders, threads=4, method="allpairs")
    status, got = _gpu_tmp(S, size, ts, te, t_end, ext)
    assert status == 0
    for p in range(5):
        want = oracle.tmp(size, ts, te, a[p])
        assert abs(got[p] - want) <= REL * want, (p, got[p], want)


@pytest.mark.parametrize("cfg", [2, 5])
def test_configs_with_extents_from_the_plan_kernel(S, oracle, cfg):
    import torch
    tr = make_trace(cfg)
    rows = [0, 1, 2, 3, 4] if cfg == 2 else [0, 2]
    orders = make_orderings(tr, CONFIGS[cfg].n_orderings, rows=rows)
    size, ta, tf = S.trace_to_device(tr)
    plan = S.stalloc_plan(size, ta, tf, tr.t_end, torch.from_numpy(orders.view(np.int32)).cuda())
    out = S.stalloc_tmp(size, ta, tf, tr.t_end, plan["peaks"])
    torch.cuda.synchronize()
    assert int(plan["status"].item()) == 0 and int(out["status"].item()) == 0
    offsets = plan["offsets"].cpu().numpy().view(np.uint64)
    got = out["tmp"].cpu().numpy()
    for p in range(len(rows)):
        want = oracle.tmp(tr.size, tr.t_alloc, tr.t_free, offsets[p])
        assert abs(got[p] - want) <= REL * want and 0.0 < got[p] <= 1.0


def test_reports_malformed_trace(S):
    size = np.array([8, 0, 8], np.uint64)
    status, _ = _gpu_tmp(S, size, np.array([0, 1, 2], np.uint32), np.array([3, 4, 5], np.uint32), 5, [16])
    assert status == 2                                                   # STALLOC_ERR_BAD_TRACE
