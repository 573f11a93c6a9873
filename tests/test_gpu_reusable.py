"""Parity of stalloc_reusable_space (through the C ABI) with the CPU oracle: interval by interval,
counts and idle bytes, on the same seeded plans and windows."""
import os

import numpy as np
import pytest

from helpers import random_trace
from test_oracle_reusable import load_reusable_golden
from workloads import CONFIGS, make_orderings, make_trace, make_windows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    return S


def _gpu(S, size, ts, te, t_end, a, windows, cap):
    import torch
    d = lambda x, t: torch.from_numpy(np.ascontiguousarray(x).view(t)).cuda()
    out = S.stalloc_reusable_space(d(size, np.int64), d(ts, np.int32), d(te, np.int32), t_end, d(a, np.int64),
                                   d(np.asarray(windows, np.uint32), np.int32), cap)
    torch.cuda.synchronize()
    status = int(out["status"].item())
    if status:
        return status, None, None, None
    ranges = out["ranges"].cpu().numpy().view(np.uint64) if cap else None
    return 0, ranges, out["counts"].cpu().numpy().view(np.uint32), out["idle_bytes"].cpu().numpy().view(np.uint64)


def _compare(S, oracle, size, ts, te, t_end, a, windows, cap, sample=None):
    status, ranges, counts, idle = _gpu(S, size, ts, te, t_end, a, windows, cap)
    assert status == 0
    which = range(len(windows)) if sample is None else sample
    for w in which:
        r, c, i = oracle.reusable_space(size, ts, te, a, (int(windows[w][0]), int(windows[w][1])), cap=cap)
        assert int(counts[w]) == c and int(idle[w]) == i, (w, windows[w])
        if cap:
            assert np.array_equal(ranges[w, :min(c, cap)], r), (w, windows[w])


def test_hand_worked_windows(S, oracle):
    size, ts, te, a, windows = load_reusable_golden()
    w = np.asarray([x[0] for x in windows], np.uint32)
    status, ranges, counts, idle = _gpu(S, size, ts, te, int(te.max()), a, w, 8)
    assert status == 0
    for q, (_, expect) in enumerate(windows):
        assert int(counts[q]) == len(expect) and np.array_equal(ranges[q, :len(expect)], expect)
        assert int(idle[q]) == int((expect[:, 1] - expect[:, 0]).sum())


@pytest.mark.parametrize("seed", range(10))
def test_random_decisions(S, oracle, seed):
    """Decisions that need not form a valid plan (the definition only unions ranges): equal addresses,
    nested and touching blocks, sizes from a byte to 2^40, counts around wave and workgroup sizes."""
    rng = np.random.default_rng(4000 + seed)
    n = [1, 2, 63, 64, 65, 255, 257, 1000, 3000, 7000][seed]
    size, ts, te, t_end = random_trace(rng, n, t_max=max(4, n // 2), unique_times=(seed % 2 == 1))
    if seed % 3 == 0:
        size = size * np.uint64(1 << 37)
    a = (rng.integers(0, max(2, 4 * n), n).astype(np.uint64)) * (size.max() if seed % 3 == 0 else np.uint64(1))
    k = 40
    lo = rng.integers(0, t_end, k)
    hi = np.minimum(lo + rng.integers(1, max(2, t_end // 2), k), t_end + 3)
    windows = np.stack([lo, hi], axis=1).astype(np.uint32)
    _compare(S, oracle, size, ts, te, t_end, a, windows, cap=n + 1)
    _compare(S, oracle, size, ts, te, t_end, a, windows, cap=3)          # truncated rows, full counts


@pytest.mark.parametrize("cfg", [1, 2])
def test_best_plans_of_configs(S, oracle, cfg):
    tr = make_trace(cfg)
    order = make_orderings(tr, CONFIGS[cfg].n_orderings, rows=[0])[0]
    a, extent = oracle.plan_allpairs(tr.size, tr.t_alloc, tr.t_free, order)
    windows = make_windows(tr, 256, seed=7000 + cfg)
    _compare(S, oracle, tr.size, tr.t_alloc, tr.t_free, tr.t_end, a, windows, cap=tr.n + 1)
    # over the whole iteration a lowest-fit plan leaves nothing idle
    status, _, counts, idle = _gpu(S, tr.size, tr.t_alloc, tr.t_free, tr.t_end, a, np.array([[0, tr.t_end]]), 4)
    assert status == 0 and int(counts[0]) == 0 and int(idle[0]) == 0


@pytest.mark.parametrize("cfg", [3, 5])
def test_large_configs_sampled_windows(S, oracle, cfg):
    """Full-size plans (size-descending order through the GPU placement kernel, itself checked against the
    oracle elsewhere; here only its addresses matter as an input): sampled windows, every interval compared."""
    import torch
    tr = make_trace(cfg)
    order = make_orderings(tr, CONFIGS[cfg].n_orderings, rows=[0])
    size, ta, tf = S.trace_to_device(tr)
    plan = S.stalloc_plan(size, ta, tf, tr.t_end, torch.from_numpy(order.view(np.int32)).cuda())
    torch.cuda.synchronize()
    a = plan["best_offsets"].cpu().numpy().view(np.uint64)
    windows = make_windows(tr, 512, seed=7000 + cfg)
    _compare(S, oracle, tr.size, tr.t_alloc, tr.t_free, tr.t_end, a, windows, cap=4096, sample=range(0, 512, 16))


def test_more_windows_than_resident_workgroups(S, oracle):
    """6000 windows over a small plan: every workgroup answers several windows in a row."""
    tr = make_trace(1)
    order = make_orderings(tr, CONFIGS[1].n_orderings, rows=[1])[0]
    a, _ = oracle.plan_allpairs(tr.size, tr.t_alloc, tr.t_free, order)
    rng = np.random.default_rng(4100)
    lo = rng.integers(0, tr.t_end, 6000)
    hi = np.minimum(lo + rng.integers(1, 40, 6000), tr.t_end)
    lo = np.minimum(lo, hi - 1)
    windows = np.stack([lo, hi], axis=1).astype(np.uint32)
    _compare(S, oracle, tr.size, tr.t_alloc, tr.t_free, tr.t_end, a, windows, cap=16)


@pytest.mark.parametrize("seed", range(6))
def test_thousands_of_windows(S, oracle, seed):
    """From 2^23 decisions x windows on, a lane takes a window and a wave 64 of them over a part of the
    sorted plan: ragged last groups and parts, tied and unique times, truncated rows; pools that 32-bit
    counts of their address unit cover (the usual case) and pools that need 64-bit byte addresses."""
    rng = np.random.default_rng(4200 + seed)
    n = [131, 300, 1025, 4099, 5000, 20000][seed]
    k = [64100, 28001, 8200, 2049, 2560, 2050][seed]
    size, ts, te, t_end = random_trace(rng, n, t_max=max(4, n // 2), unique_times=(seed % 2 == 1))
    if seed % 3 == 0:
        size = size * np.uint64(1 << 37)
    a = (rng.integers(0, max(2, 4 * n), n).astype(np.uint64)) * (size.max() if seed % 3 == 0 else np.uint64(1))
    if seed in (1, 4):                                   # odd byte addresses over 2 TB: no 32-bit unit covers the pool
        a = rng.integers(0, 1 << 41, n).astype(np.uint64) | np.uint64(1)
    lo = rng.integers(0, t_end, k)
    hi = np.minimum(lo + np.exp(rng.uniform(0, np.log(max(2, t_end // 2)), k)).astype(np.int64), t_end + 3)
    windows = np.stack([lo, np.maximum(hi, lo + 1)], axis=1).astype(np.uint32)
    sample = None if k <= 3000 and n <= 5000 else range(seed, k, max(1, k // 1500))
    _compare(S, oracle, size, ts, te, t_end, a, windows, cap=64, sample=sample)
    _compare(S, oracle, size, ts, te, t_end, a, windows, cap=2, sample=range(0, k, max(5, k // 500)))
    status, ranges, counts, idle = _gpu(S, size, ts, te, t_end, a, windows, 0)       # counts and idle bytes only
    assert status == 0 and ranges is None
    for w in range(0, k, max(11, k // 500)):
        _, c, i = oracle.reusable_space(size, ts, te, a, (int(windows[w][0]), int(windows[w][1])), cap=1)
        assert int(counts[w]) == c and int(idle[w]) == i


def test_config2_best_plan_4096_windows(S, oracle):
    tr = make_trace(2)
    order = make_orderings(tr, CONFIGS[2].n_orderings, rows=[0])[0]
    a, _ = oracle.plan_allpairs(tr.size, tr.t_alloc, tr.t_free, order)
    windows = make_windows(tr, 4096, seed=7002)
    _compare(S, oracle, tr.size, tr.t_alloc, tr.t_free, tr.t_end, a, windows, cap=64)


def test_more_window_groups_than_waves(S, oracle):
    """300 000 windows over a short plan: every wave answers several (group of 64 windows, part) units in
    a row; one malformed window in the middle is reported."""
    rng = np.random.default_rng(4300)
    n, k = 131, 300000
    size, ts, te, t_end = random_trace(rng, n, t_max=200, unique_times=False)
    a = rng.integers(0, 4 * n, n).astype(np.uint64)
    lo = rng.integers(0, t_end, k)
    hi = np.minimum(lo + rng.integers(1, 60, k), t_end)
    lo = np.minimum(lo, hi - 1)
    windows = np.stack([lo, hi], axis=1).astype(np.uint32)
    _compare(S, oracle, size, ts, te, t_end, a, windows, cap=16, sample=range(0, k, 211))
    windows[200001] = (5, 5)
    status, *_ = _gpu(S, size, ts, te, t_end, a, windows, 16)
    assert status == 7                                                   # STALLOC_ERR_BAD_WINDOW


def test_reports_malformed_inputs(S):
    size, ts, te, a, windows = load_reusable_golden()
    status, *_ = _gpu(S, size, ts, te, int(te.max()), a, np.array([[0, 3], [4, 4]], np.uint32), 4)
    assert status == 7                                                   # STALLOC_ERR_BAD_WINDOW
    bad = size.copy()
    bad[1] = 0
    status, *_ = _gpu(S, bad, ts, te, int(te.max()), a, np.array([[0, 3]], np.uint32), 4)
    assert status == 2                                                   # STALLOC_ERR_BAD_TRACE
    # counts and idle bytes only
    status, ranges, counts, idle = _gpu(S, size, ts, te, int(te.max()), a, np.array([[4, 6]], np.uint32), 0)
    assert status == 0 and ranges is None and int(counts[0]) == 4 and int(idle[0]) == 7
