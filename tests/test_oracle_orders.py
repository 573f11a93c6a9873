"""Pins of the oracle's candidate orders: published outputs of the SplitMix64 generator, the sorting
rules of the three heuristic rows checked on the result, permutations, agreement with the input
generator of workloads/ (an independent implementation in numpy), and the statistics the two random
families are meant to have."""
import numpy as np
import pytest

from helpers import random_trace
from workloads import Trace, make_orderings, make_trace

# outputs of splitmix64.c (Vigna, public domain) seeded with 1234567
SPLITMIX64_1234567 = [6457827717110365317, 3203168211198807973, 9817491932198370423,
                      4593380528125082431, 16408922859458223821]
GOLDEN_GAMMA = 0x9E3779B97F4A7C15


def test_splitmix64_published_outputs(oracle):
    x = 1234567
    for want in SPLITMIX64_1234567:
        assert oracle.splitmix64(x) == want
        x = (x + GOLDEN_GAMMA) & 0xFFFFFFFFFFFFFFFF


@pytest.mark.parametrize("seed", range(6))
def test_rows_are_permutations_and_heuristic_rows_follow_their_rules(oracle, seed):
    rng = np.random.default_rng(8500 + seed)
    n = int(rng.integers(1, 400))
    size, ts, te, _ = random_trace(rng, n, t_max=max(4, n // 3), unique_times=(seed % 2 == 1), sizes=[8, 16, 16, 512, 4096])
    o = oracle.make_orders(size, ts, te, 9, seed=77)
    for row in o:
        assert np.array_equal(np.sort(row), np.arange(n))
    s, a, life = size.astype(np.int64), ts.astype(np.int64), te.astype(np.int64) - ts.astype(np.int64)
    ids = o.astype(np.int64)
    r = ids[0]          # size descending, then allocation time, then number
    assert all((s[x], -a[x], -x) >= (s[y], -a[y], -y) for x, y in zip(r[:-1], r[1:]))
    r = ids[1]          # lifetime descending, then size descending, then number
    assert all((life[x], s[x], -x) >= (life[y], s[y], -y) for x, y in zip(r[:-1], r[1:]))
    r = ids[2]          # allocation time, then number
    assert all((a[x], x) <= (a[y], y) for x, y in zip(r[:-1], r[1:]))
    # any window of rows can be produced on its own
    assert np.array_equal(oracle.make_orders(size, ts, te, 4, seed=77, first_plan=5), o[5:9])
    assert not np.array_equal(oracle.make_orders(size, ts, te, 9, seed=78)[3:], o[3:]) or n < 3


@pytest.mark.parametrize("cfg", [1, 2])
def test_matches_the_input_generator(oracle, cfg):
    tr = make_trace(cfg)
    assert np.array_equal(oracle.make_orders(tr.size, tr.t_alloc, tr.t_free, 40, seed=1000), make_orderings(tr, 40, seed=1000))
    rows = [0, 1, 2, 3, 1000, 1001]
    got = np.concatenate([oracle.make_orders(tr.size, tr.t_alloc, tr.t_free, 1, seed=1000, first_plan=p) for p in rows])
    assert np.array_equal(got, make_orderings(tr, 1024, seed=1000, rows=rows))


def test_random_families_have_the_intended_statistics(oracle):
    rng = np.random.default_rng(8600)
    n = 64
    sizes = np.repeat(np.asarray([4096, 1024, 256, 64], np.uint64), 16)
    size = sizes[rng.permutation(n)]
    ts = np.arange(n, dtype=np.uint32)
    te = ts + np.uint32(5)
    o = oracle.make_orders(size, ts, te, 2003, seed=5)
    odd, even = o[3::2].astype(np.int64), o[4::2].astype(np.int64)
    # uniform permutations: every request is first about equally often (1000 rows, 64 requests: 15.6 +- 4)
    first = np.bincount(odd[:, 0], minlength=n)
    assert first.min() >= 3 and first.max() <= 35
    pos = np.argsort(odd, axis=1)                      # position of every request in every row
    assert abs(pos.mean() - (n - 1) / 2) < 1e-9 and abs(pos[:, 0].mean() - (n - 1) / 2) < 3.0
    # size-descending with jitter: a request is never behind one that is two or more sizes smaller
    cls = np.searchsorted(-np.asarray([4096, 1024, 256, 64], np.int64), -size.astype(np.int64))
    c = cls[even]
    assert (np.maximum.accumulate(c, axis=1) - c <= 1).all()
    # ... but neighbouring sizes do mix, and the order inside a size varies from row to row
    assert (np.diff(c, axis=1) < 0).any(axis=1).mean() > 0.9
    assert len({tuple(r[:8]) for r in even}) > 900
