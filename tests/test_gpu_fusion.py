"""Parity of stalloc_fuse_groups (fusion of two HomoPhase groups, Sec. 5.1) with the CPU oracle, through
the C ABI: order, every address, the three extents and the accept flag of every candidate pair, bit by bit."""
import numpy as np
import pytest

from workloads import Trace, make_trace
from workloads.groups import candidate_pairs, flatten_pairs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    return S


def _fuse(S, tr, members, begin, count1, largest):
    import torch
    size, ta, tf = S.trace_to_device(tr)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).cuda()
    out = S.stalloc_fuse_groups(size, ta, tf, tr.t_end, dev(members), dev(begin), dev(count1), largest)
    torch.cuda.synchronize()
    return {"status": int(out["status"].item()), "order": out["order"].cpu().numpy().view(np.uint32),
            "addr": out["addr"].cpu().numpy().view(np.uint64), "extents": out["extents"].cpu().numpy().view(np.uint64),
            "accepted": out["accepted"].cpu().numpy()}


def _compare(S, oracle, tr, groups, pairs):
    members, begin, count1, largest = flatten_pairs(groups, pairs)
    got = _fuse(S, tr, members, begin, count1, largest)
    assert got["status"] == 0
    n_acc = 0
    for k, (g, h) in enumerate(pairs):
        want = oracle.fuse_groups(tr.size, tr.t_alloc, tr.t_free, groups[g], groups[h])
        lo, hi = int(begin[k]), int(begin[k + 1])
        assert np.array_equal(got["order"][lo:hi], want["order"]), (k, g, h)
        assert np.array_equal(got["addr"][lo:hi], want["a"]), (k, g, h)
        assert np.array_equal(got["extents"][k], want["extent"]), (k, g, h)
        assert bool(got["accepted"][k]) == want["accepted"], (k, g, h)
        n_acc += int(want["accepted"])
    return n_acc


@pytest.mark.parametrize("cfg", [1, 2, 3, 5])
def test_every_candidate_pair_of_a_training_trace(S, oracle, cfg):
    tr = make_trace(cfg)
    groups, pairs = candidate_pairs(tr.p_alloc, tr.p_free)
    assert len(pairs) >= 5
    n_acc = _compare(S, oracle, tr, groups, pairs)
    if cfg in (2, 5):
        assert 0 < n_acc < len(pairs)          # both outcomes of the accept test occur


def _random_trace(rng, n, t_end, sizes):
    ts = rng.integers(0, t_end - 1, n)
    te = np.minimum(ts + rng.integers(1, max(2, t_end // 3), n), t_end)
    return Trace(name="random", size=rng.choice(np.asarray(sizes, dtype=np.uint64), n), t_alloc=ts.astype(np.uint32),
                 t_free=te.astype(np.uint32), t_end=t_end)


@pytest.mark.parametrize("seed", range(6))
def test_random_groups_with_arbitrary_lifetimes(S, oracle, seed):
    """Groups that are no HomoPhase groups at all (lifetimes overlap freely, equal keys abound): the
    kernel's sorts, its pointer walk and the leftovers on top against the oracle's."""
    rng = np.random.default_rng(4200 + seed)
    n = 3000
    tr = _random_trace(rng, n, t_end=int(rng.choice([6, 40, 900])), sizes=[512, 1024, 1536, 4096, 1 << 20, 3 << 30])
    groups, pairs = [], []
    for k in range(40):
        n1, n2 = int(rng.integers(1, 300)), int(rng.integers(1, 300))
        ids = rng.choice(n, n1 + n2, replace=False).astype(np.uint32)
        groups += [ids[:n1], ids[n1:]]
        pairs.append((2 * k, 2 * k + 1))
    _compare(S, oracle, tr, groups, pairs)


def test_single_requests_equal_extents_and_sizes_near_2_to_the_62(S, oracle):
    size = np.asarray([1 << 61, 1 << 61, 512, 512, (1 << 61) - 512, 1024], dtype=np.uint64)
    ts = np.asarray([0, 2, 0, 1, 1, 0], dtype=np.uint32)
    te = np.asarray([2, 4, 1, 3, 4, 4], dtype=np.uint32)
    tr = Trace(name="edge", size=size, t_alloc=ts, t_free=te, t_end=4)
    groups = [np.asarray(g, dtype=np.uint32) for g in ([0], [1], [2], [3], [0, 2], [4, 3], [5], [1, 4])]
    pairs = [(0, 1), (1, 0), (2, 3), (3, 2), (4, 5), (5, 4), (6, 7), (7, 6), (0, 6), (2, 0)]
    _compare(S, oracle, tr, groups, pairs)


def test_a_large_pair_at_the_lds_limit_and_errors(S, oracle):
    import torch
    rng = np.random.default_rng(77)
    n = 6000
    tr = _random_trace(rng, n, t_end=64, sizes=[512, 2048, 65536])
    ids = rng.permutation(n).astype(np.uint32)
    groups = [ids[:2500], ids[2500:4900]]
    _compare(S, oracle, tr, groups, [(0, 1), (1, 0)])
    # beyond the LDS limit: refused on the host
    members, begin, count1, largest = flatten_pairs([ids[:3000], ids[3000:]], [(0, 1)])
    with pytest.raises(S.StallocError) as err:
        _fuse(S, tr, members, begin, count1, largest)
    assert err.value.code == 9
    # a pair larger than announced, an empty group, a request number >= n: reported by the device
    members, begin, count1, largest = flatten_pairs(groups, [(0, 1)])
    assert _fuse(S, tr, members, begin, count1, 100)["status"] == 9
    assert _fuse(S, tr, members, begin, np.asarray([0], dtype=np.uint32), largest)["status"] == 1
    bad = members.copy(); bad[17] = n
    assert _fuse(S, tr, bad, begin, count1, largest)["status"] == 6
    # pairs that reach beyond the member list, or backwards: reported, nothing read or written out there
    assert _fuse(S, tr, members, np.asarray([0, len(members) + 1], dtype=np.uint32), count1, largest)["status"] == 1
    assert _fuse(S, tr, members, np.asarray([4000, 100], dtype=np.uint32), count1, largest)["status"] == 1
