"""Parity of stalloc_memory_layers and stalloc_expand_layers (through the C ABI) with the CPU oracle:
the layer of every request, the number of layers and every layer's size and lifetime, bit for bit."""
import numpy as np
import pytest

from helpers import random_trace
from test_oracle_layers import load_layers_golden
from workloads import CONFIGS, Trace, make_orderings, make_trace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    return S


def _gpu_layers(S, size, ts, te, t_end):
    import torch
    d = lambda x, t: torch.from_numpy(np.ascontiguousarray(x).view(t)).cuda()
    out = S.stalloc_memory_layers(d(size, np.int64), d(ts, np.int32), d(te, np.int32), t_end)
    torch.cuda.synchronize()
    status = int(out["status"].item())
    if status:
        return status, None, None, None, None
    L = int(out["n_layers"].item())
    return (0, out["layer_of"].cpu().numpy().view(np.uint32), out["layer_size"].cpu().numpy().view(np.uint64)[:L],
            out["layer_t_alloc"].cpu().numpy().view(np.uint32)[:L], out["layer_t_free"].cpu().numpy().view(np.uint32)[:L])


def _compare(S, oracle, size, ts, te, t_end):
    status, layer_of, l_size, l_ts, l_te = _gpu_layers(S, size, ts, te, t_end)
    assert status == 0
    w_of, w_size, w_ts, w_te = oracle.memory_layers(size, ts, te)
    assert len(l_size) == len(w_size), "number of layers"
    assert np.array_equal(layer_of, w_of), "layer of a request"
    assert np.array_equal(l_size, w_size) and np.array_equal(l_ts, w_ts) and np.array_equal(l_te, w_te)
    return layer_of, l_size, l_ts, l_te


def test_hand_worked_example(S, oracle):
    size, ts, te, want_of, want_layers = load_layers_golden()
    status, layer_of, l_size, l_ts, l_te = _gpu_layers(S, size, ts, te, int(te.max()))
    assert status == 0 and np.array_equal(layer_of, want_of)
    assert np.array_equal(np.stack([l_size.astype(np.int64), l_ts, l_te], axis=1), want_layers)


@pytest.mark.parametrize("seed", range(12))
def test_random_traces(S, oracle, seed):
    """Counts around wave, tile and chunk sizes; a handful of sizes (long groups) or all sizes distinct
    (as many groups as requests); tied and unique times; sizes up to 2^40."""
    rng = np.random.default_rng(9100 + seed)
    n = [1, 2, 63, 64, 65, 255, 257, 1023, 1025, 3000, 7000, 20000][seed]
    sizes = [[8, 16, 24], None, [512], list(range(1, 40))][seed % 4]
    size, ts, te, t_end = random_trace(rng, n, t_max=max(4, n // (2 + seed % 3)), unique_times=(seed % 2 == 1), sizes=sizes)
    if seed % 4 == 1:
        size = (rng.permutation(n).astype(np.uint64) + np.uint64(1)) << np.uint64(20 * (seed % 3))   # all distinct
    _compare(S, oracle, size, ts, te, t_end)


@pytest.mark.parametrize("n0", [700, 1300])
def test_group_with_more_layers_than_registers_hold(S, oracle, n0):
    """700 or 1300 requests of one size alive together, then waves of requests that take over released
    layers: up to 1024 layers of a group sit in registers (eleven of them for 700), the layers past the
    1024th are kept in memory."""
    rng = np.random.default_rng(9200)
    n1 = 1500
    ts0 = rng.integers(0, 50, n0)
    te0 = 100 + rng.integers(0, 400, n0)
    ts1 = rng.integers(100, 900, n1)
    te1 = ts1 + rng.integers(1, 300, n1)
    ts = np.concatenate([ts0, ts1]).astype(np.uint32)
    te = np.concatenate([te0, te1]).astype(np.uint32)
    size = np.full(n0 + n1, 4096, np.uint64)
    size[rng.integers(0, n0 + n1, 40)] = 64            # a second, small group beside it
    layer_of, l_size, _, _ = _compare(S, oracle, size, ts, te, int(te.max()))
    assert int((l_size == 4096).sum()) > (512 if n0 == 700 else 1024)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5, 6])
def test_configs(S, oracle, cfg):
    tr = make_trace(cfg)
    _compare(S, oracle, tr.size, tr.t_alloc, tr.t_free, tr.t_end)


@pytest.mark.parametrize("cfg", [1, 2, 6])
def test_layers_planned_and_expanded(S, oracle, cfg):
    """The layers of a configuration planned by stalloc_plan under several orders, expanded back to the
    requests: addresses equal the oracle's (layer plan by the oracle, gathered), no plan has a conflict,
    extents are those of the layer plans and not below the lower bound."""
    import torch
    tr = make_trace(cfg)
    layer_of, l_size, l_ts, l_te = _compare(S, oracle, tr.size, tr.t_alloc, tr.t_free, tr.t_end)
    ltr = Trace(name="layers", size=l_size, t_alloc=l_ts, t_free=l_te, t_end=tr.t_end)
    orders = make_orderings(ltr, 8)
    d = lambda x, t: torch.from_numpy(np.ascontiguousarray(x).view(t)).cuda()
    plan = S.stalloc_plan(d(l_size, np.int64), d(l_ts, np.int32), d(l_te, np.int32), tr.t_end, d(orders, np.int32))
    out = S.stalloc_expand_layers(d(layer_of, np.int32), plan["offsets"])
    torch.cuda.synchronize()
    assert int(plan["status"].item()) == 0 and int(out["status"].item()) == 0
    got = out["offsets"].cpu().numpy().view(np.uint64)
    a_layers, ext = oracle.plan_many(l_size, l_ts, l_te, orders, threads=4, method="allpairs")
    assert np.array_equal(got, a_layers[:, layer_of])
    assert np.array_equal((got + tr.size[None, :]).max(axis=1), ext)
    size, ta, tf = S.trace_to_device(tr)
    val = S.stalloc_validate(size, ta, tf, tr.t_end, out["offsets"])
    torch.cuda.synchronize()
    assert int(val["status"].item()) == 0 and not val["conflicts"].cpu().numpy().any()
    lb, _ = oracle.lower_bound(tr.size, tr.t_alloc, tr.t_free, tr.t_end)
    assert int(ext.min()) >= lb


def test_reports_malformed_inputs(S):
    import torch
    size, ts, te, want_of, _ = load_layers_golden()
    bad = size.copy()
    bad[3] = 0
    status, *_ = _gpu_layers(S, bad, ts, te, int(te.max()))
    assert status == 2                                                   # STALLOC_ERR_BAD_TRACE
    d = lambda x, t: torch.from_numpy(np.ascontiguousarray(x).view(t)).cuda()
    offs = d(np.arange(8, dtype=np.uint64).reshape(2, 4) * np.uint64(64), np.int64)
    out = S.stalloc_expand_layers(d(want_of, np.int32), offs)
    torch.cuda.synchronize()
    assert int(out["status"].item()) == 0
    assert np.array_equal(out["offsets"].cpu().numpy()[1], (4 + want_of.astype(np.int64)) * 64)
    wrong = want_of.copy()
    wrong[5] = 4                                                         # there are four layers
    out = S.stalloc_expand_layers(d(wrong, np.int32), offs)
    torch.cuda.synchronize()
    assert int(out["status"].item()) == 8                                # STALLOC_ERR_BAD_LAYER
