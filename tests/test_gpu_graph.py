"""The calls allocate nothing and work on the caller's stream only, so a sequence of them can be captured
in a graph and replayed: every replay must give what the eager calls give."""
import numpy as np
import pytest

from workloads import make_orderings, make_trace

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_eager():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16274_amd as S
    tr = make_trace(1)
    orders_a = make_orderings(tr, 64)
    orders_b = orders_a[::-1].copy()
    size, ta, tf = S.trace_to_device(tr)
    orders = torch.from_numpy(orders_a.view(np.int32)).cuda()
    P, n = orders.shape
    caches = [{}, {}, {}]
    outs = {"offsets": torch.empty((P, n), dtype=torch.int64, device="cuda"),
            "peaks": torch.empty(P, dtype=torch.int64, device="cuda"),
            "best_offsets": torch.empty(n, dtype=torch.int64, device="cuda"),
            "best_plan": torch.empty(1, dtype=torch.int32, device="cuda"),
            "status": torch.empty(1, dtype=torch.int32, device="cuda")}

    def step():
        plan = S.stalloc_plan(size, ta, tf, tr.t_end, orders, out=outs, workspace_cache=caches[0])
        val = S.stalloc_validate(size, ta, tf, tr.t_end, plan["offsets"], workspace_cache=caches[1])
        lb = S.stalloc_lower_bound(size, ta, tf, tr.t_end, workspace_cache=caches[2])
        return plan, val, lb

    def snapshot(plan, val, lb):
        torch.cuda.synchronize()
        return [plan["offsets"].cpu().numpy().copy(), plan["peaks"].cpu().numpy().copy(), int(plan["best_plan"].item()),
                int(plan["status"].item()), val["conflicts"].cpu().numpy().copy(), int(lb["lower_bound"].item())]

    eager_a = snapshot(*step())                      # also sizes the workspaces and sets kernel attributes
    orders.copy_(torch.from_numpy(orders_b.view(np.int32)))
    eager_b = snapshot(*step())
    assert not np.array_equal(eager_a[1], eager_b[1])

    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        step()                                       # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            captured = step()
    torch.cuda.current_stream().wait_stream(stream)
    torch.cuda.synchronize()

    for which in (orders_a, orders_b, orders_a, orders_b):
        orders.copy_(torch.from_numpy(which.view(np.int32)))
        outs["offsets"].zero_()                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot(*captured)
        want = eager_a if which is orders_a else eager_b
        for g, w in zip(got, want):
            assert np.array_equal(g, w)
